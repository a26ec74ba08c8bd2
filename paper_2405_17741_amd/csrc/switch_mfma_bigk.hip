// liblsw device code (gfx950): the fused adapter switch on the matrix cores for fused ranks 72..256.
#include "lsw_device.h"
#include "lsw_mfma.h"

namespace lsw {

// ---------------------------------------------------------------------------
// Fused switch on the matrix cores for large fused ranks (64 < K = terms * r <= 256).
//
// Same launch shape, tile mapping, operand split and W addressing as k_switch_mfma.  What differs:
// the Q operand of one 256-column step no longer fits LDS (K * 256 columns * 4 bytes = 256 KB at
// K = 256), so the fused rank is cut into chunks of 4 k-steps (64 ranks, 64 KB of Q) that are
// double-buffered in LDS, and the fp32 accumulators of the whole 32 x 256 tile stay in registers
// across the chunks of a step.  P (coeff * B, split) for the whole fused rank stays in registers for
// the item.
//
// Schedule of one step (per wave).  Chunk 0: request the copy of chunk 1's Q quarter, store the
// previous step's tile, request the next tile into the registers just stored from; then compute,
// widening the W words of block pair q+1 into their accumulators while the matrix pipe works on
// pair q.  Chunks 1..: two LDS-copy instructions of the following chunk's Q ride along with each of
// the first 8 of the 16 groups of matrix instructions; in the last chunk the finished accumulators of pair q-1 are
// rounded to bf16 while pair q computes.  Every chunk ends with "my LDS copies have landed" + a
// workgroup barrier.  The vector-memory counter is in order, so the wait after chunk 0 lets the 32
// younger W requests fly on (they get two chunks to complete); the waits after the other chunks
// drain everything.  At K = 256 the three-pass product needs longer on the matrix cores than the W
// traffic needs on HBM: this kernel is bound by the matrix cores.
// ---------------------------------------------------------------------------
constexpr int BK_KC = 4;                       // k-steps per LDS chunk
constexpr int BK_MAX_GROUPS = 32;              // 8-rank groups of the fused rank: K <= 256
template <int QP>
constexpr int kBkBufBytes = BK_KC * 8 * QP * 64 * 16;    // one LDS buffer: 64 KB (32 KB when Q has no low part)

// 16-byte-per-lane LDS copy, source = scalar base + 32-bit lane offset + immediate (see lds_dma16);
// lane l lands at lds_addr + 16*l.  The hardware adds the instruction's immediate to the LDS address as
// well as to the memory address (measured), so it is taken off the LDS base here.
template <int IMM>
__device__ __forceinline__ void lds_dma16_s(uint32_t voff, const void* sbase, uint32_t lds_addr) {
  static_assert(IMM >= 0 && IMM < 4096, "13-bit signed immediate");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:%3" ::"v"(voff), "s"(sbase),
               "s"(lds_addr - uint32_t(IMM)), "n"(IMM)
               : "memory", "m0");
}

// What one wave needs to copy its quarter of a Q chunk: instruction d = (2*kk + j)*QP + hl moves block
// 2*wave + j, part hl, of k-step kk.
struct BkCopy {
  const void* sbase;          // packed A of the linear + column block + this wave's two blocks (uniform)
  uint32_t lds_base;          // LDS byte address of the target buffer + this wave's two blocks (uniform)
  uint32_t voff[BK_KC];       // per lane: start of the (expert, rank group) of this lane's half of k-step kk, + 16 * n
};

template <int D, int QP>
__device__ __forceinline__ void bk_copy_one(const BkCopy& c) {
  constexpr int kk = D / (2 * QP), j = (D / QP) & 1, hl = D % QP;
  lds_dma16_s<(QP * j + hl) * 512>(c.voff[kk], c.sbase, c.lds_base + uint32_t((kk * 16 + j * 2) * QP * 512 + hl * 1024));
}

template <int D0, int D1, int QP>
__device__ __forceinline__ void bk_copy_range(const BkCopy& c) {
  if constexpr (D0 < D1) {
    bk_copy_one<D0, QP>(c);
    bk_copy_range<D0 + 1, D1, QP>(c);
  }
}

template <typename F, int... I>
__device__ __forceinline__ void bk_for_each_group(F& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}

// One chunk: acc += P[chunk] * Q[chunk] for the 8 blocks of the step, three passes, in 16 groups of six
// matrix instructions (pair q outermost, k-step kk inside).  FIRST: widen the W words of pair q+1
// during pair q (pair 0 is widened by the caller).  LAST: round pair q-1 during pair q (pair 3 by the
// caller).  COPY: issue the 16 LDS-copy instructions of `cp` along with the first 8 groups.
//
// H (exact factors, one pass): with bf16-stored factors and a rank that is a multiple of 16 every k-step belongs to ONE
// term, and B and A are exact matrix-core operands.  The accumulators then start at zero and collect the bare products
// B_c A_c; the gate enters in fp32 BETWEEN the terms (Horner: before the first k-step of term c the accumulators are
// multiplied by rho = coeff_{c-1} / coeff_c, terms sorted by rising |coeff| so that |rho| <= 1) and W joins at the very end,
// W + coeff_last * acc, rounded once.  One matrix instruction per block and k-step instead of two, no low part of P.
template <bool FIRST, bool LAST, bool COPY, int QP, bool H>
__device__ __forceinline__ void bk_chunk(const u32x4* p_hi, const u32x4* p_lo /* the chunk's BK_KC entries */,
                                         const u32x4* qbuf /* LDS: slot 0 of the chunk's buffer + lane */,
                                         f32x16 (&a0)[4], f32x16 (&a1)[4], u32x4 (&wcur)[16], const BkCopy& cp,
                                         const float* rho /* H: the chunk's BK_KC Horner factors (uniform) */, float coeff_last) {
  u32x4 qr[2][2][QP];          // [parity][block of the pair][high, low]
  auto fetch = [&](int idx) {
    const int q = idx / BK_KC, kk = idx % BK_KC;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int hl = 0; hl < QP; ++hl) qr[idx & 1][j][hl] = qbuf[((kk * 8 + 2 * q + j) * QP + hl) * 64];
  };
  fetch(0);
  __builtin_amdgcn_sched_barrier(0);
  auto group = [&](auto IDX) {
    constexpr int idx = decltype(IDX)::value;
    constexpr int q = idx / BK_KC, kk = idx % BK_KC;
    if (idx + 1 < 4 * BK_KC) fetch(idx + 1);
    if constexpr (COPY && idx < 8) {          // the 8 * QP copies in the first half: the last one has half a chunk to land
      bk_copy_range<QP * idx, QP * idx + QP, QP>(cp);
    }
    constexpr int kRowsPer = 16 / BK_KC;
#pragma unroll
    for (int v = kk * kRowsPer; v < (kk + 1) * kRowsPer; ++v) {
      if constexpr (FIRST && q + 1 < 4) {
        a0[q + 1][v] = H ? 0.0f : bf16_lo(wcur[v][q + 1]);
        a1[q + 1][v] = H ? 0.0f : bf16_hi(wcur[v][q + 1]);
      }
      if constexpr (LAST && q > 0) {
        uint32_t w = H ? pack_bf16(fmaf(coeff_last, a0[q - 1][v], bf16_lo(wcur[v][q - 1])),
                                   fmaf(coeff_last, a1[q - 1][v], bf16_hi(wcur[v][q - 1])))
                       : pack_bf16(a0[q - 1][v], a1[q - 1][v]);   // the one rounding
        asm volatile("" : "+v"(w));
        wcur[v][q - 1] = w;
      }
    }
    if constexpr (H) {
      if (rho[kk] != 1.0f) {          // a new term starts with this k-step (uniform)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          a0[q][v] *= rho[kk];
          a1[q][v] *= rho[kk];
        }
      }
    }
    const bf16x8 ph = __builtin_bit_cast(bf16x8, p_hi[kk]);
    const bf16x8 pl = __builtin_bit_cast(bf16x8, p_lo[kk]);
    const bf16x8 h0 = __builtin_bit_cast(bf16x8, qr[idx & 1][0][0]);
    const bf16x8 h1 = __builtin_bit_cast(bf16x8, qr[idx & 1][1][0]);
    if constexpr (!H) {
      a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl, h0, a0[q], 0, 0, 0);
      a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl, h1, a1[q], 0, 0, 0);
    }
    if constexpr (QP == 2) {
      const bf16x8 l0 = __builtin_bit_cast(bf16x8, qr[idx & 1][0][QP - 1]);
      const bf16x8 l1 = __builtin_bit_cast(bf16x8, qr[idx & 1][1][QP - 1]);
      a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, l0, a0[q], 0, 0, 0);
      a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, l1, a1[q], 0, 0, 0);
    }
    a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, h0, a0[q], 0, 0, 0);
    a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, h1, a1[q], 0, 0, 0);
    if constexpr (!H) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * QP, 0);     // the next group's LDS reads first
#pragma unroll
      for (int i = 0; i < 2 + 2 * QP; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one matrix instruction
        __builtin_amdgcn_sched_group_barrier(0x002, (FIRST || LAST) ? 2 : 0, 0);   // a few vector instructions
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  bk_for_each_group(group, std::make_integer_sequence<int, 4 * BK_KC>{});
}

// the wave's LDS copies (and everything older) have landed; up to NEWER younger requests may still fly
template <int NEWER>
__device__ __forceinline__ void bk_drain_and_barrier() {
  static_assert(NEWER == 0 || NEWER == 32, "encoded below");
  // No fence builtins here: a workgroup-scope release would make the compiler wait for EVERY outstanding
  // vector-memory request, the younger W loads and stores included.  The LDS copies count in the wave's
  // vector-memory counter in issue order, so waiting until only NEWER requests remain proves they have
  // landed; LDS itself needs no cache maintenance.  The empty asm statements keep the compiler from moving
  // LDS reads across the barrier.
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(NEWER == 0 ? 0x0F70 : 0x8F70);      // vmcnt(0) or vmcnt(32); expcnt, lgkmcnt untouched
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

template <int NCH>
struct BkWave {             // per-wave state of the chunked kernel that outlives a step
  u32x4 p_hi[BK_KC * NCH], p_lo[BK_KC * NCH];
  int32_t eg[2][BK_KC * NCH];       // expert * (r/8) + rank group of lane half h, k-step ks (uniform: scalar registers)
  float rho[BK_KC * NCH];           // exact-factor mode: Horner factor applied before k-step ks (1 = none), uniform
  float coeff_last;                 // exact-factor mode: coefficient of the last term, applied with W at the end
  int32_t eg_bytes;                 // bytes of one (expert, rank group) slab of the linear's packed A: column blocks * 4 KB * Q parts (uniform)
  const uint16_t* Apk;
  const uint16_t* W;
  const uint16_t* Wsrc;             // where tiles are read from: W, or the base copy when re-basing
  int wbytes;
  uint32_t stride;
  uint32_t lds0;                    // LDS byte address of buffer 0 + this wave's two blocks
  int n, h;
};

template <int NCH, int QP>
__device__ __forceinline__ BkCopy bk_copy_desc(const BkWave<NCH>& w, int cs, int ch, int buf) {
  BkCopy c;
  c.sbase = uniform(reinterpret_cast<const char*>(w.Apk) + (long long)(cs / MT_STEP) * (4096 * QP));
  c.lds_base = w.lds0 + uint32_t(buf) * kBkBufBytes<QP>;
#pragma unroll
  for (int kk = 0; kk < BK_KC; ++kk)
    c.voff[kk] = uint32_t(w.h ? w.eg[1][ch * BK_KC + kk] * w.eg_bytes : w.eg[0][ch * BK_KC + kk] * w.eg_bytes) + uint32_t(16 * w.n);
  return c;
}

// One 32 x 256 step of a wave.  wcur holds the tile to update (loaded one step ago); wprev holds the finished
// tile of the previous step: it is stored, then reloaded with the tile of the next step.
template <int NCH, int QP, bool H>
__device__ __forceinline__ void bk_step(const BkWave<NCH>& w, int cs, bool more, int lane, int& buf, uint32_t prev_off,
                                        uint32_t next_off, u32x4 (&wcur)[16], u32x4 (&wprev)[16]) {
  const __amdgpu_buffer_rsrc_t res = w_resource(w.W, w.wbytes);
  const __amdgpu_buffer_rsrc_t res_src = w_resource(w.Wsrc, w.wbytes);
  f32x16 a0[4], a1[4];
  {
    const BkCopy cp = bk_copy_desc<NCH, QP>(w, cs, 1 % NCH, buf ^ 1);
    bk_copy_range<0, 8 * QP, QP>(cp);
    __builtin_amdgcn_sched_barrier(0);                    // keep the W requests younger than the Q copy
#pragma unroll
    for (int v = 0; v < 16; ++v)
      __builtin_amdgcn_raw_buffer_store_b128(wprev[v], res, prev_off + uint32_t(8 * (v >> 2) + (v & 3)) * w.stride, 0, kWStoreAux);
    asm volatile("" : "+v"(next_off) : "v"(prev_off));      // keep the loads after the stores that free their registers
#pragma unroll
    for (int v = 0; v < 16; ++v)
      wprev[v] = __builtin_amdgcn_raw_buffer_load_b128(res_src, next_off + uint32_t(8 * (v >> 2) + (v & 3)) * w.stride, 0, kWLoadAux);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      a0[0][v] = H ? 0.0f : bf16_lo(wcur[v][0]);
      a1[0][v] = H ? 0.0f : bf16_hi(wcur[v][0]);
    }
    bk_chunk<true, false, false, QP, H>(w.p_hi, w.p_lo, wg_lds + buf * (kBkBufBytes<QP> / 16) + lane, a0, a1, wcur, cp, w.rho, w.coeff_last);
    bk_drain_and_barrier<32>();
    buf ^= 1;
  }
#pragma unroll
  for (int ch = 1; ch < NCH; ++ch) {
    // the following chunk's Q (after the last chunk: chunk 0 of the next step; after the last step a harmless re-read)
    const BkCopy cp = bk_copy_desc<NCH, QP>(w, (ch + 1 < NCH || !more) ? cs : cs + MT_STEP, (ch + 1) % NCH, buf ^ 1);
    if (ch + 1 < NCH) {
      bk_chunk<false, false, true, QP, H>(w.p_hi + ch * BK_KC, w.p_lo + ch * BK_KC, wg_lds + buf * (kBkBufBytes<QP> / 16) + lane, a0, a1, wcur, cp,
                                          w.rho + ch * BK_KC, w.coeff_last);
    } else {
      bk_chunk<false, true, true, QP, H>(w.p_hi + ch * BK_KC, w.p_lo + ch * BK_KC, wg_lds + buf * (kBkBufBytes<QP> / 16) + lane, a0, a1, wcur, cp,
                                         w.rho + ch * BK_KC, w.coeff_last);
#pragma unroll
      for (int v = 0; v < 16; ++v)
        wcur[v][3] = H ? pack_bf16(fmaf(w.coeff_last, a0[3][v], bf16_lo(wcur[v][3])), fmaf(w.coeff_last, a1[3][v], bf16_hi(wcur[v][3])))
                       : pack_bf16(a0[3][v], a1[3][v]);
    }
    bk_drain_and_barrier<0>();
    buf ^= 1;
  }
}

template <int NCH, int QP, bool H>
__global__ __launch_bounds__(256) void k_switch_mfma_bigk(LaunchPlan p, Terms t, const Terms* t_dev, int r) {
  constexpr int NKS = BK_KC * NCH;
  static_assert(NCH >= 2 && 2 * NKS <= BK_MAX_GROUPS, "chunks per step");
  static_assert(!H || QP == 1, "the one-pass mode needs exact (bf16-stored) factors");
  __shared__ float s_rho[BK_KC * 4];
  __shared__ int32_t s_te[kMaxTerms];
  __shared__ float s_tc[kMaxTerms];
  __shared__ int32_t s_e[BK_MAX_GROUPS], s_g[BK_MAX_GROUPS], s_eg[BK_MAX_GROUPS];
  __shared__ float s_c[BK_MAX_GROUPS];
  const int lane = threadIdx.x & 63;
  const int wave = uniform(int(threadIdx.x >> 6));
  const int n = lane & 31, h = lane >> 5;
  const int gpr = r >> 3;
  int n_terms;
  LSW_LOAD_TERMS(t, t_dev, s_te, s_tc, n_terms);
  if (n_terms == 0) return;             // nothing to merge or unmerge (device-built lists only): W stays untouched
  const int n_groups = n_terms * gpr;
  __syncthreads();
  if constexpr (H) {
    // terms by rising |coeff| (the sum does not depend on their order), then the Horner factor of every k-step
    if (threadIdx.x == 0) {
      for (int a = 1; a < n_terms; ++a)
        for (int b = a; b > 0 && fabsf(s_tc[b]) < fabsf(s_tc[b - 1]); --b) {
          const float tc = s_tc[b]; s_tc[b] = s_tc[b - 1]; s_tc[b - 1] = tc;
          const int32_t te = s_te[b]; s_te[b] = s_te[b - 1]; s_te[b - 1] = te;
        }
      const int kpt = r >> 4;                  // k-steps per term
      for (int ks = 0; ks < NKS; ++ks) {
        const int c = ks / kpt;
        s_rho[ks] = (ks > 0 && ks % kpt == 0 && c < n_terms) ? s_tc[c - 1] / s_tc[c] : 1.0f;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x < BK_MAX_GROUPS) {           // group G of the fused rank: (expert, 8-rank group, coefficient); padding gets 0
    const int G = threadIdx.x;
    const bool valid = G < n_groups;
    const int c = valid ? G / gpr : 0;
    const int g = valid ? G - c * gpr : 0;
    const int e = p.Z ? c : s_te[c];          // adapter-path mode: all experts in order, coefficient 1
    s_e[G] = e;
    s_g[G] = g;
    s_eg[G] = e * gpr + g;
    s_c[G] = valid ? (p.Z ? 1.0f : s_tc[c]) : 0.0f;
  }
  __syncthreads();

  BkWave<NCH> w;
  w.n = n;
  w.h = h;
  w.lds0 = uniform(int(uint32_t(uintptr_t((const __attribute__((address_space(3))) void*)wg_lds)))) + uint32_t(wave) * (2048u * QP);
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    w.eg[0][ks] = uniform(s_eg[2 * ks]);
    w.eg[1][ks] = uniform(s_eg[2 * ks + 1]);
    w.rho[ks] = H ? __builtin_bit_cast(float, uniform(__builtin_bit_cast(int, s_rho[ks]))) : 1.0f;
  }
  w.coeff_last = H ? __builtin_bit_cast(float, uniform(__builtin_bit_cast(int, s_tc[n_terms - 1]))) : 1.0f;

  const int grid = gridDim.x;
  // Items of a fixed width, workgroup b taking b', b' + grid, ...; or (LaunchPlan::flat, adapter mode) the numbering is in single
  // column steps and the workgroup works off ONE contiguous range of it, every item running to the end of its row of steps
  // or of the range
  int first_item = p.xcd_remap ? xcd_contiguous_block(blockIdx.x, grid) : int(blockIdx.x);
  int item_end = p.n_items, advance = grid;
  if (p.flat) flat_range(p.n_items, grid, int(blockIdx.x), &first_item, &item_end);
  int buf = 0;
  for (int item = first_item; item < item_end; item += advance) {       // uniform over the workgroup
    const bool adapter = p.Z != nullptr;
    LinDesc L;
    int local = item;
    if (adapter) {
      const int seg = uniform(find_segment(p.ad_first, p.n_sel, item));
      L.W = uniform(p.ad[seg].W);
      L.B = uniform(p.ad[seg].B);            // this linear's Z
      L.Apk = uniform(p.ad[seg].Apk);
      L.Wbase = nullptr;
      L.out = uniform(p.ad[seg].out);
      L.in = uniform(p.ad[seg].in);
      L.ld = uniform(p.ad[seg].ld);
      local = uniform(item - p.ad_first[seg]);
    } else {
      const int seg = uniform(find_segment(p.first, p.n_sel, item));
      const LinDesc* Lp = p.lin + uniform(p.sel[seg]);
      L.W = uniform(Lp->W);
      L.B = uniform(Lp->B);
      L.Apk = uniform(Lp->Apk);
      L.Wbase = p.from_base ? uniform(Lp->Wbase) : nullptr;
      L.out = uniform(Lp->out);
      L.in = uniform(Lp->in);
      L.ld = uniform(Lp->ld);
      local = uniform(item - p.first[seg]);
    }
    const void* B = L.B;
    const int out = L.out, in = L.in;
    int row0, col0;
    decode_item(local, out, in, kMfmaTileRows, p.tile_cols, 0, &row0, &col0);
    row0 += 32 * wave;
    int col_end = min(in, col0 + p.tile_cols);
    if (p.flat) {
      advance = flat_item_units(in, col0, item, item_end);
      col_end = min(in, col0 + MT_STEP * advance);
    }
    const int ncb = ceil_div(in, MT_STEP);
    w.W = L.W;
    w.Wsrc = p.from_base ? L.Wbase : w.W;
    w.wbytes = w_extent_bytes(out, in, L.ld);
    w.stride = uint32_t(L.ld) * 2u;
    // the packed A of the linear, advanced to this wave's two blocks inside a column block
    w.Apk = uniform(reinterpret_cast<const uint16_t*>(reinterpret_cast<const char*>(L.Apk) + wave * (1024 * QP)));
    w.eg_bytes = ncb * (4096 * QP);
    const uint32_t row0_byte = uint32_t(row0) * w.stride;

    // P = coeff * B for this lane's row and its half of every k-step, split into bf16 high + low
    {
      const int prow = min(row0 + n, out - 1);
      const bool prow_ok = row0 + n < out;       // rows past the end: zero coefficient (their W offsets lie outside the buffer)
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const int G = 2 * ks + h;
        if constexpr (H) {       // B as stored: an exact operand; rows past the end and padding groups contribute zeros
          const u32x4 raw = *(const LSW_GLOBAL u32x4*)(reinterpret_cast<const uint16_t*>(B) + ((long long)s_e[G] * out + prow) * r + 8 * s_g[G]);
          const bool on = prow_ok && s_c[G] != 0.0f;
          w.p_hi[ks] = on ? raw : u32x4{0u, 0u, 0u, 0u};
          w.p_lo[ks] = u32x4{0u, 0u, 0u, 0u};
        } else {
          float b[8];
          if (adapter) load8<2>(B, (long long)prow * p.z_stride + 8 * s_eg[G], b);
          else load8<QP>(B, ((long long)s_e[G] * out + prow) * r + 8 * s_g[G], b);
          const float c = prow_ok ? s_c[G] : 0.0f;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            uint32_t hi, lo;
            split2(c * b[2 * q], c * b[2 * q + 1], &hi, &lo);
            w.p_hi[ks][q] = hi;
            w.p_lo[ks][q] = lo;
          }
        }
      }
    }

    auto lane_offset = [&](int cs) {
      const int col = cs + 8 * n;
      return col < col_end ? row0_byte + uint32_t(4 * h) * w.stride + uint32_t(col) * 2u : kOutOfRange;
    };
    // prologue of the item: its first tile and the first Q chunk
    u32x4 wa[16], wb[16];
    uint32_t off_a = lane_offset(col0), off_b = kOutOfRange;
    {
      const __amdgpu_buffer_rsrc_t res = w_resource(w.Wsrc, w.wbytes);
      const BkCopy cp = bk_copy_desc<NCH, QP>(w, col0, 0, buf);
      bk_copy_range<0, 8 * QP, QP>(cp);
#pragma unroll
      for (int v = 0; v < 16; ++v)
        wa[v] = __builtin_amdgcn_raw_buffer_load_b128(res, off_a + uint32_t(8 * (v >> 2) + (v & 3)) * w.stride, 0, kWLoadAux);
#pragma unroll
      for (int v = 0; v < 16; ++v) wb[v] = u32x4{0u, 0u, 0u, 0u};
      bk_drain_and_barrier<0>();
    }
    // steps alternate the roles of wa and wb; the offsets travel with the registers
    int cs = col0;
    bool last_in_a = true;
    while (true) {
      bool more = uniform(int(cs + MT_STEP < col_end)) != 0;
      {
        const uint32_t nxt = more ? lane_offset(cs + MT_STEP) : kOutOfRange;
        bk_step<NCH, QP, H>(w, cs, more, lane, buf, off_b, nxt, wa, wb);     // stores wb (previous tile), reloads it, updates wa
        off_b = nxt;
      }
      last_in_a = true;
      if (!more) break;
      cs += MT_STEP;
      more = uniform(int(cs + MT_STEP < col_end)) != 0;
      {
        const uint32_t nxt = more ? lane_offset(cs + MT_STEP) : kOutOfRange;
        bk_step<NCH, QP, H>(w, cs, more, lane, buf, off_a, nxt, wb, wa);
        off_a = nxt;
      }
      last_in_a = false;
      if (!more) break;
      cs += MT_STEP;
    }
    {   // the item's last finished tile
      const __amdgpu_buffer_rsrc_t res = w_resource(w.W, w.wbytes);
      const uint32_t cs_off = lane_offset(cs);
      if (last_in_a) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          __builtin_amdgcn_raw_buffer_store_b128(wa[v], res, cs_off + uint32_t(8 * (v >> 2) + (v & 3)) * w.stride, 0, kWStoreAux);
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          __builtin_amdgcn_raw_buffer_store_b128(wb[v], res, cs_off + uint32_t(8 * (v >> 2) + (v & 3)) * w.stride, 0, kWStoreAux);
      }
    }
  }
}

template <int NCH, int QP, bool H>
static hipError_t launch_bigk(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int grid, hipStream_t s) {
  const size_t lds = size_t(2) * kBkBufBytes<QP>;     // 2 x 64 KB (2 x 32 KB for bf16 factors)
  // once per process (function-local statics are initialised exactly once, also under concurrent first calls)
  static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_switch_mfma_bigk<NCH, QP, H>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
  if (lds_ok != hipSuccess) return lds_ok;
  hipLaunchKernelGGL((k_switch_mfma_bigk<NCH, QP, H>), dim3(grid), dim3(256), lds, s, p, t, t_dev, r);
  return hipGetLastError();
}

template <int QP, bool H>
static hipError_t launch_bigk_qp(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int grid, hipStream_t s) {
  const int n_groups = t.n * (r / 8);
  switch ((n_groups + 2 * BK_KC - 1) / (2 * BK_KC)) {
    case 2: return launch_bigk<2, QP, H>(p, t, t_dev, r, grid, s);
    case 3: return launch_bigk<3, QP, H>(p, t, t_dev, r, grid, s);
    case 4: return launch_bigk<4, QP, H>(p, t, t_dev, r, grid, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_switch_mfma_bigk(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int qp, int grid, hipStream_t s) {
  if (qp == 2) return launch_bigk_qp<2, false>(p, t, t_dev, r, grid, s);
  // exact factors: one pass when every k-step of 16 ranks belongs to one term (not in adapter mode: Z is fp32)
  if (r % 16 == 0 && p.Z == nullptr && p.exact_one_pass) return launch_bigk_qp<1, true>(p, t, t_dev, r, grid, s);
  return launch_bigk_qp<1, false>(p, t, t_dev, r, grid, s);
}

}  // namespace lsw
