// What the matrix-core switch kernels share: tile constants, the W buffer resource, the per-item state of a wave, the
// tile update on the matrix cores, the copy of the shared operand into LDS, and the order in which workgroups take items.
// The tile mapping, operand split and memory schedule are described at the top of switch_mfma.hip.
#pragma once
#include "lsw_device.h"

namespace lsw {
constexpr int MT_STEP = kApkBlockCols;
constexpr int WG_WAVES = 4;
constexpr int WG_ROWS = kMfmaTileRows;
constexpr uint32_t kOutOfRange = 0x80000000u;   // byte offset beyond any W (out*in*2 < 2^31 is checked at create)
// Cache-policy bits of the W accesses (buffer instruction aux operand on gfx950: 1 = sc0, 2 = nt, 16 = sc1): non-temporal
// both ways.  Stores that are also written through at device scope (nt + sc1) make a bare in-place pass 1-3 % faster,
// but the switch kernels 2-3 % slower (measured on the 7B and 13B stacks), so they are not used.
constexpr int kWLoadAux = 2;
constexpr int kWStoreAux = 2;
extern __shared__ u32x4 wg_lds[];               // [2 buffers][NKS][8 blocks][high, low][64 lanes]

__device__ __forceinline__ __amdgpu_buffer_rsrc_t w_resource(const uint16_t* W, int wbytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(uniform(W)), 0, uniform(wbytes), 0x00020000);
}

template <int NKS>
struct MfmaItem {           // what a wave keeps per work item
  const uint16_t* W;        // the buffer resource is rebuilt from these two where it is used, so
  int wbytes;               // that it provably lives in scalar registers
  const uint16_t* Wsrc;     // where the tile is read from: W, or the base copy when re-basing
  const uint16_t* Apk;      // packed A of the linear
  int ncb;                  // its column blocks
  int col0, col_end;
  uint32_t row0_byte;       // byte offset of this wave's first row (uniform)
  uint32_t stride_byte;     // bytes per row (uniform)
  u32x4 p_hi[NKS], p_lo[NKS];
};

template <int NKS, int QP, bool PROBE = false>
__device__ __forceinline__ void mfma_load_item(const LaunchPlan& p, int item, int n, int gpr, int r,
                                               const int (&term_e)[NKS], const int (&term_g)[NKS],
                                               const float (&term_c)[NKS], MfmaItem<NKS>& it,
                                               int tile_rows, int row_shift, int flat_end = 0) {
  const bool adapter = p.Z != nullptr;          // adapter-path mode: one matrix, rows = tokens, row operand = rows of Z
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
  int row0, col0;
  decode_item(local, L.out, L.in, tile_rows, p.tile_cols, p.panel_group, &row0, &col0);
  row0 += row_shift;          // the calling wave's 32 rows inside a taller item (may lie past the last row)
  it.W = L.W;
  it.Wsrc = p.from_base ? L.Wbase : L.W;
  it.wbytes = w_extent_bytes(L.out, L.in, L.ld);
  it.Apk = L.Apk;
  it.ncb = ceil_div(L.in, MT_STEP);
  it.col0 = col0;
  it.col_end = min(L.in, col0 + p.tile_cols);
  // flat numbering (flat_end = end of the workgroup's range): the item takes every unit up to the end of its row of units
  // or of the range, whichever comes first
  if (flat_end > 0) it.col_end = min(L.in, col0 + MT_STEP * flat_item_units(L.in, col0, item, flat_end));
  it.stride_byte = uint32_t(L.ld) * 2u;
  it.row0_byte = uint32_t(row0) * it.stride_byte;
  const int prow = min(row0 + n, L.out - 1);
  const bool prow_ok = row0 + n < L.out;       // rows past the end get a zero coefficient and an offset outside W
  if constexpr (PROBE) return;
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    float b[8];
    if (adapter) load8<2>(L.B, (long long)prow * p.z_stride + 8 * (term_e[ks] * gpr + term_g[ks]), b);
    else load8<QP>(L.B, ((long long)term_e[ks] * L.out + prow) * r + 8 * term_g[ks], b);
    const float c = prow_ok ? term_c[ks] : 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint32_t hi, lo;
      split2(c * b[2 * q], c * b[2 * q + 1], &hi, &lo);
      it.p_hi[ks][q] = hi;
      it.p_lo[ks][q] = lo;
    }
  }
}

// byte offset of this lane's first row (register 0) at column step cs; register v adds
// (8*(v/4) + v%4) rows, which is uniform over the wave
template <int NKS>
__device__ __forceinline__ uint32_t mfma_lane_offset(const MfmaItem<NKS>& it, int cs, int n, int h) {
  const int col = cs + 8 * n;
  const uint32_t off = it.row0_byte + uint32_t(4 * h) * it.stride_byte + uint32_t(col) * 2u;
  return col < it.col_end ? off : kOutOfRange;
}

template <int NKS>
__device__ __forceinline__ void mfma_load_w(const MfmaItem<NKS>& it, uint32_t lane_off, u32x4 (&wbuf)[16]) {
  const __amdgpu_buffer_rsrc_t res = w_resource(it.Wsrc, it.wbytes);
#pragma unroll
  for (int v = 0; v < 16; ++v)
    wbuf[v] = __builtin_amdgcn_raw_buffer_load_b128(
        res, lane_off + uint32_t(8 * (v >> 2) + (v & 3)) * it.stride_byte, 0, kWLoadAux);
}

template <int NKS, int QP>
__device__ __forceinline__ void wg_compute(const u32x4 (&p_hi)[NKS], const u32x4 (&p_lo)[NKS],
                                           const u32x4* qbuf /* LDS: slot 0 of this step's buffer + lane */,
                                           u32x4 (&wcur)[16]) {
  // Pair q = blocks 2q and 2q+1 = low and high bf16 half of word q of each row.  The work is a
  // chain of 4*NKS chunks (pair q, k-step ks), each 6 matrix instructions (4 when the factors are
  // stored as bf16 and Q has no low part) on the pair's two accumulators.  While the matrix pipe runs a chunk, LDS delivers the operands of the next chunk
  // and the vector ALU widens pair q+1 and rounds pair q-1; the scheduling directives pin that
  // interleaving, which the compiler would otherwise undo.
  f32x16 a0[4], a1[4];
  u32x4 qr[2][2][QP];          // [chunk parity][block of the pair][high, low]
  auto fetch = [&](int chunk) {
    const int q = chunk / NKS, ks = chunk % NKS;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int hl = 0; hl < QP; ++hl) qr[chunk & 1][j][hl] = qbuf[((ks * 8 + 2 * q + j) * QP + hl) * 64];
  };
  fetch(0);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    a0[0][v] = bf16_lo(wcur[v][0]);
    a1[0][v] = bf16_hi(wcur[v][0]);
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const int chunk = q * NKS + ks;
      if (chunk + 1 < 4 * NKS) fetch(chunk + 1);
      // vector work spread over the pair's k-steps: widen pair q+1, round pair q-1
      constexpr int kRowsPer = (16 + NKS - 1) / NKS;
#pragma unroll
      for (int v = ks * kRowsPer; v < (ks + 1) * kRowsPer && v < 16; ++v) {
        if (q + 1 < 4) {
          a0[q + 1][v] = bf16_lo(wcur[v][q + 1]);
          a1[q + 1][v] = bf16_hi(wcur[v][q + 1]);
        }
        if (q > 0) {
          uint32_t w = pack_bf16(a0[q - 1][v], a1[q - 1][v]);   // the one rounding
          asm volatile("" : "+v"(w));
          wcur[v][q - 1] = w;
        }
      }
      const bf16x8 ph = __builtin_bit_cast(bf16x8, p_hi[ks]);
      const bf16x8 pl = __builtin_bit_cast(bf16x8, p_lo[ks]);
      const bf16x8 h0 = __builtin_bit_cast(bf16x8, qr[chunk & 1][0][0]);
      const bf16x8 h1 = __builtin_bit_cast(bf16x8, qr[chunk & 1][1][0]);
      a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl, h0, a0[q], 0, 0, 0);
      a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl, h1, a1[q], 0, 0, 0);
      if constexpr (QP == 2) {
        const bf16x8 l0 = __builtin_bit_cast(bf16x8, qr[chunk & 1][0][QP - 1]);
        const bf16x8 l1 = __builtin_bit_cast(bf16x8, qr[chunk & 1][1][QP - 1]);
        a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, l0, a0[q], 0, 0, 0);
        a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, l1, a1[q], 0, 0, 0);
      }
      a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, h0, a0[q], 0, 0, 0);
      a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, h1, a1[q], 0, 0, 0);
      constexpr int kMfma = 2 + 2 * QP;
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * QP, 0);     // the next chunk's LDS reads first
#pragma unroll
      for (int i = 0; i < kMfma; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one matrix instruction
        __builtin_amdgcn_sched_group_barrier(0x002, (3 * kRowsPer + kMfma - 1) / kMfma, 0);   // a few vector instructions
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) wcur[v][3] = pack_bf16(a0[3][v], a1[3][v]);
}

// The probe's stand-in for wg_compute: every bf16 widened, +0.0f, rounded back (finite values unchanged).
__device__ __forceinline__ void wg_probe_compute(u32x4 (&wcur)[16]) {
#pragma unroll
  for (int v = 0; v < 16; ++v)
#pragma unroll
    for (int q = 0; q < 4; ++q) wcur[v][q] = pack_bf16(bf16_lo(wcur[v][q]) + 0.0f, bf16_hi(wcur[v][q]) + 0.0f);
}

// This wave's quarter of the Q operand of column step `cs` (blocks 2w and 2w+1, all k-steps),
// copied from L2 straight into LDS: lane l of a 16-byte LDS-DMA load lands at base + 16*l, which is
// exactly the [slot][lane] layout wg_compute reads.  No registers are involved; the data is
// complete when the wave's vector-memory counter has drained.
template <int NKS, int QP>
__device__ __forceinline__ void wg_fetch_q(const uint16_t* Apk, int ncb, int cs, int n, int gpr, int wave,
                                           const int (&term_e)[NKS], const int (&term_g)[NKS],
                                           u32x4* buf /* LDS: slot 0 of the target buffer */) {
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const u32x4* src = reinterpret_cast<const u32x4*>(
        Apk + (((long long)term_e[ks] * gpr + term_g[ks]) * ncb + cs / MT_STEP) * (8 * QP * 32 * 8)) + n;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int hl = 0; hl < QP; ++hl)
        lds_dma16(src + (QP * (2 * wave + j) + hl) * 32, buf + ((ks * 8 + 2 * wave + j) * QP + hl) * 64);
  }
}

// All of this wave's outstanding global traffic has landed (its LDS-DMA loads in particular), then
// the workgroup meets: after it every wave may read the buffer the others filled.
__device__ __forceinline__ void wg_drain_and_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0); expcnt and lgkmcnt untouched
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  __builtin_amdgcn_sched_barrier(0);
}

// ---------------------------------------------------------------------------
// The order in which the workgroups of a matrix-core launch take the work items.
//
// Global order: workgroup b takes items b', b' + grid, ... (b' = b, or b's place in the XCD-contiguous numbering).
// Per-XCD order: XCD x (workgroups x, x + 8, ...: the hardware deals workgroups round-robin) owns items
// [x * per, (x + 1) * per), its grid / 8 workgroups taking consecutive items per round.  The XCDs do not run these
// kernels equally fast then (on the machines measured every second one needs 2-3 % longer for the same share,
// whichever share it is given), so with a pool counter (LaunchPlan::pool) the last 1 / pool_div of every XCD's range
// is not dealt statically: those items form a pool that a workgroup draws from, one item at a time through an atomic
// counter, once its own column is done.  Wave 0 claims one item ahead (the answer has a whole item's time to arrive)
// and hands the claim to the other waves through LDS at a workgroup barrier.  Nothing waits for another workgroup.
// The last workgroup to finish resets the counters, so every launch finds them at zero.
// ---------------------------------------------------------------------------
struct ItemWalk {             // every field is uniform over the workgroup
  int step;                   // distance of a workgroup's consecutive static items
  int static_end;             // end of the statically dealt items this workgroup draws from
  int per;                    // items per XCD range (the last range may be shorter)
  int n_items;
  int pool_len;               // items every XCD range gives to the pool (its last ones); 0 = no pool
  int32_t* pool;              // [0] claims made so far, [1] workgroups that have finished
  int after;                  // the item after the next one when that is a static one, else -1
  bool after_pool;            // the item after the next one comes from the pool: wave 0 holds the claim for it
  int slot;                   // which of the two LDS words the next claim is handed over in
};

// Wave 0's claims, for the other waves.  Two words used in turn: with one-step items a wave may still be reading the
// claim handed over at the last barrier while wave 0 already writes the next one.
static __shared__ int32_t s_walk_claim[2];

// wave 0, before the barrier that precedes walk_take_claim: hand the answered claim to the workgroup
__device__ __forceinline__ void walk_publish_claim(const ItemWalk& w, int wave, int claim) {
  if (wave == 0) s_walk_claim[w.slot] = __builtin_amdgcn_readfirstlane(claim);
}

// every wave, after that barrier: the claimed item, or -1 when the pool was empty
__device__ __forceinline__ int walk_take_claim(ItemWalk& w) {
  const int item = walk_pool_item(w.n_items, w.per, w.pool_len, uniform(s_walk_claim[w.slot]));
  w.slot ^= 1;
  w.after_pool = false;       // until walk_plan_after says otherwise
  return item;
}

// Sets up the walk and returns the workgroup's first item (none if it is not below static_end: never with a pool).
__device__ __forceinline__ int walk_init(const LaunchPlan& p, bool per_xcd, ItemWalk& w) {
  w.n_items = p.n_items;
  w.pool = p.pool;
  w.pool_len = 0;
  w.after = -1;
  w.after_pool = false;
  w.slot = 0;
  if (!per_xcd) {
    w.step = int(gridDim.x);
    w.per = p.n_items;
    w.static_end = p.n_items;
    return p.xcd_remap ? xcd_contiguous_block(blockIdx.x, gridDim.x) : int(blockIdx.x);
  }
  const WalkShare sh = walk_share(p.n_items, int(gridDim.x), int(blockIdx.x), p.pool != nullptr, p.pool_div);
  w.step = sh.step;
  w.per = sh.per;
  w.pool_len = sh.pool_len;
  w.static_end = sh.static_end;
  return sh.first;
}

// Flat numbering (LaunchPlan::flat): the workgroup takes the units of flat_range.  w.step is the length of the item loaded
// last (mfma_item_units), set by the caller after every load.  Returns the first unit.
__device__ __forceinline__ int walk_init_flat(const LaunchPlan& p, ItemWalk& w) {
  w.n_items = p.n_items;
  w.pool = nullptr;
  w.pool_len = 0;
  w.after = -1;
  w.after_pool = false;
  w.slot = 0;
  w.per = p.n_items;
  w.step = 1;
  int first;
  flat_range(p.n_items, int(gridDim.x), int(blockIdx.x), &first, &w.static_end);
  return first;
}

template <int NKS>
__device__ __forceinline__ int mfma_item_units(const MfmaItem<NKS>& it) { return ceil_div(it.col_end - it.col0, MT_STEP); }

// after `item` has become the next one: where the item after it comes from (wave 0 claims it now if it is a pool item)
__device__ __forceinline__ void walk_plan_after(ItemWalk& w, int item, bool item_from_pool, int wave, int lane, int& claim) {
  w.after = -1;
  w.after_pool = false;
  if (!item_from_pool && item + w.step < w.static_end) {
    w.after = item + w.step;
  } else if (w.pool_len > 0) {
    w.after_pool = true;
    if (wave == 0 && lane == 0) claim = __hip_atomic_fetch_add(w.pool, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// End of the kernel.  Only wave 0 touches the pool counters and its last claim has been answered (an empty pool is how
// it got here), so when the count of finished workgroups is complete nobody will claim again in this launch.
__device__ __forceinline__ void walk_finish(const ItemWalk& w) {
  if (w.pool_len > 0 && threadIdx.x == 0) {
    const int done = __hip_atomic_fetch_add(w.pool + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (done == int(gridDim.x) - 1) {
      __hip_atomic_store(w.pool, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(w.pool + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace lsw
