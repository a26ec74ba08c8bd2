// Device code of liblsw for gfx950 (MI355X): the fused adapter switch in two
// flavours (matrix-core and fp32 vector-ALU), the A re-layout kernel and the
// merged GEMV.  Sec. 3.3-3.4 of LoRA-Switch define what is computed; the tiling,
// data movement and launch shape are this library's own.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "lsw_internal.h"

namespace lsw {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// two fp32 -> two bf16 (round to nearest even, hardware convert), first value in the low half
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// x = hi + lo + O(2^-18 |x|): hi is x rounded to bf16, lo the rounded remainder (exact subtraction)
__device__ __forceinline__ void split2(float x0, float x1, uint32_t* hi, uint32_t* lo) {
  uint32_t h = pack_bf16(x0, x1);
  *hi = h;
  *lo = pack_bf16(x0 - bf16_lo(h), x1 - bf16_hi(h));
}

// Blocks are dealt round-robin to the 8 XCDs; this gives XCD x a contiguous eighth of every
// grid-wide round of items, so one XCD's L2 sees neighbouring tiles of the same linear.
__device__ __forceinline__ int xcd_contiguous_block(int b, int grid) {
  return (b & 7) * (grid >> 3) + (b >> 3);
}

// Values that are the same in every lane, told to the compiler so they live in scalar registers.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ T* uniform(T* ptr) {
  const uint64_t u = reinterpret_cast<uint64_t>(ptr);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(u));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(u >> 32));
  return reinterpret_cast<T*>((uint64_t(hi) << 32) | lo);
}

// ---------------------------------------------------------------------------
// A re-layout for the matrix-core kernel
//   A   fp32 [E][r][in]                       (LoRA_DOWN as the caller stores it)
//   Apk bf16 [E][r/8][ncb][8][2][32][8]       ncb = ceil(in/256) column blocks of 256
// For expert e, rank group g (ranks 8g..8g+7) and column j = 256*cb + 8*n + b the 8 ranks are
// stored as 8 bf16 high parts at [e][g][cb][b][0][n][.] and 8 bf16 low parts at [..][b][1][n][.]
// (columns past `in` hold zeros).  A matrix-core lane wants 8 consecutive k of one column; in this
// order the 32 lanes of one access (n = 0..31, fixed b) read 512 contiguous bytes.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pack_A(const float* __restrict__ A, uint16_t* __restrict__ Apk,
                                                int E, int r, int in) {
  const int gpr = r >> 3;
  const int in_pad = ceil_div(in, kApkBlockCols) * kApkBlockCols;
  const long long total = (long long)E * gpr * in_pad;
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int j = int(idx % in_pad);
    const long long eg = idx / in_pad;
    const int g = int(eg % gpr);
    const int e = int(eg / gpr);
    float x[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) x[q] = 0.0f;
    if (j < in) {
      const float* src = A + ((long long)e * r + 8 * g) * in + j;
#pragma unroll
      for (int q = 0; q < 8; ++q) x[q] = src[(long long)q * in];
    }
    u32x4 hi, lo;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint32_t h, l;
      split2(x[2 * q], x[2 * q + 1], &h, &l);
      hi[q] = h;
      lo[q] = l;
    }
    const int cb = j / kApkBlockCols, jj = j % kApkBlockCols, n = jj >> 3, b = jj & 7;
    // element offset of [e][g][cb][b][0][n][0]
    const long long base = ((eg * (in_pad / kApkBlockCols) + cb) * 8 + b) * (2 * 32 * 8) + n * 8;
    *reinterpret_cast<u32x4*>(Apk + base) = hi;
    *reinterpret_cast<u32x4*>(Apk + base + 32 * 8) = lo;
  }
}

hipError_t launch_pack_A(const float* A, uint16_t* Apk, int E, int r, int in, hipStream_t s) {
  const long long total = (long long)E * (r / 8) * (ceil_div(in, kApkBlockCols) * kApkBlockCols);
  int grid = int(std::min<long long>((total + 255) / 256, 1 << 16));
  hipLaunchKernelGGL(k_pack_A, dim3(grid), dim3(256), 0, s, A, Apk, E, r, in);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Fused switch, fp32 vector-ALU flavour (any rank).
// One work item = 64 x 128 tile of one W.  256 threads, each owning 4 rows x 8 columns.
// The fused factors of Eq. 9 are staged in LDS in slices of 32 along the concatenated rank:
//   sB[i][k] = coeff_c * B[e_c][row0+i][rho]   (the gate and the sign of the old set live here)
//   sA[k][j] = A[e_c][rho][col0+j]             with k = c*r + rho
// ---------------------------------------------------------------------------
constexpr int VT_ROWS = kValuTileRows, VT_COLS = kValuTileCols, VT_K = 32;

__global__ __launch_bounds__(256) void k_switch_valu(LaunchPlan p, Terms t, int r) {
  __shared__ float sB[VT_ROWS][VT_K + 1];
  __shared__ float sA[VT_K][VT_COLS];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int K = t.n * r;
  const int vb = xcd_contiguous_block(blockIdx.x, gridDim.x);

  for (int item = vb; item < p.n_items; item += gridDim.x) {
    const int s = find_segment(p.first, p.n_sel, item);
    const LinDesc L = p.lin[p.sel[s]];
    int row0, col0;
    decode_item(item - p.first[s], L.in, VT_ROWS, VT_COLS, &row0, &col0);

    float acc[4][8];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[m][q] = 0.0f;

    for (int k0 = 0; k0 < K; k0 += VT_K) {
      __syncthreads();
      for (int idx = tid; idx < VT_ROWS * VT_K; idx += 256) {
        const int i = idx / VT_K, kk = idx % VT_K;
        const int k = k0 + kk, row = row0 + i;
        float v = 0.0f;
        if (k < K && row < L.out) {
          const int c = k / r, rho = k - c * r;
          v = t.coeff[c] * L.B[((long long)t.e[c] * L.out + row) * r + rho];
        }
        sB[i][kk] = v;
      }
      for (int idx = tid; idx < VT_K * VT_COLS; idx += 256) {
        const int kk = idx / VT_COLS, j = idx % VT_COLS;
        const int k = k0 + kk, col = col0 + j;
        float v = 0.0f;
        if (k < K && col < L.in) {
          const int c = k / r, rho = k - c * r;
          v = L.A[((long long)t.e[c] * r + rho) * L.in + col];
        }
        sA[kk][j] = v;
      }
      __syncthreads();
#pragma unroll 8
      for (int kk = 0; kk < VT_K; ++kk) {
        const f32x4 a0 = *reinterpret_cast<const f32x4*>(&sA[kk][tx * 8]);
        const f32x4 a1 = *reinterpret_cast<const f32x4*>(&sA[kk][tx * 8 + 4]);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const float b = sB[ty * 4 + m][kk];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            acc[m][q] = fmaf(b, a0[q], acc[m][q]);
            acc[m][4 + q] = fmaf(b, a1[q], acc[m][4 + q]);
          }
        }
      }
    }

    const int col = col0 + tx * 8;
    if (col < L.in) {
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const int row = row0 + ty * 4 + m;
        if (row < L.out) {
          u32x4* ptr = reinterpret_cast<u32x4*>(L.W + (long long)row * L.in + col);
          const u32x4 w = __builtin_nontemporal_load(ptr);
          u32x4 o;
#pragma unroll
          for (int q = 0; q < 4; ++q)
            o[q] = pack_bf16(bf16_lo(w[q]) + acc[m][2 * q], bf16_hi(w[q]) + acc[m][2 * q + 1]);
          __builtin_nontemporal_store(o, ptr);
        }
      }
    }
  }
}

hipError_t launch_switch_valu(const LaunchPlan& p, const Terms& t, int r, int grid, hipStream_t s) {
  hipLaunchKernelGGL(k_switch_valu, dim3(grid), dim3(256), 0, s, p, t, r);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Fused switch, matrix-core flavour (rank a multiple of 8, fused rank K <= 64).
//
// One wave per workgroup, no LDS staging of tiles, no barrier in the streaming loop.
// A work item is 32 rows x up to 1024 columns of one W; the wave walks it in steps of
// 32 rows x 256 columns (512 contiguous bytes per row, 16 KB per step) and keeps going
// through its items without draining: the W tile of the next step (of the next item, at an
// item boundary) is requested before the matrix work of the current one starts.
//
// v_mfma_f32_32x32x16_bf16 computes D[m][n] += sum_k P[m][k] Q[k][n]; lane l supplies
// P[m = l%32][8*(l/32) .. +8] and Q[8*(l/32) .. +8][n = l%32] and owns, in register v of D,
// the element (m = 8*(v/4) + 4*(l/32) + v%4, n = l%32).
// Mapping: m <-> row of W (row0 + m), and in matrix block b (0..7) n <-> column 8n + b of the
// step.  A lane therefore owns, for each of its 16 rows, the 8 CONTIGUOUS columns 8n..8n+7
// (one per block): a 16-byte load of W fills one register of each of the 8 accumulators, and
// lanes 0..31 (resp. 32..63) of one access cover 512 contiguous bytes of one row.  The
// accumulator layout IS the coalesced layout, so W goes global -> registers -> global with
// nothing in between.
//
// Precision: P = coeff * B (fp32 product) and Q = A are each split into bf16 high + low parts;
// high*high + high*low + low*high keeps the update accurate to about 2^-16 relative, far
// below the one bf16 rounding of the result.  W itself is loaded into the fp32 accumulators,
// so the sum is rounded to bf16 exactly once.
// ---------------------------------------------------------------------------
constexpr int MT_ROWS = kMfmaTileRows, MT_COLS = kMfmaTileCols, MT_STEP = kApkBlockCols;
constexpr uint32_t kOutOfRange = 0x80000000u;   // byte offset beyond any W (out*in*2 < 2^31 is checked at create)

// W is addressed through a buffer resource whose size is the matrix: a row past the last one or
// a lane whose columns lie past the tile gets an offset outside the buffer, which the hardware
// answers with zeros on loads and drops on stores.  No clamping or predication in the loop.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t w_resource(const uint16_t* W, int out, int in) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(W), 0, out * in * 2, 0x00020000);
}

template <int NKS>
struct MfmaItem {           // what a wave keeps per work item
  __amdgpu_buffer_rsrc_t Wres;
  const uint16_t* Apk;      // packed A of the linear
  int ncb;                  // its column blocks
  int col0, col_end;
  uint32_t row0_byte;       // byte offset of row row0 (uniform)
  uint32_t stride_byte;     // bytes per row (uniform)
  u32x4 p_hi[NKS], p_lo[NKS];
};

template <int NKS>
__device__ __forceinline__ void mfma_load_item(const LaunchPlan& p, int item, int n, int gpr, int r,
                                               const int (&term_e)[NKS], const int (&term_g)[NKS],
                                               const float (&term_c)[NKS], MfmaItem<NKS>& it) {
  const int seg = uniform(find_segment(p.first, p.n_sel, item));
  const LinDesc* Lp = p.lin + uniform(p.sel[seg]);
  LinDesc L;
  L.W = uniform(Lp->W);
  L.B = uniform(Lp->B);
  L.Apk = uniform(Lp->Apk);
  L.out = uniform(Lp->out);
  L.in = uniform(Lp->in);
  int row0, col0;
  decode_item(uniform(item - p.first[seg]), L.in, MT_ROWS, MT_COLS, &row0, &col0);
  it.Wres = w_resource(L.W, L.out, L.in);
  it.Apk = L.Apk;
  it.ncb = ceil_div(L.in, MT_STEP);
  it.col0 = col0;
  it.col_end = min(L.in, col0 + MT_COLS);
  it.stride_byte = uint32_t(L.in) * 2u;
  it.row0_byte = uint32_t(row0) * it.stride_byte;
  const int prow = min(row0 + n, L.out - 1);
  const bool prow_ok = row0 + n < L.out;
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const float* src = L.B + ((long long)term_e[ks] * L.out + prow) * r + 8 * term_g[ks];
    const f32x4 b0 = *reinterpret_cast<const f32x4*>(src);
    const f32x4 b1 = *reinterpret_cast<const f32x4*>(src + 4);
    const float c = prow_ok ? term_c[ks] : 0.0f;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      uint32_t hi, lo;
      split2(c * b0[2 * q], c * b0[2 * q + 1], &hi, &lo);
      it.p_hi[ks][q] = hi;
      it.p_lo[ks][q] = lo;
      split2(c * b1[2 * q], c * b1[2 * q + 1], &hi, &lo);
      it.p_hi[ks][2 + q] = hi;
      it.p_lo[ks][2 + q] = lo;
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
#pragma unroll
  for (int v = 0; v < 16; ++v)
    wbuf[v] = __builtin_amdgcn_raw_buffer_load_b128(
        it.Wres, lane_off + uint32_t(8 * (v >> 2) + (v & 3)) * it.stride_byte, 0, /*nt*/ 2);
}

template <int NKS>
__device__ __forceinline__ void mfma_load_q(const MfmaItem<NKS>& it, int cs, int n, int gpr, int e, int g,
                                            u32x4 (&q_hi)[8], u32x4 (&q_lo)[8]) {
  const u32x4* src = reinterpret_cast<const u32x4*>(
      it.Apk + (((long long)e * gpr + g) * it.ncb + cs / MT_STEP) * (8 * 2 * 32 * 8)) + n;
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    q_hi[b] = src[(2 * b) * 32];
    q_lo[b] = src[(2 * b + 1) * 32];
  }
}

template <int NKS>
__global__ __launch_bounds__(64) void k_switch_mfma(LaunchPlan p, Terms t, int r) {
  __shared__ int32_t s_e[kMaxTerms];
  __shared__ float s_coeff[kMaxTerms];
  const int lane = threadIdx.x;
  if (lane < kMaxTerms) {
    s_e[lane] = t.e[lane];
    s_coeff[lane] = t.coeff[lane];
  }
  __syncthreads();

  const int n = lane & 31, h = lane >> 5;
  const int gpr = r >> 3;              // rank groups of 8 per expert
  const int n_groups = t.n * gpr;      // <= 2 * NKS
  const int grid = gridDim.x;

  // per k-step: which (term, rank group) this lane's 8 k-values belong to
  int term_e[NKS], term_g[NKS];
  float term_c[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const int G = 2 * ks + h;
    const bool valid = G < n_groups;
    const int c = valid ? G / gpr : 0;
    term_e[ks] = s_e[c];
    term_g[ks] = valid ? G - c * gpr : 0;
    term_c[ks] = valid ? s_coeff[c] : 0.0f;      // a zero coefficient blanks the padded k-group
  }

  int item = xcd_contiguous_block(blockIdx.x, grid);
  if (item >= p.n_items) return;
  MfmaItem<NKS> cur;
  mfma_load_item<NKS>(p, item, n, gpr, r, term_e, term_g, term_c, cur);
  int cs = cur.col0;
  uint32_t lane_off = mfma_lane_offset<NKS>(cur, cs, n, h);
  u32x4 wbuf[16];
  mfma_load_w<NKS>(cur, lane_off, wbuf);

  constexpr int QB = NKS < 2 ? NKS : 2;     // Q buffers in registers
  while (true) {
    u32x4 q_hi[QB][8], q_lo[QB][8];
#pragma unroll
    for (int ks = 0; ks < QB; ++ks)
      mfma_load_q<NKS>(cur, cs, n, gpr, term_e[ks], term_g[ks], q_hi[ks], q_lo[ks]);

    // W -> accumulators
    f32x16 acc[8];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc[2 * q][v] = bf16_lo(wbuf[v][q]);
        acc[2 * q + 1][v] = bf16_hi(wbuf[v][q]);
      }
    }

    // where the wave goes next
    const bool same = cs + MT_STEP < cur.col_end;
    const int nitem = same ? item : item + grid;
    const bool have_next = same || nitem < p.n_items;
    MfmaItem<NKS> nxt = cur;
    int ncs = cs + MT_STEP;
    uint32_t nlane_off = kOutOfRange;

#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      // request the next W tile once every Q load of this step has been issued: loads complete
      // in issue order, so anything requested after it would have to wait for it
      if (ks == (NKS > 2 ? NKS - 2 : 0)) {
        if (have_next) {
          if (!same) {
            mfma_load_item<NKS>(p, nitem, n, gpr, r, term_e, term_g, term_c, nxt);
            ncs = nxt.col0;
          }
          nlane_off = mfma_lane_offset<NKS>(nxt, ncs, n, h);
          mfma_load_w<NKS>(nxt, nlane_off, wbuf);
        }
      }
      const bf16x8 ph = __builtin_bit_cast(bf16x8, cur.p_hi[ks]);
      const bf16x8 pl = __builtin_bit_cast(bf16x8, cur.p_lo[ks]);
      u32x4(&qh)[8] = q_hi[ks % QB];
      u32x4(&ql)[8] = q_lo[ks % QB];
#pragma unroll
      for (int b = 0; b < 8; ++b)
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl, __builtin_bit_cast(bf16x8, qh[b]), acc[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < 8; ++b)
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, __builtin_bit_cast(bf16x8, ql[b]), acc[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < 8; ++b)
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, __builtin_bit_cast(bf16x8, qh[b]), acc[b], 0, 0, 0);
      if (ks + 2 < NKS)
        mfma_load_q<NKS>(cur, cs, n, gpr, term_e[ks + 2], term_g[ks + 2], qh, ql);
    }

    // accumulators -> W (one rounding)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      u32x4 o;
#pragma unroll
      for (int q = 0; q < 4; ++q) o[q] = pack_bf16(acc[2 * q][v], acc[2 * q + 1][v]);
      __builtin_amdgcn_raw_buffer_store_b128(
          o, cur.Wres, lane_off + uint32_t(8 * (v >> 2) + (v & 3)) * cur.stride_byte, 0, /*nt*/ 2);
    }
    if (!have_next) break;
    cur = nxt;
    cs = ncs;
    item = nitem;
    lane_off = nlane_off;
  }
}

hipError_t launch_switch_mfma(const LaunchPlan& p, const Terms& t, int r, int grid, hipStream_t s) {
  const int n_groups = t.n * (r / 8);
  const int nks = (n_groups + 1) / 2;
  switch (nks) {
    case 1: hipLaunchKernelGGL(k_switch_mfma<1>, dim3(grid), dim3(64), 0, s, p, t, r); break;
    case 2: hipLaunchKernelGGL(k_switch_mfma<2>, dim3(grid), dim3(64), 0, s, p, t, r); break;
    case 3: hipLaunchKernelGGL(k_switch_mfma<3>, dim3(grid), dim3(64), 0, s, p, t, r); break;
    case 4: hipLaunchKernelGGL(k_switch_mfma<4>, dim3(grid), dim3(64), 0, s, p, t, r); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Merged decode: y = W x, bf16 inputs, fp32 accumulation.  One wave per 4 rows.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_gemv(const uint16_t* __restrict__ W, const uint16_t* __restrict__ x,
                                              float* __restrict__ y, int out, int in) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row0 = (blockIdx.x * 4 + wave) * 4;
  if (row0 >= out) return;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  const uint16_t* rows[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) rows[m] = W + (long long)min(row0 + m, out - 1) * in;
  for (int j = lane * 8; j < in; j += 512) {
    const u32x4 xv = *reinterpret_cast<const u32x4*>(x + j);
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rows[m] + j));
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc[m] = fmaf(bf16_lo(w[q]), bf16_lo(xv[q]), acc[m]);
        acc[m] = fmaf(bf16_hi(w[q]), bf16_hi(xv[q]), acc[m]);
      }
    }
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    float v = acc[m];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0 && row0 + m < out) y[row0 + m] = v;
  }
}

hipError_t launch_gemv(const uint16_t* W, const uint16_t* x, float* y, int out, int in, hipStream_t s) {
  const int grid = (out + 15) / 16;
  hipLaunchKernelGGL(k_gemv, dim3(grid), dim3(256), 0, s, W, x, y, out, in);
  return hipGetLastError();
}

}  // namespace lsw
