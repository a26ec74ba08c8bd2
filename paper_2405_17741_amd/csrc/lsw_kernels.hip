// Device code of liblsw for gfx950 (MI355X): the fused adapter switch (two matrix-core kernels, for fused ranks up
// to 64 and up to 256, and an fp32 vector-ALU kernel for any rank), the operand re-layout kernels, the device-side
// router and term-list builder, the in-place bandwidth probe, the merged-decode GEMVs, and the un-merged adapter path
// for prompts.  Sec. 3.2-3.4 of LoRA-Switch define what is computed; the tiling, data movement and launch shapes are
// this library's own.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>
#include <utility>

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
// Pointers read from the descriptor table are generic to the compiler; casts to this address space tell it
// they point to global memory, so it emits global_load (vmcnt only) instead of flat_load.
#define LSW_GLOBAL __attribute__((address_space(1)))
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

// Eight consecutive factor elements as fp32.  QP = 2: the factors are stored as fp32 (the matrix-core kernels
// split them into bf16 high + low parts, "two Q parts"); QP = 1: they are stored as bf16 and are exact as they are.
template <int QP>
__device__ __forceinline__ void load8(const void* base, long long elem, float (&x)[8]) {
  if constexpr (QP == 2) {
    const LSW_GLOBAL f32x4* src = (const LSW_GLOBAL f32x4*)(reinterpret_cast<const float*>(base) + elem);
    const f32x4 b0 = src[0], b1 = src[1];
#pragma unroll
    for (int q = 0; q < 4; ++q) { x[q] = b0[q]; x[4 + q] = b1[q]; }
  } else {
    const u32x4 w = *(const LSW_GLOBAL u32x4*)(reinterpret_cast<const uint16_t*>(base) + elem);
#pragma unroll
    for (int q = 0; q < 4; ++q) { x[2 * q] = bf16_lo(w[q]); x[2 * q + 1] = bf16_hi(w[q]); }
  }
}
template <int QP>
__device__ __forceinline__ float load1(const void* base, long long elem) {
  if constexpr (QP == 2) return reinterpret_cast<const float*>(base)[elem];
  else return __uint_as_float(uint32_t(reinterpret_cast<const uint16_t*>(base)[elem]) << 16);
}

// Blocks are dealt round-robin to the 8 XCDs; this gives XCD x a contiguous eighth of every
// grid-wide round of items, so one XCD's L2 sees neighbouring tiles of the same linear.
__device__ __forceinline__ int xcd_contiguous_block(int b, int grid) {
  return (b & 7) * (grid >> 3) + (b >> 3);
}

template <typename T>
__device__ __forceinline__ const LSW_GLOBAL T* as_global(const T* ptr) {
  return (const LSW_GLOBAL T*)ptr;
}

// One 16-byte-per-lane copy from global memory straight into LDS (no registers): lane l's 16 bytes
// land at lds_base + 16*l.  Written as inline assembly on purpose: the compiler's wait-count pass
// treats its own LDS-DMA builtin as "may touch both memory kinds" and, while one is in flight, turns
// every later wait on an LDS read or a global load into a full drain, which serialises the LDS
// prefetch of the matrix-core loops.  Hidden from that pass, the copy only makes the compiler's own
// vector-memory waits more conservative (the counter is in order); its completion is waited for by
// hand (s_waitcnt vmcnt) before the workgroup barrier that publishes the buffer.  M0 is written here
// and has no other user in these kernels.
__device__ __forceinline__ void lds_dma16(const void* src, const void* lds_base) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
      uint32_t(uintptr_t((const __attribute__((address_space(3))) void*)lds_base)));
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr) : "memory", "m0");
}

// The term list of a launch comes by value with the launch (host-side lists) or from device memory
// (device-resident routing: a small kernel wrote it just before on the same stream).
#define LSW_LOAD_TERMS(t, t_dev, s_e, s_c, n_out)                         \
  do {                                                                    \
    if (threadIdx.x < kMaxTerms) {                                        \
      if (t_dev) {                                                        \
        s_e[threadIdx.x] = t_dev->e[threadIdx.x];                         \
        s_c[threadIdx.x] = t_dev->coeff[threadIdx.x];                     \
      } else {                                                            \
        s_e[threadIdx.x] = t.e[threadIdx.x];                              \
        s_c[threadIdx.x] = t.coeff[threadIdx.x];                          \
      }                                                                   \
    }                                                                     \
    n_out = __builtin_amdgcn_readfirstlane(t_dev ? t_dev->n : t.n);       \
  } while (0)

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
//   A   fp32 or bf16 [E][r][in]               (LoRA_DOWN as the caller stores it)
//   Apk bf16 [E][r/8][ncb][8][QP][32][8]      ncb = ceil(in/256) column blocks of 256
// For expert e, rank group g (ranks 8g..8g+7) and column j = 256*cb + 8*n + b the 8 ranks are
// stored as 8 bf16 high parts at [e][g][cb][b][0][n][.] and, for fp32 factors (QP = 2), 8 bf16 low
// parts at [..][b][1][n][.]; bf16 factors (QP = 1) are exact in the one part (columns past `in` hold zeros).  A matrix-core lane wants 8 consecutive k of one column; in this
// order the 32 lanes of one access (n = 0..31, fixed b) read 512 contiguous bytes.
// ---------------------------------------------------------------------------
// TRANSPOSED: the source is B [E][out][r] read as B^T [E][r][out] (`in` is then the number of its columns, out): the
// Q operand of the un-merged adapter path, whose matrix rows are tokens and whose columns are output features.
template <int QP, bool TRANSPOSED>
__global__ __launch_bounds__(256) void k_pack_A(const void* __restrict__ A, uint16_t* __restrict__ Apk,
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
#pragma unroll
      for (int q = 0; q < 8; ++q)
        x[q] = load1<QP>(A, TRANSPOSED ? ((long long)e * in + j) * r + 8 * g + q : ((long long)e * r + 8 * g + q) * in + j);
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
    const long long base = ((eg * (in_pad / kApkBlockCols) + cb) * 8 + b) * (QP * 32 * 8) + n * 8;
    *reinterpret_cast<u32x4*>(Apk + base) = hi;
    if constexpr (QP == 2) *reinterpret_cast<u32x4*>(Apk + base + 32 * 8) = lo;
  }
}

hipError_t launch_pack_A(const void* A, uint16_t* Apk, int E, int r, int in, int qp, int transposed, hipStream_t s) {
  const long long total = (long long)E * (r / 8) * (ceil_div(in, kApkBlockCols) * kApkBlockCols);
  int grid = int(std::min<long long>((total + 255) / 256, 1 << 16));
  if (qp == 2 && !transposed) hipLaunchKernelGGL((k_pack_A<2, false>), dim3(grid), dim3(256), 0, s, A, Apk, E, r, in);
  else if (qp == 2) hipLaunchKernelGGL((k_pack_A<2, true>), dim3(grid), dim3(256), 0, s, A, Apk, E, r, in);
  else if (!transposed) hipLaunchKernelGGL((k_pack_A<1, false>), dim3(grid), dim3(256), 0, s, A, Apk, E, r, in);
  else hipLaunchKernelGGL((k_pack_A<1, true>), dim3(grid), dim3(256), 0, s, A, Apk, E, r, in);
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

template <int QP>
__global__ __launch_bounds__(256) void k_switch_valu(LaunchPlan p, Terms t, const Terms* t_dev, int r) {
  __shared__ float sB[VT_ROWS][VT_K + 1];
  __shared__ float sA[VT_K][VT_COLS];
  __shared__ int32_t s_te[kMaxTerms];
  __shared__ float s_tc[kMaxTerms];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  int n_terms;
  LSW_LOAD_TERMS(t, t_dev, s_te, s_tc, n_terms);
  if (n_terms == 0) return;             // nothing to merge or unmerge (device-built lists only): W stays untouched
  __syncthreads();
  const int K = n_terms * r;
  const int vb = p.xcd_remap ? xcd_contiguous_block(blockIdx.x, gridDim.x) : int(blockIdx.x);

  for (int item = vb; item < p.n_items; item += gridDim.x) {
    const int s = find_segment(p.first, p.n_sel, item);
    const LinDesc L = p.lin[p.sel[s]];
    int row0, col0;
    decode_item(item - p.first[s], L.out, L.in, VT_ROWS, VT_COLS, 0, &row0, &col0);

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
          v = s_tc[c] * load1<QP>(L.B, ((long long)s_te[c] * L.out + row) * r + rho);
        }
        sB[i][kk] = v;
      }
      for (int idx = tid; idx < VT_K * VT_COLS; idx += 256) {
        const int kk = idx / VT_COLS, j = idx % VT_COLS;
        const int k = k0 + kk, col = col0 + j;
        float v = 0.0f;
        if (k < K && col < L.in) {
          const int c = k / r, rho = k - c * r;
          v = load1<QP>(L.A, ((long long)s_te[c] * r + rho) * L.in + col);
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
          const u32x4 w = __builtin_nontemporal_load(
              p.from_base ? reinterpret_cast<const u32x4*>(L.Wbase + (long long)row * L.in + col) : ptr);
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

hipError_t launch_switch_valu(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int qp, int grid, hipStream_t s) {
  if (qp == 2) hipLaunchKernelGGL(k_switch_valu<2>, dim3(grid), dim3(256), 0, s, p, t, t_dev, r);
  else hipLaunchKernelGGL(k_switch_valu<1>, dim3(grid), dim3(256), 0, s, p, t, t_dev, r);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Fused switch, matrix-core flavour (rank a multiple of 8, fused rank K = terms * r <= 64).
//
// Launch shape.  A workgroup is 4 waves (one per SIMD), one workgroup per CU, persistent: it
// walks work items  blockIdx, blockIdx + grid, ...  A work item is 128 rows x tile_cols columns
// of one W; wave w owns rows 32w..32w+31 and walks the item in steps of 32 rows x 256 columns
// (512 contiguous bytes per row, 16 KB per wave and step).
//
// Tile mapping.  v_mfma_f32_32x32x16_bf16 computes D[m][n] += sum_k P[m][k] Q[k][n]; lane l
// supplies P[m = l%32][8*(l/32) .. +8] and Q[8*(l/32) .. +8][n = l%32] and owns, in register v of
// D, the element (m = 8*(v/4) + 4*(l/32) + v%4, n = l%32).  Here m <-> row of W, and in matrix
// block b (0..7) n <-> column 8n + b of the step.  A lane therefore owns, for each of its 16
// rows, the 8 CONTIGUOUS columns 8n..8n+7 (one per block): one 16-byte load of W feeds one
// register of each of the 8 accumulators, and lanes 0..31 (resp. 32..63) of one access cover 512
// contiguous bytes of one row.  The accumulator layout IS the coalesced layout, so W goes
// global -> registers -> global with no shuffle in between.
//
// Operands.  P = coeff * B (the gate and the sign of the unmerged set, Eq. 5 / Eq. 9), computed in
// fp32 once per item and kept in registers.  Q = A comes from the packed copy (see k_pack_A); the
// Q of a step is the same for the 4 waves, so each wave copies a quarter of it from L2 into LDS
// (LDS-DMA, no registers) one step ahead, and all read it from there.
//
// Precision.  P and Q are each split into bf16 high + low parts; high*high + high*low + low*high
// keeps the update accurate to about 2^-16 relative, far below the one bf16 rounding of the
// result.  W itself is widened into the fp32 accumulators, so the sum is rounded to bf16 once.
//
// Memory schedule of one step (per wave): start the LDS copy of the next step's Q quarter; store
// the previous step's finished tile; request the next W tile into the registers just stored from
// (next item's first tile at an item boundary: scalar selects, no branch); compute; wait for
// everything requested to land; workgroup barrier (LDS-only fence).  One W tile per wave is in
// flight at any time, which is what the memory system sustains best for this in-place pattern.
// W is addressed through a buffer resource sized to the matrix: rows past the end and lanes whose
// columns lie past the tile get an offset outside the buffer, which the hardware answers with
// zeros on loads and drops on stores, so the loop has no clamping and no predication.
// ---------------------------------------------------------------------------
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

template <int NKS, int QP>
__device__ __forceinline__ void mfma_load_item(const LaunchPlan& p, int item, int n, int gpr, int r,
                                               const int (&term_e)[NKS], const int (&term_g)[NKS],
                                               const float (&term_c)[NKS], MfmaItem<NKS>& it,
                                               int tile_rows, int row_shift) {
  const bool adapter = p.Z != nullptr;          // adapter-path mode: one matrix, rows = tokens, row operand = rows of Z
  LinDesc L;
  int local = item;
  if (adapter) {
    L.W = p.one.W;
    L.B = nullptr;
    L.Apk = p.one.Apk;
    L.Wbase = nullptr;
    L.out = p.one.out;
    L.in = p.one.in;
  } else {
    const int seg = uniform(find_segment(p.first, p.n_sel, item));
    const LinDesc* Lp = p.lin + uniform(p.sel[seg]);
    L.W = uniform(Lp->W);
    L.B = uniform(Lp->B);
    L.Apk = uniform(Lp->Apk);
    L.Wbase = p.from_base ? uniform(Lp->Wbase) : nullptr;
    L.out = uniform(Lp->out);
    L.in = uniform(Lp->in);
    local = uniform(item - p.first[seg]);
  }
  int row0, col0;
  decode_item(local, L.out, L.in, tile_rows, p.tile_cols, p.panel_group, &row0, &col0);
  row0 += row_shift;          // the calling wave's 32 rows inside a taller item (may lie past the last row)
  it.W = L.W;
  it.Wsrc = p.from_base ? L.Wbase : L.W;
  it.wbytes = L.out * L.in * 2;
  it.Apk = L.Apk;
  it.ncb = ceil_div(L.in, MT_STEP);
  it.col0 = col0;
  it.col_end = min(L.in, col0 + p.tile_cols);
  it.stride_byte = uint32_t(L.in) * 2u;
  it.row0_byte = uint32_t(row0) * it.stride_byte;
  const int prow = min(row0 + n, L.out - 1);
  const bool prow_ok = row0 + n < L.out;       // rows past the end get a zero coefficient and an offset outside W
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    float b[8];
    if (adapter) load8<2>(p.Z, (long long)prow * p.z_stride + 8 * (term_e[ks] * gpr + term_g[ks]), b);
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
__shared__ int32_t s_walk_claim[2];

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

// One step of a wave: start the copy of the next step's Q quarter into the idle LDS buffer, store
// the previous step's tile, request the next tile into the freed registers, update the current
// tile, then drain and meet the workgroup.  Everything requested at the top has the whole compute
// phase to arrive.  Returns false after the last tile of the workgroup.
template <int NKS, int QP>
__device__ __forceinline__ bool wg_step(const LaunchPlan& p, int n, int h, int lane, int wave, int gpr, int r,
                                        const int (&term_e)[NKS], const int (&term_g)[NKS],
                                        const float (&term_c)[NKS], MfmaItem<NKS>& cur, MfmaItem<NKS>& nxt,
                                        bool& have_nxt, ItemWalk& walk, int& claim, int& cs, uint32_t& lane_off,
                                        __amdgpu_buffer_rsrc_t& prev_res, uint32_t& prev_off, uint32_t& prev_stride,
                                        u32x4 (&wcur)[16], u32x4 (&wprev)[16], int buf) {
  constexpr int kBufSlots = NKS * 8 * QP * 64;
  const bool last = uniform(int(!(cs + MT_STEP < cur.col_end))) != 0;
  const bool more = !last || have_nxt;
  const __amdgpu_buffer_rsrc_t nres = w_resource(last ? nxt.Wsrc : cur.Wsrc, last ? nxt.wbytes : cur.wbytes);
  const int ncs = uniform(last ? nxt.col0 : cs + MT_STEP);
  const int ncol_end = uniform(last ? nxt.col_end : cur.col_end);
  const uint32_t nrow0_byte = uint32_t(uniform(int(last ? nxt.row0_byte : cur.row0_byte)));
  const uint32_t nstride = uint32_t(uniform(int(last ? nxt.stride_byte : cur.stride_byte)));
  uint32_t nlane_off = kOutOfRange;
  {
    const int col = ncs + 8 * n;
    if (more && col < ncol_end) nlane_off = nrow0_byte + uint32_t(4 * h) * nstride + uint32_t(col) * 2u;
  }
  {   // (a finished workgroup re-reads its last block, which is harmless)
    const int qcs = uniform(more ? ncs : cs);
    const uint16_t* qApk = uniform((more && last) ? nxt.Apk : cur.Apk);
    const int qncb = uniform((more && last) ? nxt.ncb : cur.ncb);
    wg_fetch_q<NKS, QP>(qApk, qncb, qcs, n, gpr, wave, term_e, term_g, wg_lds + (buf ^ 1) * kBufSlots);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v)
    __builtin_amdgcn_raw_buffer_store_b128(
        wprev[v], prev_res, prev_off + uint32_t(8 * (v >> 2) + (v & 3)) * prev_stride, 0, kWStoreAux);
  asm volatile("" : "+v"(nlane_off) : "v"(prev_off));      // keep the loads after the stores that free their registers
#pragma unroll
  for (int v = 0; v < 16; ++v)
    wprev[v] = __builtin_amdgcn_raw_buffer_load_b128(
        nres, nlane_off + uint32_t(8 * (v >> 2) + (v & 3)) * nstride, 0, kWLoadAux);

  wg_compute<NKS, QP>(cur.p_hi, cur.p_lo, wg_lds + buf * kBufSlots + lane, wcur);

  if (last && walk.after_pool) walk_publish_claim(walk, wave, claim);
  wg_drain_and_barrier();

  prev_res = w_resource(cur.W, cur.wbytes);
  prev_off = lane_off;
  prev_stride = cur.stride_byte;
  lane_off = nlane_off;
  cs = ncs;
  if (last) {                      // item boundary: rare, and the only branch of the step (uniform over the workgroup)
    if (!have_nxt) return false;
    cur = nxt;
    const bool via_pool = walk.after_pool;
    const int following = via_pool ? walk_take_claim(walk) : walk.after;
    have_nxt = following >= 0;
    if (have_nxt) {
      mfma_load_item<NKS, QP>(p, following, n, gpr, r, term_e, term_g, term_c, nxt, WG_ROWS, 32 * wave);
      walk_plan_after(walk, following, via_pool, wave, lane, claim);
    }
  }
  return true;
}

template <int NKS, int QP>
__global__ __launch_bounds__(64 * WG_WAVES) void k_switch_mfma(LaunchPlan p, Terms t, const Terms* t_dev, int r) {
  __shared__ int32_t s_e[kMaxTerms];
  __shared__ float s_coeff[kMaxTerms];
  const int lane = threadIdx.x & 63;
  const int wave = uniform(int(threadIdx.x >> 6));
  int n_terms;
  LSW_LOAD_TERMS(t, t_dev, s_e, s_coeff, n_terms);
  if (n_terms == 0) return;             // nothing to merge or unmerge (device-built lists only): W stays untouched
  __syncthreads();

  const int n = lane & 31, h = lane >> 5;
  const int gpr = r >> 3;
  const int n_groups = n_terms * gpr;
  const bool adapter = p.Z != nullptr;      // adapter-path mode: the "terms" are all experts 0..n_terms-1, coefficient 1
  int term_e[NKS], term_g[NKS];
  float term_c[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const int G = 2 * ks + h;
    const bool valid = G < n_groups;
    const int c = valid ? G / gpr : 0;
    term_e[ks] = adapter ? c : s_e[c];
    term_g[ks] = valid ? G - c * gpr : 0;
    term_c[ks] = valid ? (adapter ? 1.0f : s_coeff[c]) : 0.0f;
  }

  ItemWalk walk;
  const int item0 = walk_init(p, p.xcd_remap == 2, walk);
  if (item0 >= walk.static_end) return; // uniform over the workgroup (never with a pool)
  MfmaItem<NKS> cur, nxt;
  mfma_load_item<NKS, QP>(p, item0, n, gpr, r, term_e, term_g, term_c, cur, WG_ROWS, 32 * wave);
  bool have_nxt = item0 + walk.step < walk.static_end;
  int claim = 0;
  if (have_nxt) {
    mfma_load_item<NKS, QP>(p, item0 + walk.step, n, gpr, r, term_e, term_g, term_c, nxt, WG_ROWS, 32 * wave);
    walk_plan_after(walk, item0 + walk.step, false, wave, lane, claim);
  } else {
    nxt = cur;
  }
  int cs = cur.col0;
  uint32_t lane_off = mfma_lane_offset<NKS>(cur, cs, n, h);
  u32x4 wa[16], wb[16];
  mfma_load_w<NKS>(cur, lane_off, wa);
#pragma unroll
  for (int v = 0; v < 16; ++v) wb[v] = u32x4{0u, 0u, 0u, 0u};
  wg_fetch_q<NKS, QP>(cur.Apk, cur.ncb, cs, n, gpr, wave, term_e, term_g, wg_lds);
  wg_drain_and_barrier();
  __amdgpu_buffer_rsrc_t prev_res = w_resource(cur.W, cur.wbytes);
  uint32_t prev_off = kOutOfRange, prev_stride = 0;

  bool a_is_cur = true;
  while (true) {
    if (!wg_step<NKS, QP>(p, n, h, lane, wave, gpr, r, term_e, term_g, term_c, cur, nxt, have_nxt, walk, claim, cs, lane_off,
                      prev_res, prev_off, prev_stride, wa, wb, 0)) { a_is_cur = true; break; }
    if (!wg_step<NKS, QP>(p, n, h, lane, wave, gpr, r, term_e, term_g, term_c, cur, nxt, have_nxt, walk, claim, cs, lane_off,
                      prev_res, prev_off, prev_stride, wb, wa, 1)) { a_is_cur = false; break; }
  }
  if (a_is_cur) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
      __builtin_amdgcn_raw_buffer_store_b128(
          wa[v], prev_res, prev_off + uint32_t(8 * (v >> 2) + (v & 3)) * prev_stride, 0, kWStoreAux);
  } else {
#pragma unroll
    for (int v = 0; v < 16; ++v)
      __builtin_amdgcn_raw_buffer_store_b128(
          wb[v], prev_res, prev_off + uint32_t(8 * (v >> 2) + (v & 3)) * prev_stride, 0, kWStoreAux);
  }
  walk_finish(walk);
}

template <int NKS, int QP>
static hipError_t launch_wg(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int grid, hipStream_t s) {
  const size_t lds = size_t(2) * NKS * 8 * QP * 64 * sizeof(u32x4);     // 16 KB per k-step and Q part, two buffers
  // once per process (function-local statics are initialised exactly once, also under concurrent first calls)
  static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_switch_mfma<NKS, QP>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
  if (lds_ok != hipSuccess) return lds_ok;
  hipLaunchKernelGGL((k_switch_mfma<NKS, QP>), dim3(grid), dim3(64 * WG_WAVES), lds, s, p, t, t_dev, r);
  return hipGetLastError();
}

template <int QP>
static hipError_t launch_wg_qp(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int grid, hipStream_t s) {
  const int n_groups = t.n * (r / 8);
  switch ((n_groups + 1) / 2) {
    case 1: return launch_wg<1, QP>(p, t, t_dev, r, grid, s);
    case 2: return launch_wg<2, QP>(p, t, t_dev, r, grid, s);
    case 3: return launch_wg<3, QP>(p, t, t_dev, r, grid, s);
    case 4: return launch_wg<4, QP>(p, t, t_dev, r, grid, s);
    default: return hipErrorInvalidValue;
  }
}

// t.n sizes the kernel (k-steps kept in registers); with t_dev the kernel takes the list itself, which may
// be shorter, from device memory
hipError_t launch_switch_mfma(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int qp, int grid, hipStream_t s) {
  return qp == 2 ? launch_wg_qp<2>(p, t, t_dev, r, grid, s) : launch_wg_qp<1>(p, t, t_dev, r, grid, s);
}

// ---------------------------------------------------------------------------
// Fused switch on the matrix cores with the Q operand of a whole work item RESIDENT in LDS (k_switch_mfma_res).
//
// Same tile mapping, operand split, arithmetic and W addressing as k_switch_mfma, for launches whose Q of one item
// (fused rank x tile_cols columns, 128 KB at K = 32 and 1024 columns) fits LDS.  Two things differ.
//
// Order.  Each XCD walks its own contiguous eighth of the item list, its 32 workgroups taking 32 consecutive items
// per round.  The matrices the eight XCDs touch at one time are then eight, not one, which costs nothing (measured),
// and a workgroup's consecutive items are 32 apart: in a linear with 4 or 8 column panels (4096 or 8192 columns at
// 1024 per item) they lie in the SAME panel, 8 or 4 row blocks further down.
//
// Q.  The item's whole Q is copied into LDS when the panel changes and kept while it does not, so most items of such
// linears copy nothing (the streaming kernel copies 32 KB per 64 KB of W, which costs it about 2 %), and there is no
// per-step workgroup barrier: the four waves run free and meet only where the panel changes.
//
// Per step a wave stores the previous tile, requests the next one (the first tile of the following item at an item
// boundary, with the B rows of that item right behind it), updates the current tile, and at an item boundary turns the
// B rows into the next P.
//
// Balance.  The last sixteenth of every XCD's range goes through the item pool (see ItemWalk); pool items reload Q.
// ---------------------------------------------------------------------------
struct ResItem {            // one work item (128 rows x tile_cols columns of one linear); every field is uniform
  const uint16_t* W;
  const uint16_t* Wsrc;     // where tiles are read from: W, or the base copy when re-basing
  const void* B;
  const uint16_t* Apk;
  int out, in;
  int seg;                  // position of the linear in the launch's selection
  int item;
  int row0, col0;
};

__device__ __forceinline__ void res_item_at(const LaunchPlan& p, int item, ResItem& c) {
  c.seg = uniform(find_segment(p.first, p.n_sel, item));
  const LinDesc* Lp = p.lin + uniform(p.sel[c.seg]);
  c.W = uniform(Lp->W);
  c.Wsrc = p.from_base ? uniform(Lp->Wbase) : c.W;
  c.B = uniform(Lp->B);
  c.Apk = uniform(Lp->Apk);
  c.out = uniform(Lp->out);
  c.in = uniform(Lp->in);
  c.item = item;
  decode_item(uniform(item - p.first[c.seg]), c.out, c.in, kMfmaTileRows, p.tile_cols, p.panel_group, &c.row0, &c.col0);
}

// the B rows of this lane's row of item c (its half of every k-step), as stored
template <int NKS, int QP>
__device__ __forceinline__ void res_load_b(const ResItem& c, int wave, int n, int r, const int (&term_e)[NKS],
                                           const int (&term_g)[NKS], float (&b)[NKS][8]) {
  const int prow = min(c.row0 + 32 * wave + n, c.out - 1);
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) load8<QP>(c.B, ((long long)term_e[ks] * c.out + prow) * r + 8 * term_g[ks], b[ks]);
}

// P = coeff * B, split into bf16 high + low; rows past the end get a zero coefficient (their W offsets lie outside W)
template <int NKS>
__device__ __forceinline__ void res_make_p(const ResItem& c, int wave, int n, const float (&term_c)[NKS],
                                           const float (&b)[NKS][8], u32x4 (&p_hi)[NKS], u32x4 (&p_lo)[NKS]) {
  const bool ok = c.row0 + 32 * wave + n < c.out;
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const float coef = ok ? term_c[ks] : 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint32_t hi, lo;
      split2(coef * b[ks][2 * q], coef * b[ks][2 * q + 1], &hi, &lo);
      p_hi[ks][q] = hi;
      p_lo[ks][q] = lo;
    }
  }
}

// the whole Q of item c into LDS: [column step][k-step][8 blocks][parts][64 lanes]; this wave copies blocks 2*wave and
// 2*wave+1 of every step (column blocks past the last one of the linear are not touched)
template <int NKS, int QP>
__device__ __forceinline__ void res_fetch_q(const LaunchPlan& p, const ResItem& c, int n, int gpr, int wave,
                                            const int (&term_e)[NKS], const int (&term_g)[NKS]) {
  constexpr int kStepSlots = NKS * 8 * QP * 64;
  const int ncb = ceil_div(c.in, MT_STEP);
  const int cb0 = c.col0 / MT_STEP;
  const int nst = uniform(min(p.tile_cols / MT_STEP, ncb - cb0));
  for (int j = 0; j < nst; ++j)
    wg_fetch_q<NKS, QP>(c.Apk, ncb, (cb0 + j) * MT_STEP, n, gpr, wave, term_e, term_g, wg_lds + j * kStepSlots);
}

template <int NKS, int QP>
__device__ __forceinline__ bool res_step(const LaunchPlan& p, int n, int h, int lane, int wave, int gpr, int r,
                                         const int (&term_e)[NKS], const int (&term_g)[NKS], const float (&term_c)[NKS],
                                         ResItem& cur, ResItem& nxt, bool& have_nxt_io, ItemWalk& walk, int& claim,
                                         int& cs, uint32_t& lane_off,
                                         __amdgpu_buffer_rsrc_t& prev_res, uint32_t& prev_off, uint32_t& prev_stride,
                                         u32x4 (&p_hi)[NKS], u32x4 (&p_lo)[NKS], u32x4 (&wcur)[16], u32x4 (&wprev)[16]) {
  constexpr int kStepSlots = NKS * 8 * QP * 64;
  const int col_end = uniform(min(cur.in, cur.col0 + p.tile_cols));
  const bool last = uniform(int(!(cs + MT_STEP < col_end))) != 0;        // last column step of the item
  const bool have_nxt = have_nxt_io;
  const bool more = !last || have_nxt;
  // the tile after this one: the next column step, or the first tile of the following item (scalar selects, no branch)
  const int nout = uniform(last ? nxt.out : cur.out), nin = uniform(last ? nxt.in : cur.in);
  const __amdgpu_buffer_rsrc_t nres = w_resource(last ? nxt.Wsrc : cur.Wsrc, nout * nin * 2);
  const uint32_t nstride = uint32_t(nin) * 2u;
  const int ncs = uniform(last ? nxt.col0 : cs + MT_STEP);
  const int ncol_end = uniform(last ? min(nxt.in, nxt.col0 + p.tile_cols) : col_end);
  const uint32_t nrow0_byte = uint32_t(uniform((last ? nxt.row0 : cur.row0) + 32 * wave)) * nstride;
  uint32_t nlane_off = kOutOfRange;
  {
    const int col = ncs + 8 * n;
    if (more && col < ncol_end) nlane_off = nrow0_byte + uint32_t(4 * h) * nstride + uint32_t(col) * 2u;
  }
#pragma unroll
  for (int v = 0; v < 16; ++v)
    __builtin_amdgcn_raw_buffer_store_b128(
        wprev[v], prev_res, prev_off + uint32_t(8 * (v >> 2) + (v & 3)) * prev_stride, 0, kWStoreAux);
  asm volatile("" : "+v"(nlane_off) : "v"(prev_off));      // keep the loads after the stores that free their registers
#pragma unroll
  for (int v = 0; v < 16; ++v)
    wprev[v] = __builtin_amdgcn_raw_buffer_load_b128(
        nres, nlane_off + uint32_t(8 * (v >> 2) + (v & 3)) * nstride, 0, kWLoadAux);
  const bool boundary = last && have_nxt;
  float braw[NKS][8];
  if (boundary) res_load_b<NKS, QP>(nxt, wave, n, r, term_e, term_g, braw);

  wg_compute<NKS, QP>(p_hi, p_lo, wg_lds + ((cs - cur.col0) / MT_STEP) * kStepSlots + lane, wcur);

  prev_res = w_resource(cur.W, cur.out * cur.in * 2);
  prev_off = lane_off;
  prev_stride = uint32_t(cur.in) * 2u;
  lane_off = nlane_off;
  cs = ncs;
  if (last) {                      // item boundary (uniform over the workgroup: all four waves walk the same items)
    if (!have_nxt) return false;
    res_make_p<NKS>(nxt, wave, n, term_c, braw, p_hi, p_lo);
    const bool via_pool = walk.after_pool;       // the item after nxt is the one wave 0 claimed a boundary ago
    const bool new_panel = uniform(int(via_pool || nxt.seg != cur.seg || nxt.col0 != cur.col0)) != 0;
    cur = nxt;
    int following = walk.after;
    if (!via_pool) {
      have_nxt_io = following >= 0;
      if (have_nxt_io) res_item_at(p, following, nxt);
    }
    if (new_panel) {
      if (via_pool) walk_publish_claim(walk, wave, claim);
      wg_drain_and_barrier();      // every wave has finished with the old panel's Q (and sees wave 0's claim)
      if (via_pool) {
        following = walk_take_claim(walk);
        have_nxt_io = following >= 0;
        if (have_nxt_io) res_item_at(p, following, nxt);
      }
      res_fetch_q<NKS, QP>(p, cur, n, gpr, wave, term_e, term_g);
      wg_drain_and_barrier();      // the new one is complete (and every wave has read the claim)
    }
    if (have_nxt_io) walk_plan_after(walk, following, via_pool, wave, lane, claim);
  }
  return true;
}

template <int NKS, int QP>
__global__ __launch_bounds__(64 * WG_WAVES) void k_switch_mfma_res(LaunchPlan p, Terms t, const Terms* t_dev, int r) {
  __shared__ int32_t s_e[kMaxTerms];
  __shared__ float s_coeff[kMaxTerms];
  const int lane = threadIdx.x & 63;
  const int wave = uniform(int(threadIdx.x >> 6));
  int n_terms;
  LSW_LOAD_TERMS(t, t_dev, s_e, s_coeff, n_terms);
  if (n_terms == 0) return;             // nothing to merge or unmerge (device-built lists only): W stays untouched
  __syncthreads();

  const int n = lane & 31, h = lane >> 5;
  const int gpr = r >> 3;
  const int n_groups = n_terms * gpr;
  int term_e[NKS], term_g[NKS];
  float term_c[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const int G = 2 * ks + h;
    const bool valid = G < n_groups;
    const int c = valid ? G / gpr : 0;
    term_e[ks] = s_e[c];
    term_g[ks] = valid ? G - c * gpr : 0;
    term_c[ks] = valid ? s_coeff[c] : 0.0f;
  }

  // XCD x (workgroups x, x + 8, ...: the hardware deals workgroups round-robin) owns items [x * per, (x + 1) * per)
  ItemWalk walk;
  const int item0 = walk_init(p, true, walk);
  if (item0 >= walk.static_end) return; // uniform over the workgroup (never with a pool)
  ResItem cur, nxt;
  res_item_at(p, item0, cur);
  nxt = cur;
  bool have_nxt = item0 + walk.step < walk.static_end;
  int claim = 0;
  if (have_nxt) {
    res_item_at(p, item0 + walk.step, nxt);
    walk_plan_after(walk, nxt.item, false, wave, lane, claim);
  }
  u32x4 p_hi[NKS], p_lo[NKS];
  {
    float braw[NKS][8];
    res_load_b<NKS, QP>(cur, wave, n, r, term_e, term_g, braw);
    res_make_p<NKS>(cur, wave, n, term_c, braw, p_hi, p_lo);
  }
  int cs = cur.col0;
  uint32_t lane_off = kOutOfRange;
  {
    const int col = cs + 8 * n;
    const uint32_t stride = uint32_t(cur.in) * 2u;
    if (col < min(cur.in, cur.col0 + p.tile_cols))
      lane_off = uint32_t(cur.row0 + 32 * wave + 4 * h) * stride + uint32_t(col) * 2u;
  }
  u32x4 wa[16], wb[16];
  {
    const __amdgpu_buffer_rsrc_t res = w_resource(cur.Wsrc, cur.out * cur.in * 2);
#pragma unroll
    for (int v = 0; v < 16; ++v)
      wa[v] = __builtin_amdgcn_raw_buffer_load_b128(
          res, lane_off + uint32_t(8 * (v >> 2) + (v & 3)) * (uint32_t(cur.in) * 2u), 0, kWLoadAux);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) wb[v] = u32x4{0u, 0u, 0u, 0u};
  res_fetch_q<NKS, QP>(p, cur, n, gpr, wave, term_e, term_g);
  wg_drain_and_barrier();
  __amdgpu_buffer_rsrc_t prev_res = w_resource(cur.W, cur.out * cur.in * 2);
  uint32_t prev_off = kOutOfRange, prev_stride = 0;

  bool a_is_cur = true;
  while (true) {
    if (!res_step<NKS, QP>(p, n, h, lane, wave, gpr, r, term_e, term_g, term_c, cur, nxt, have_nxt, walk, claim, cs, lane_off,
                           prev_res, prev_off, prev_stride, p_hi, p_lo, wa, wb)) { a_is_cur = true; break; }
    if (!res_step<NKS, QP>(p, n, h, lane, wave, gpr, r, term_e, term_g, term_c, cur, nxt, have_nxt, walk, claim, cs, lane_off,
                           prev_res, prev_off, prev_stride, p_hi, p_lo, wb, wa)) { a_is_cur = false; break; }
  }
  if (a_is_cur) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
      __builtin_amdgcn_raw_buffer_store_b128(
          wa[v], prev_res, prev_off + uint32_t(8 * (v >> 2) + (v & 3)) * prev_stride, 0, kWStoreAux);
  } else {
#pragma unroll
    for (int v = 0; v < 16; ++v)
      __builtin_amdgcn_raw_buffer_store_b128(
          wb[v], prev_res, prev_off + uint32_t(8 * (v >> 2) + (v & 3)) * prev_stride, 0, kWStoreAux);
  }
  walk_finish(walk);
}

template <int NKS, int QP>
static hipError_t launch_res(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int grid, hipStream_t s) {
  const size_t lds = size_t(p.tile_cols / MT_STEP) * NKS * 8 * QP * 64 * sizeof(u32x4);     // 8 KB per column step, k-step and Q part
  if (lds > size_t(kResidentLdsBytes) || p.Z != nullptr) return hipErrorInvalidValue;
  // once per process (function-local statics are initialised exactly once, also under concurrent first calls)
  static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_switch_mfma_res<NKS, QP>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kResidentLdsBytes);
  if (lds_ok != hipSuccess) return lds_ok;
  hipLaunchKernelGGL((k_switch_mfma_res<NKS, QP>), dim3(grid), dim3(64 * WG_WAVES), lds, s, p, t, t_dev, r);
  return hipGetLastError();
}

template <int QP>
static hipError_t launch_res_qp(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int grid, hipStream_t s) {
  const int n_groups = t.n * (r / 8);
  switch ((n_groups + 1) / 2) {
    case 1: return launch_res<1, QP>(p, t, t_dev, r, grid, s);
    case 2: return launch_res<2, QP>(p, t, t_dev, r, grid, s);
    case 3: return launch_res<3, QP>(p, t, t_dev, r, grid, s);
    case 4: return launch_res<4, QP>(p, t, t_dev, r, grid, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_switch_mfma_res(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int qp, int grid, hipStream_t s) {
  return qp == 2 ? launch_res_qp<2>(p, t, t_dev, r, grid, s) : launch_res_qp<1>(p, t, t_dev, r, grid, s);
}

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
  const int first_item = p.xcd_remap ? xcd_contiguous_block(blockIdx.x, grid) : int(blockIdx.x);
  int buf = 0;
  for (int item = first_item; item < p.n_items; item += grid) {       // uniform over the workgroup
    const bool adapter = p.Z != nullptr;
    LinDesc L;
    int local = item;
    if (adapter) {
      L = p.one;
    } else {
      const int seg = uniform(find_segment(p.first, p.n_sel, item));
      const LinDesc* Lp = p.lin + uniform(p.sel[seg]);
      L.W = uniform(Lp->W);
      L.B = uniform(Lp->B);
      L.Apk = uniform(Lp->Apk);
      L.Wbase = p.from_base ? uniform(Lp->Wbase) : nullptr;
      L.out = uniform(Lp->out);
      L.in = uniform(Lp->in);
      local = uniform(item - p.first[seg]);
    }
    const void* B = L.B;
    const int out = L.out, in = L.in;
    int row0, col0;
    decode_item(local, out, in, kMfmaTileRows, p.tile_cols, 0, &row0, &col0);
    row0 += 32 * wave;
    const int col_end = min(in, col0 + p.tile_cols);
    const int ncb = ceil_div(in, MT_STEP);
    w.W = L.W;
    w.Wsrc = p.from_base ? L.Wbase : w.W;
    w.wbytes = out * in * 2;
    w.stride = uint32_t(in) * 2u;
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
          if (adapter) load8<2>(p.Z, (long long)prow * p.z_stride + 8 * s_eg[G], b);
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

// ---------------------------------------------------------------------------
// Device-resident routing (Alg. 1 step 1 and steps 2-3 without a trip to the host).
//
// k_route: G = Softmax(TopK(logits)) on one wave.  k selection passes; in each, every lane scans its
// share of the logits for the largest one not yet taken (equal logits: the lower index; +0 == -0) and a
// butterfly over the lanes picks the wave's winner.  The softmax runs over the k winners in double
// precision and is rounded once to fp32, as the host router does.  A NaN logit raises the sticky error
// word and yields ids of -1, which the term builder rejects.
//
// k_build_terms: the signed coefficient list of one switch from device-resident (ids, gates) lists,
// with the host routine's arithmetic (no fused multiply-add) and its checks.  A bad list raises the
// sticky error word and leaves an empty list, which makes the switch kernels return at once.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_route(const float* __restrict__ logits, int E, int k, int32_t* __restrict__ ids,
                                              float* __restrict__ gates, int32_t* __restrict__ err) {
  const int lane = threadIdx.x;
  logits += (long long)blockIdx.x * E;       // one workgroup per token
  ids += (long long)blockIdx.x * k;
  gates += (long long)blockIdx.x * k;
  bool nan = false;
  for (int i = lane; i < E; i += 64) nan |= (logits[i] != logits[i]);
  if (__any(nan)) {
    if (lane == 0) atomicOr(err, 1);
    if (lane < k) { ids[lane] = -1; gates[lane] = 0.0f; }
    return;
  }
  int chosen[LSW_MAX_K];
  float chosen_v[LSW_MAX_K];
#pragma unroll
  for (int c = 0; c < LSW_MAX_K; ++c) { chosen[c] = -1; chosen_v[c] = 0.0f; }
#pragma unroll
  for (int c = 0; c < LSW_MAX_K; ++c) {
    if (c < k) {
      int best = -1;
      float best_v = 0.0f;
      for (int i = lane; i < E; i += 64) {
        bool taken = false;
#pragma unroll
        for (int d = 0; d < LSW_MAX_K; ++d) taken |= (chosen[d] == i);
        const float v = logits[i];
        if (!taken && (best < 0 || v > best_v)) { best = i; best_v = v; }      // ascending i: `>` keeps the lower index
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const int o = __shfl_xor(best, off, 64);
        const float ov = __shfl_xor(best_v, off, 64);
        if (o >= 0 && (best < 0 || ov > best_v || (ov == best_v && o < best))) { best = o; best_v = ov; }
      }
      chosen[c] = best;
      chosen_v[c] = best_v;
    }
  }
  if (lane == 0) {
    const double top = double(chosen_v[0]);
    double ex[LSW_MAX_K], sum = 0.0;
#pragma unroll
    for (int c = 0; c < LSW_MAX_K; ++c) {
      ex[c] = c < k ? exp(double(chosen_v[c]) - top) : 0.0;
      sum += ex[c];
    }
#pragma unroll
    for (int c = 0; c < LSW_MAX_K; ++c)
      if (c < k) { ids[c] = chosen[c]; gates[c] = float(ex[c] / sum); }
  }
}

hipError_t launch_route(const float* logits, int n_tokens, int E, int k, int32_t* ids, float* gates, int32_t* err, hipStream_t s) {
  hipLaunchKernelGGL(k_route, dim3(n_tokens), dim3(64), 0, s, logits, E, k, ids, gates, err);
  return hipGetLastError();
}

__global__ __launch_bounds__(64) void k_build_terms(const int32_t* __restrict__ old_ids, const float* __restrict__ old_gates, int k_old,
                                                    const int32_t* __restrict__ new_ids, const float* __restrict__ new_gates, int k_new,
                                                    int E, float scale, Terms* __restrict__ out, int32_t* __restrict__ err) {
  if (threadIdx.x != 0) return;
  Terms t;
  t.n = 0;
  for (int i = 0; i < kMaxTerms; ++i) { t.e[i] = 0; t.coeff[i] = 0.0f; }
  bool ok = true;
  auto check = [&](const int32_t* ids, const float* gates, int k) {
    for (int a = 0; a < k; ++a) {
      const float g = gates[a];
      ok &= (ids[a] >= 0 && ids[a] < E) && (g - g == 0.0f);           // in range, finite
      for (int b = 0; b < a; ++b) ok &= (ids[b] != ids[a]);
    }
  };
  check(old_ids, old_gates, k_old);
  check(new_ids, new_gates, k_new);
  if (ok) {
    for (int a = 0; a < k_new; ++a) {
      float coeff = __fmul_rn(scale, new_gates[a]);
      for (int b = 0; b < k_old; ++b)
        if (old_ids[b] == new_ids[a]) coeff = __fsub_rn(__fmul_rn(scale, new_gates[a]), __fmul_rn(scale, old_gates[b]));
      if (coeff != 0.0f) { t.e[t.n] = new_ids[a]; t.coeff[t.n] = coeff; ++t.n; }
    }
    for (int b = 0; b < k_old; ++b) {
      bool also_new = false;
      for (int a = 0; a < k_new; ++a) also_new |= (new_ids[a] == old_ids[b]);
      if (also_new) continue;
      const float coeff = -__fmul_rn(scale, old_gates[b]);
      if (coeff != 0.0f) { t.e[t.n] = old_ids[b]; t.coeff[t.n] = coeff; ++t.n; }
    }
  } else {
    atomicOr(err, 2);
  }
  *out = t;
}

hipError_t launch_build_terms(const int32_t* old_ids, const float* old_gates, int k_old, const int32_t* new_ids,
                              const float* new_gates, int k_new, int E, float scale, Terms* out, int32_t* err, hipStream_t s) {
  hipLaunchKernelGGL(k_build_terms, dim3(1), dim3(64), 0, s, old_ids, old_gates, k_old, new_ids, new_gates, k_new, E, scale, out, err);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Un-merged adapter path for many tokens (Eq. 2: y = f(x) + sum_i G(x1)_i E_i(x), E_i(x) = W_up (W_down x)).
//
// Three launches per linear.  (1) k_adapter_down: U = X A_all^T on the matrix cores, all E*r down-projection rows of
// all experts at once (N = E*r is at most 256, so computing the unselected experts too costs nothing next to the
// traffic), the long contraction over `in` cut into slices whose partial sums go to Upart[slice][T][N].
// (2) k_adapter_gate: Z[t][e*r+rho] = scale * g(t,e) * sum_slices Upart (zero for experts token t did not select):
// the gather of the token's experts is a multiplication by a mostly-zero gate table.  (3) the matrix-core switch
// kernels in adapter mode: Y[T,out] <- rne(Y + Z B_all^T), rows = tokens, the row operand read from Z, the shared
// operand B^T packed like A (k_pack_A, transposed source).
//
// k_adapter_down.  A workgroup is 32 tokens x one slice of `in`, its four waves sharing the slice.  X is bf16 and needs no split; A is
// split into bf16 high + low (two passes).  The contraction index inside a 64-column chunk u is laid out so that a
// lane reads 64 contiguous bytes of its token's row: k-step s (0..3), lane half h, element i  <->  column
// 64u + 32h + 8s + i.  The A operand comes from a re-laid-out copy built once (k_pack_Atk):
//   Atk bf16 [N/32 blocks][in/64 chunks][4 k-steps][parts][64 lanes][8]
// holding for lane (h, n) the 8 values A_all[32*block + n][64u + 32h + 8s + i]: one operand load of a wave is 1 KB
// contiguous.  Rows of A_all past E*r and columns past `in` hold zeros.
// ---------------------------------------------------------------------------
constexpr int AD_CHUNK = 64;        // columns of `in` per chunk (4 k-steps of 16)

// 32-row blocks of A_all the layout holds: more than 4 are rounded up to 8 (the kernel takes them in two groups of 4)
__host__ __device__ static inline int adapter_blocks_dev(int N) { const int nb = ceil_div(N, 32); return nb > 4 ? 8 : nb; }
static int adapter_blocks(int N) { return adapter_blocks_dev(N); }

int64_t adapter_atk_elems(int E, int r, int in, int qp) {
  return int64_t(adapter_blocks(E * r)) * ceil_div(in, AD_CHUNK) * 4 * qp * 64 * 8;
}

// 64-column chunks one workgroup (4 waves, chunks dealt round-robin to the waves) contracts: about 512 workgroups per
// launch, at least 4 chunks each (one per wave) unless the matrix has fewer
static int adapter_chunks_per_slice(int T, int in) {
  const int nch = ceil_div(in, AD_CHUNK);
  const long long tiles = ceil_div(T, 32);
  const long long cps = std::max<long long>(4, (nch * tiles + 511) / 512);
  return int(std::min<long long>(nch, cps));
}

int adapter_slices(int T, int in) { return ceil_div(ceil_div(in, AD_CHUNK), adapter_chunks_per_slice(T, in)); }

template <int QP>
__global__ __launch_bounds__(256) void k_pack_Atk(const void* __restrict__ A, uint16_t* __restrict__ Atk, int N, int in) {
  const int nb_count = adapter_blocks_dev(N), nch = ceil_div(in, AD_CHUNK);
  const long long total = (long long)nb_count * nch * 4 * 64;
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long long)gridDim.x * blockDim.x) {
    const int lane = int(idx & 63), s4 = int((idx >> 6) & 3);
    const long long bu = idx >> 8;
    const int u = int(bu % nch), nb = int(bu / nch);
    const int row = 32 * nb + (lane & 31), j = AD_CHUNK * u + 32 * (lane >> 5) + 8 * s4;
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (row < N && j < in) ? load1<QP>(A, (long long)row * in + j + i) : 0.0f;   // in % 8 == 0: all 8 or none
    u32x4 hi, lo;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint32_t hh, ll;
      split2(x[2 * q], x[2 * q + 1], &hh, &ll);
      hi[q] = hh;
      lo[q] = ll;
    }
    const long long base = (((long long)(nb * nch + u) * 4 + s4) * QP * 64 + lane) * 8;
    *reinterpret_cast<u32x4*>(Atk + base) = hi;
    if constexpr (QP == 2) *reinterpret_cast<u32x4*>(Atk + base + 64 * 8) = lo;
  }
}

hipError_t launch_pack_Atk(const void* A, uint16_t* Atk, int E, int r, int in, int qp, hipStream_t s) {
  const long long total = (long long)adapter_blocks(E * r) * ceil_div(in, AD_CHUNK) * 4 * 64;
  const int grid = int(std::min<long long>((total + 255) / 256, 1 << 16));
  if (qp == 2) hipLaunchKernelGGL(k_pack_Atk<2>, dim3(grid), dim3(256), 0, s, A, Atk, E * r, in);
  else hipLaunchKernelGGL(k_pack_Atk<1>, dim3(grid), dim3(256), 0, s, A, Atk, E * r, in);
  return hipGetLastError();
}

template <int NB, int QP>
struct AdChunk {            // the operands of one 64-column chunk: this lane's 64 bytes of X and its pieces of A
  u32x4 xp[4];
  u32x4 qv[NB][4][QP];
};

template <int NB, int QP>
__device__ __forceinline__ void ad_load_chunk(AdChunk<NB, QP>& c, __amdgpu_buffer_rsrc_t xres, uint32_t row_off, int in, int nch,
                                              int u, int h, const LSW_GLOBAL u32x4* q0) {
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4) {
    const int j = AD_CHUNK * u + 32 * h + 8 * s4;
    c.xp[s4] = __builtin_amdgcn_raw_buffer_load_b128(xres, (u < nch && j < in) ? row_off + uint32_t(j) * 2u : kOutOfRange, 0, 0);
  }
  const int uq = min(u, nch - 1);       // past the last chunk: X reads zeros, A re-reads a valid chunk
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const LSW_GLOBAL u32x4* q = q0 + ((long long)(nb * nch + uq) * 4) * QP * 64;      // q0 is block 0 of this workgroup's group
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
      for (int hl = 0; hl < QP; ++hl) c.qv[nb][s4][hl] = q[(s4 * QP + hl) * 64];
  }
}

template <int NB, int QP>
__device__ __forceinline__ void ad_compute_chunk(const AdChunk<NB, QP>& c, f32x16 (&acc)[NB]) {
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
      for (int hl = QP - 1; hl >= 0; --hl)       // the small (low-part) products first
        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, c.xp[s4]),
                                                          __builtin_bit_cast(bf16x8, c.qv[nb][s4][hl]), acc[nb], 0, 0, 0);
}

// A workgroup = 32 tokens x one slice of `in` (cps chunks); its 4 waves take the chunks u0 + w, u0 + w + 4, ... with the
// operands of the next chunk requested before the current one is multiplied, then add their accumulators through LDS.
template <int NB, int QP>
__global__ __launch_bounds__(256) void k_adapter_down(const uint16_t* __restrict__ X, const uint16_t* __restrict__ Atk,
                                                      float* __restrict__ Upart, int T, int in, int N, int cps) {
  __shared__ float red[3][NB][16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, h = lane >> 5;
  const int tile = blockIdx.x, slice = blockIdx.y;
  const int nch = ceil_div(in, AD_CHUNK);
  const int u0 = slice * cps, u1 = min(nch, u0 + cps);
  // X through a buffer resource: token rows past T lie outside it and read as zeros
  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(X), 0, T * in * 2, 0x00020000);
  const uint32_t row_off = uint32_t(32 * tile + n) * uint32_t(in) * 2u;
  f32x16 acc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[nb][v] = 0.0f;
  const int nb0 = blockIdx.z * NB;       // N above 128: the 32-column blocks are split over blockIdx.z
  const LSW_GLOBAL u32x4* q0 = (const LSW_GLOBAL u32x4*)Atk + (long long)nb0 * nch * 4 * QP * 64 + lane;
  AdChunk<NB, QP> ca, cb;
  int u = u0 + wave;
  if (u < u1) ad_load_chunk<NB, QP>(ca, xres, row_off, in, nch, u, h, q0);
  while (u < u1) {                       // two chunks per trip: one in flight while the other is multiplied
    if (u + 4 < u1) ad_load_chunk<NB, QP>(cb, xres, row_off, in, nch, u + 4, h, q0);
    ad_compute_chunk<NB, QP>(ca, acc);
    u += 4;
    if (u >= u1) break;
    if (u + 4 < u1) ad_load_chunk<NB, QP>(ca, xres, row_off, in, nch, u + 4, h, q0);
    ad_compute_chunk<NB, QP>(cb, acc);
    u += 4;
  }
  if (wave > 0) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[wave - 1][nb][v][lane] = acc[nb][v];
  }
  __syncthreads();
  if (wave > 0) return;
  // acc[nb][v] is U[token 32*tile + 8*(v/4) + 4h + v%4][column 32*nb + n]
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int col = 32 * (nb0 + nb) + n;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int t = 32 * tile + 8 * (v >> 2) + 4 * h + (v & 3);
      const float sum = ((acc[nb][v] + red[0][nb][v][lane]) + red[1][nb][v][lane]) + red[2][nb][v][lane];
      if (t < T && col < N) Upart[((long long)slice * T + t) * N + col] = sum;
    }
  }
}

hipError_t launch_adapter_down(const uint16_t* X, const uint16_t* Atk, float* Upart, int T, int in, int N, int qp, hipStream_t s) {
  const int cps = adapter_chunks_per_slice(T, in);
  const int nb = ceil_div(N, 32);
  const dim3 grid(ceil_div(T, 32), adapter_slices(T, in), nb > 4 ? 2 : 1);
#define LSW_AD(NB_)                                                                                              \
  do {                                                                                                           \
    if (qp == 2) hipLaunchKernelGGL((k_adapter_down<NB_, 2>), grid, dim3(256), 0, s, X, Atk, Upart, T, in, N, cps); \
    else hipLaunchKernelGGL((k_adapter_down<NB_, 1>), grid, dim3(256), 0, s, X, Atk, Upart, T, in, N, cps);         \
  } while (0)
  if (nb <= 1) LSW_AD(1);
  else if (nb <= 2) LSW_AD(2);
  else if (nb <= 8) LSW_AD(4);            // 5..8 blocks: two groups of 4 (the packed layout is padded to whole groups)
  else return hipErrorInvalidValue;
#undef LSW_AD
  return hipGetLastError();
}

// Z[t][col] = scale * g(t, expert of col) * sum over the slices of Upart[.][t][col]; columns N..z_stride-1 are zeroed.
// A token's list is checked as the switch's lists are: an id outside [0, E), a duplicate id or a non-finite gate
// raises the sticky error word (flag 2) and gives that token an all-zero row (its output stays what it was).
__global__ __launch_bounds__(256) void k_adapter_gate(const float* __restrict__ Upart, int n_slices, const int32_t* __restrict__ ids,
                                                      const float* __restrict__ gates, int k, int T, int E, int r, float scale,
                                                      float* __restrict__ Z, int z_stride, int32_t* __restrict__ err) {
  const int N = E * r;
  const long long total = (long long)T * z_stride;
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long long)gridDim.x * blockDim.x) {
    const int t = int(idx / z_stride), col = int(idx - (long long)t * z_stride);
    float z = 0.0f;
    if (col < N) {
      const int e = col / r;
      bool ok = true;
      float coeff = 0.0f;
      for (int c = 0; c < k; ++c) {
        const int id = ids[(long long)t * k + c];
        const float g = gates[(long long)t * k + c];
        ok &= (id >= 0 && id < E) && (g - g == 0.0f);
        for (int d = 0; d < c; ++d) ok &= (ids[(long long)t * k + d] != id);
        if (id == e) coeff = __fmul_rn(scale, g);
      }
      if (!ok) {
        if (col == 0) atomicOr(err, 2);
      } else if (coeff != 0.0f) {
        float u = 0.0f;
        for (int s = 0; s < n_slices; ++s) u += Upart[((long long)s * T + t) * N + col];
        z = coeff * u;
      }
    }
    Z[idx] = z;
  }
}

hipError_t launch_adapter_gate(const float* Upart, int n_slices, const int32_t* ids, const float* gates, int k, int T, int E, int r,
                               float scale, float* Z, int z_stride, int32_t* err, hipStream_t s) {
  const long long total = (long long)T * z_stride;
  const int grid = int(std::min<long long>((total + 255) / 256, 1 << 16));
  hipLaunchKernelGGL(k_adapter_gate, dim3(grid), dim3(256), 0, s, Upart, n_slices, ids, gates, k, T, E, r, scale, Z, z_stride, err);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Bandwidth probe: the switch kernel's W traffic and nothing else.  A persistent grid of
// single-wave workgroups walks 32-row x tile_cols items in 32 x 256 steps (the same 512-byte row
// segments, non-temporal 16-byte accesses and one-step-ahead requests as the switch), widens each
// bf16 to fp32, adds +0.0f, rounds back and stores in place: every finite value is unchanged (a
// negative zero becomes +0).  What this sustains is the ceiling of the in-place access pattern on
// the given matrices, without factor traffic or matrix work.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_probe_inplace(LaunchPlan p) {
  const int lane = threadIdx.x, n = lane & 31, h = lane >> 5;
  const int grid = gridDim.x;
  const int first_item = p.xcd_remap ? xcd_contiguous_block(blockIdx.x, grid) : int(blockIdx.x);
  for (int item = first_item; item < p.n_items; item += grid) {
    const int seg = uniform(find_segment(p.first, p.n_sel, item));
    const LinDesc* Lp = p.lin + uniform(p.sel[seg]);
    const int out = uniform(Lp->out), in = uniform(Lp->in);
    int row0, col0;
    decode_item(uniform(item - p.first[seg]), out, in, 32, p.tile_cols, 0, &row0, &col0);
    const int col_end = min(in, col0 + p.tile_cols);
    const __amdgpu_buffer_rsrc_t res = w_resource(uniform(Lp->W), out * in * 2);
    const uint32_t stride = uint32_t(in) * 2u;
    auto offset = [&](int cs) {
      const int col = cs + 8 * n;
      return col < col_end ? uint32_t(row0 + 4 * h) * stride + uint32_t(col) * 2u : kOutOfRange;
    };
    u32x4 buf[2][16];
    uint32_t off[2];
    off[0] = offset(col0);
#pragma unroll
    for (int v = 0; v < 16; ++v)
      buf[0][v] = __builtin_amdgcn_raw_buffer_load_b128(res, off[0] + uint32_t(8 * (v >> 2) + (v & 3)) * stride, 0, 2);
    for (int cs = col0; cs < col_end; cs += 2 * MT_STEP) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int c = cs + half * MT_STEP;
        if (c < col_end) {
          off[half ^ 1] = (c + MT_STEP < col_end) ? offset(c + MT_STEP) : kOutOfRange;
#pragma unroll
          for (int v = 0; v < 16; ++v)
            buf[half ^ 1][v] = __builtin_amdgcn_raw_buffer_load_b128(
                res, off[half ^ 1] + uint32_t(8 * (v >> 2) + (v & 3)) * stride, 0, 2);
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            u32x4 o;
#pragma unroll
            for (int q = 0; q < 4; ++q)
              o[q] = pack_bf16(bf16_lo(buf[half][v][q]) + 0.0f, bf16_hi(buf[half][v][q]) + 0.0f);
            __builtin_amdgcn_raw_buffer_store_b128(o, res, off[half] + uint32_t(8 * (v >> 2) + (v & 3)) * stride, 0, kWStoreAux);
          }
        }
      }
    }
  }
}

hipError_t launch_probe_inplace(const LaunchPlan& p, int grid, hipStream_t s) {
  hipLaunchKernelGGL(k_probe_inplace, dim3(grid), dim3(64), 0, s, p);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Merged decode (Eq. 3): y = W x with the merged weights, bf16 inputs, fp32 accumulation.
// HBM-bound: every weight is read once (2 bytes per weight), x comes from L1/L2.
//
// A wave owns GV_ROWS consecutive rows of one linear and walks them in steps of 512 columns: per step
// one 16-byte non-temporal load per row and lane (the 64 lanes of a load cover 1 KB of one row) and one
// 16-byte load of x shared by the rows.  Two column steps are requested before the first is used, so a
// wave keeps 2 * GV_ROWS KB of W in flight.  A workgroup is 4 waves on consecutive row blocks, so
// they read the same x at about the same time.  The lanes' partial sums meet in a butterfly of
// cross-lane adds; lane 0 writes the GV_ROWS results.
// ---------------------------------------------------------------------------
constexpr int GV_ROWS = kGemvRows;

__device__ __forceinline__ float gv_dot8(const u32x4 w, const u32x4 x, float acc) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    acc = fmaf(bf16_lo(w[q]), bf16_lo(x[q]), acc);
    acc = fmaf(bf16_hi(w[q]), bf16_hi(x[q]), acc);
  }
  return acc;
}

// rows row0 .. row0+GV_ROWS-1 of W (rows past `out` are clamped for the loads and not written)
__device__ __forceinline__ void gv_rows(const uint16_t* W, const uint16_t* x, float* y, int out, int in, int row0, int lane) {
  const LSW_GLOBAL u32x4* wrow[GV_ROWS];
#pragma unroll
  for (int m = 0; m < GV_ROWS; ++m)
    wrow[m] = as_global(reinterpret_cast<const u32x4*>(W + (long long)min(row0 + m, out - 1) * in));
  const LSW_GLOBAL u32x4* xv = as_global(reinterpret_cast<const u32x4*>(x));
  float acc[GV_ROWS];
#pragma unroll
  for (int m = 0; m < GV_ROWS; ++m) acc[m] = 0.0f;
  const int nvec = in >> 3;                     // 16-byte vectors per row
  int j = lane;
  for (; j + 64 < nvec; j += 128) {             // two column steps per trip
    u32x4 w0[GV_ROWS], w1[GV_ROWS];
#pragma unroll
    for (int m = 0; m < GV_ROWS; ++m) w0[m] = __builtin_nontemporal_load(wrow[m] + j);
#pragma unroll
    for (int m = 0; m < GV_ROWS; ++m) w1[m] = __builtin_nontemporal_load(wrow[m] + j + 64);
    const u32x4 x0 = xv[j], x1 = xv[j + 64];
#pragma unroll
    for (int m = 0; m < GV_ROWS; ++m) acc[m] = gv_dot8(w0[m], x0, acc[m]);
#pragma unroll
    for (int m = 0; m < GV_ROWS; ++m) acc[m] = gv_dot8(w1[m], x1, acc[m]);
  }
  if (j < nvec) {                               // one ragged step is left
    const u32x4 x0 = xv[j];
#pragma unroll
    for (int m = 0; m < GV_ROWS; ++m) acc[m] = gv_dot8(__builtin_nontemporal_load(wrow[m] + j), x0, acc[m]);
  }
#pragma unroll
  for (int m = 0; m < GV_ROWS; ++m) {
    float v = acc[m];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0 && row0 + m < out) y[row0 + m] = v;
  }
}

// one linear
__global__ __launch_bounds__(256) void k_gemv(const uint16_t* __restrict__ W, const uint16_t* __restrict__ x,
                                              float* __restrict__ y, int out, int in) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_blocks = ceil_div(out, GV_ROWS);
  for (int rb = blockIdx.x * 4 + wave; rb < n_blocks; rb += gridDim.x * 4)
    gv_rows(W, x, y, out, in, rb * GV_ROWS, lane);
}

hipError_t launch_gemv(const uint16_t* W, const uint16_t* x, float* y, int out, int in, int grid_cap, hipStream_t s) {
  const int grid = std::max(1, std::min(ceil_div(ceil_div(out, GV_ROWS), 4), grid_cap));
  hipLaunchKernelGGL(k_gemv, dim3(grid), dim3(256), 0, s, W, x, y, out, in);
  return hipGetLastError();
}

// every selected linear in one launch: an item is a block of GV_ROWS rows of one linear (plan tile = GV_ROWS x
// whole row); x_all / y_all hold the linears' inputs / outputs back to back in registration order
__global__ __launch_bounds__(256) void k_gemv_all(LaunchPlan p, const uint16_t* __restrict__ x_all, float* __restrict__ y_all) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int vb = p.xcd_remap ? xcd_contiguous_block(blockIdx.x, gridDim.x) : int(blockIdx.x);
  for (int item = vb * 4 + wave; item < p.n_items; item += gridDim.x * 4) {
    const int seg = uniform(find_segment(p.first, p.n_sel, uniform(item)));
    const LinDesc* Lp = p.lin + uniform(p.sel[seg]);
    const int out = uniform(Lp->out), in = uniform(Lp->in);
    const int row0 = uniform(item - p.first[seg]) * GV_ROWS;
    gv_rows(uniform(Lp->W), x_all + Lp->x_off, y_all + Lp->y_off, out, in, row0, lane);
  }
}

hipError_t launch_gemv_all(const LaunchPlan& p, const uint16_t* x_all, float* y_all, int grid, hipStream_t s) {
  hipLaunchKernelGGL(k_gemv_all, dim3(grid), dim3(256), 0, s, p, x_all, y_all);
  return hipGetLastError();
}

}  // namespace lsw
