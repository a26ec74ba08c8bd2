// liblsw device code (gfx950): the merged-decode GEMVs.
#include "lsw_device.h"

namespace lsw {

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
__device__ __forceinline__ void gv_rows(const uint16_t* W, const uint16_t* x, float* y, int out, int in, int ld, int row0, int lane) {
  const LSW_GLOBAL u32x4* wrow[GV_ROWS];
#pragma unroll
  for (int m = 0; m < GV_ROWS; ++m)
    wrow[m] = as_global(reinterpret_cast<const u32x4*>(W + (long long)min(row0 + m, out - 1) * ld));
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
                                              float* __restrict__ y, int out, int in, int ld) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_blocks = ceil_div(out, GV_ROWS);
  for (int rb = blockIdx.x * 4 + wave; rb < n_blocks; rb += gridDim.x * 4)
    gv_rows(W, x, y, out, in, ld, rb * GV_ROWS, lane);
}

hipError_t launch_gemv(const uint16_t* W, const uint16_t* x, float* y, int out, int in, int ld, int grid_cap, hipStream_t s) {
  const int grid = std::max(1, std::min(ceil_div(ceil_div(out, GV_ROWS), 4), grid_cap));
  hipLaunchKernelGGL(k_gemv, dim3(grid), dim3(256), 0, s, W, x, y, out, in, ld);
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
    const int out = uniform(Lp->out), in = uniform(Lp->in), ld = uniform(Lp->ld);
    const int row0 = uniform(item - p.first[seg]) * GV_ROWS;
    gv_rows(uniform(Lp->W), x_all + Lp->x_off, y_all + Lp->y_off, out, in, ld, row0, lane);
  }
}

hipError_t launch_gemv_all(const LaunchPlan& p, const uint16_t* x_all, float* y_all, int grid, hipStream_t s) {
  hipLaunchKernelGGL(k_gemv_all, dim3(grid), dim3(256), 0, s, p, x_all, y_all);
  return hipGetLastError();
}

}  // namespace lsw
