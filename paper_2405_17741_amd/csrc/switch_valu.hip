// liblsw device code (gfx950): the fused adapter switch on the fp32 vector ALU (any rank).
#include "lsw_device.h"

namespace lsw {

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
          u32x4* ptr = reinterpret_cast<u32x4*>(L.W + (long long)row * L.ld + col);
          const u32x4 w = __builtin_nontemporal_load(
              p.from_base ? reinterpret_cast<const u32x4*>(L.Wbase + (long long)row * L.ld + col) : ptr);
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

}  // namespace lsw
