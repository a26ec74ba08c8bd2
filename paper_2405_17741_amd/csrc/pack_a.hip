// liblsw device code (gfx950): re-layout of the LoRA down-projection factors for the matrix-core kernels.
#include "lsw_device.h"

namespace lsw {

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

}  // namespace lsw
