// liblsw device code (gfx950): what the inner loop of the chunked matrix-core switch sustains with nothing around it.
#include "lsw_device.h"
#include "lsw_mfma.h"

namespace lsw {

// ---------------------------------------------------------------------------
// The chunk loop of k_switch_mfma_bigk in isolation: per group 4 LDS reads of the shared operand and 6 matrix
// instructions (v_mfma_f32_32x32x16_bf16: low x high, high x low, high x high for two blocks), 16 groups per chunk,
// 8 accumulators, the row operand of 16 k-steps in registers, 4 waves per workgroup, one workgroup per CU.  No weight
// traffic, no barriers.  COPIES per group: LDS-DMA copies of 1 KB riding along (the kernel issues 2 per group in the
// first half of a chunk).  The matrix pipe needs 6 x 32 = 192 cycles per group; how many nanoseconds a group takes here
// is the clock the chip holds under this load, i.e. the ceiling of the three-pass kernel whatever its memory schedule.
// ---------------------------------------------------------------------------
template <int COPIES>
__global__ __launch_bounds__(256) void k_probe_matrix_loop(u32x4* out, const u32x4* pin, int iters, const u32x4* qsrc, int zero_operands) {
  constexpr int NP = 16;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < 4096; i += 256) {          // 64 KB of operand data: bf16 values near 1 with varied mantissas, or zeros
    const uint32_t s = uint32_t(i) * 2654435761u;
    wg_lds[i] = zero_operands ? u32x4{0u, 0u, 0u, 0u}
                              : u32x4{(s & 0x0fff0fffu) | 0x3c003c00u, ((s * 3) & 0x0fff0fffu) | 0x3c003c00u,
                                      ((s * 5) & 0x0fff0fffu) | 0xbc003c00u, ((s * 7) & 0x0fff0fffu) | 0x3c00bc00u};
  }
  __syncthreads();
  const u32x4* qbuf = wg_lds + lane;
  f32x16 a0[4], a1[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) { a0[q][v] = 0.0f; a1[q][v] = 0.0f; }
  u32x4 p_hi[NP], p_lo[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    p_hi[i] = zero_operands ? u32x4{0u, 0u, 0u, 0u} : pin[i * 64 + lane];
    p_lo[i] = zero_operands ? u32x4{0u, 0u, 0u, 0u} : pin[(i + NP) * 64 + lane];
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int ch = 0; ch < NP / 4; ++ch) {
      u32x4 qr[2][2][2];
      auto fetch = [&](int idx) {
        const int q = idx / 4, kk = idx % 4;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int hl = 0; hl < 2; ++hl) qr[idx & 1][j][hl] = qbuf[((kk * 8 + 2 * q + j) * 2 + hl) * 64];
      };
      fetch(0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const int idx = q * 4 + kk;
          if (idx + 1 < 16) fetch(idx + 1);
          if constexpr (COPIES >= 1)
            lds_dma16(qsrc + ((it * 16 + idx) % 64) * 1024 + wave * 256 + (idx % 4) * 64 + lane,
                      reinterpret_cast<const u32x4*>(wg_lds) + 4096 + wave * 1024 + (idx % 16) * 64);
          if constexpr (COPIES >= 2)
            lds_dma16(qsrc + ((it * 16 + idx) % 64) * 1024 + 32768 + wave * 256 + (idx % 4) * 64 + lane,
                      reinterpret_cast<const u32x4*>(wg_lds) + 4096 + wave * 1024 + ((idx + 8) % 16) * 64);
          const bf16x8 ph = __builtin_bit_cast(bf16x8, p_hi[ch * 4 + kk]), pl = __builtin_bit_cast(bf16x8, p_lo[ch * 4 + kk]);
          const bf16x8 h0 = __builtin_bit_cast(bf16x8, qr[idx & 1][0][0]), l0 = __builtin_bit_cast(bf16x8, qr[idx & 1][0][1]);
          const bf16x8 h1 = __builtin_bit_cast(bf16x8, qr[idx & 1][1][0]), l1 = __builtin_bit_cast(bf16x8, qr[idx & 1][1][1]);
          a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl, h0, a0[q], 0, 0, 0);
          a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl, h1, a1[q], 0, 0, 0);
          a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, l0, a0[q], 0, 0, 0);
          a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, l1, a1[q], 0, 0, 0);
          a0[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, h0, a0[q], 0, 0, 0);
          a1[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph, h1, a1[q], 0, 0, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
  u32x4 acc = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int q = 0; q < 4; ++q) acc[q] = __float_as_uint(a0[q][q] + a1[q][15 - q]);
  __builtin_amdgcn_s_waitcnt(0x0F70);                 // the last copies have landed before the workgroup ends
  out[blockIdx.x * 256 + threadIdx.x] = acc;
}

// out: grid * 256 x 16 bytes; pin: 32 x 64 x 16 bytes of row-operand data; qsrc: 4 MiB the copies read (all DEVICE)
hipError_t launch_probe_matrix_loop(void* out, const void* pin, const void* qsrc, int grid, int iters, int copies, int zero_operands, hipStream_t s) {
  constexpr size_t lds = 131072;                      // 64 KB read by the loop + 64 KB the copies write into
  auto go = [&](auto kernel) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), lds, s, static_cast<u32x4*>(out), static_cast<const u32x4*>(pin), iters,
                       static_cast<const u32x4*>(qsrc), zero_operands);
    return hipGetLastError();
  };
  if (copies <= 0) return go(k_probe_matrix_loop<0>);
  if (copies == 1) return go(k_probe_matrix_loop<1>);
  return go(k_probe_matrix_loop<2>);
}

}  // namespace lsw
