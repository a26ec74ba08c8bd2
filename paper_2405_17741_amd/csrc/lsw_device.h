// Device-side helpers shared by the kernels of liblsw (gfx950 only): vector types, bf16 packing and the split into
// high + low parts, typed loads of the stored factors, LDS-DMA copies, the term-list loader.
#pragma once
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

}  // namespace lsw
