// liblsw device code (gfx950): the device-side router and term-list builder.
#include "lsw_device.h"

namespace lsw {

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

}  // namespace lsw
