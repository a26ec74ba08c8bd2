// liblsw device code (gfx950): the un-merged adapter path for prompts (down-projection, gate table).
#include "lsw_device.h"
#include "lsw_mfma.h"

#include <mutex>

namespace lsw {

// ---------------------------------------------------------------------------
// Workspace of lsw_adapter_forward_static: device memory that exists from the moment the library is loaded on a GPU
// until the process ends, so that the call needs no allocation and no workspace from its caller.  Each GPU holds its own
// copy at its own address; host code never uses the array's name as an address, only what hipGetSymbolAddress returned
// for the device that was current (looked up once per device, at lsw_enable_adapter_path).
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t adapter_static_scratch(int device, void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* table[kMaxDevices] = {};
  if (device < 0 || device >= kMaxDevices || !ptr) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> guard(mu);
  if (!table[device]) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return e;
    if (cur != device) return hipErrorInvalidDevice;      // the address belongs to the device that is current
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    table[device] = p;
  }
  *ptr = table[device];
  return hipSuccess;
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

// 32-row blocks of A_all the layout holds = the blocks the down-projection reads: 1, 2, 4 (3 is rounded up: the kernel
// exists for 1, 2 and 4 blocks per workgroup) or 8 (two groups of 4); the rows past E*r hold zeros
__host__ __device__ static inline int adapter_blocks_dev(int N) { const int nb = ceil_div(N, 32); return nb > 4 ? 8 : nb == 3 ? 4 : nb; }
static int adapter_blocks(int N) { return adapter_blocks_dev(N); }

int64_t adapter_atk_elems(int E, int r, int in, int qp) {
  return int64_t(adapter_blocks(E * r)) * ceil_div(in, AD_CHUNK) * 4 * qp * 64 * 8;
}

// 64-column chunks one workgroup (4 waves, chunks dealt round-robin to the waves) contracts: about 512 workgroups per
// launch, at least 4 chunks each (one per wave) unless the matrix has fewer
int adapter_chunks_per_slice(int T, int in) {
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
// One launch covers every linear of the call: workgroups jobs.first[i] .. jobs.first[i+1]-1 belong to linear i and are
// numbered (group of 4 row blocks, slice, token tile), the token tile fastest.
template <int NB, int QP>
__global__ __launch_bounds__(256) void k_adapter_down(AdJobs jobs, int N) {
  __shared__ float red[3][NB][16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, h = lane >> 5;
  const int job = uniform(find_segment(jobs.first, jobs.n, int(blockIdx.x)));
  const uint16_t* __restrict__ X = uniform(jobs.X[job]);
  const uint16_t* __restrict__ Atk = uniform(jobs.Atk[job]);
  float* __restrict__ Upart = uniform(jobs.Upart[job]);
  const int T = jobs.T, in = uniform(jobs.in[job]), cps = uniform(jobs.cps[job]), n_slices = uniform(jobs.n_slices[job]);
  const int n_tiles = ceil_div(T, 32);
  const int local = uniform(int(blockIdx.x) - jobs.first[job]);
  const int tile = local % n_tiles, slice = (local / n_tiles) % n_slices, zgroup = local / (n_tiles * n_slices);
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
  const int nb0 = zgroup * NB;           // N above 128: the 32-column blocks come in two groups of workgroups
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

hipError_t launch_adapter_down(const AdJobs& jobs_in, int N, int qp, hipStream_t s) {
  AdJobs jobs = jobs_in;
  const int nb = ceil_div(N, 32);
  const int zgroups = nb > 4 ? 2 : 1;
  const int nb_read = nb <= 1 ? 1 : nb <= 2 ? 2 : 4 * zgroups;       // blocks of Atk a workgroup row reads
  if (jobs.n < 1 || jobs.n > kAdMaxLin || nb > 8 || nb_read != adapter_blocks(N)) return hipErrorInvalidValue;   // never beyond what k_pack_Atk laid out
  long long total = 0;
  for (int i = 0; i < jobs.n; ++i) {
    jobs.first[i] = int(total);
    total += (long long)ceil_div(jobs.T, 32) * jobs.n_slices[i] * zgroups;
    if (total > INT32_MAX) return hipErrorInvalidValue;
  }
  for (int i = jobs.n; i <= kAdMaxLin; ++i) jobs.first[i] = int(total);
  const dim3 grid{unsigned(total)};
#define LSW_AD(NB_)                                                                                  \
  do {                                                                                               \
    if (qp == 2) hipLaunchKernelGGL((k_adapter_down<NB_, 2>), grid, dim3(256), 0, s, jobs, N);       \
    else hipLaunchKernelGGL((k_adapter_down<NB_, 1>), grid, dim3(256), 0, s, jobs, N);               \
  } while (0)
  if (nb <= 1) LSW_AD(1);
  else if (nb <= 2) LSW_AD(2);
  else LSW_AD(4);                         // 3..4 blocks: one group of 4; 5..8: two groups of 4 (the layout is padded to whole groups)
#undef LSW_AD
  return hipGetLastError();
}

// Z[t][col] = scale * g(t, expert of col) * sum over the slices of Upart[.][t][col]; columns N..z_stride-1 are zeroed.
// A token's list is checked as the switch's lists are: an id outside [0, E), a duplicate id or a non-finite gate
// raises the sticky error word (flag 2) and gives that token an all-zero row (its output stays what it was).
__global__ __launch_bounds__(256) void k_adapter_gate(AdJobs jobs, const int32_t* __restrict__ ids,
                                                      const float* __restrict__ gates, int k, int E, int r, float scale,
                                                      int z_stride, int32_t* __restrict__ err) {
  const int N = E * r, T = jobs.T;
  const long long per = (long long)T * z_stride, total = per * jobs.n;      // every linear of the call, one after the other
  for (long long gidx = (long long)blockIdx.x * blockDim.x + threadIdx.x; gidx < total; gidx += (long long)gridDim.x * blockDim.x) {
    const int job = int(gidx / per);
    const long long idx = gidx - job * per;
    const float* __restrict__ Upart = jobs.Upart[job];
    float* __restrict__ Z = jobs.Z[job];
    const int n_slices = jobs.n_slices[job];
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
        if (col == 0 && job == 0) atomicOr(err, 2);
      } else if (coeff != 0.0f) {
        float u = 0.0f;
        for (int s = 0; s < n_slices; ++s) u += Upart[((long long)s * T + t) * N + col];
        z = coeff * u;
      }
    }
    Z[idx] = z;
  }
}

hipError_t launch_adapter_gate(const AdJobs& jobs, const int32_t* ids, const float* gates, int k, int E, int r,
                               float scale, int z_stride, int32_t* err, hipStream_t s) {
  const long long total = (long long)jobs.T * z_stride * jobs.n;
  const int grid = int(std::min<long long>((total + 255) / 256, 1 << 16));
  hipLaunchKernelGGL(k_adapter_gate, dim3(grid), dim3(256), 0, s, jobs, ids, gates, k, E, r, scale, z_stride, err);
  return hipGetLastError();
}

}  // namespace lsw
