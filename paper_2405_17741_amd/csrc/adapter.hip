// liblsw device code (gfx950): the un-merged adapter path for prompts (down-projection, gate table).
#include "lsw_device.h"
#include "lsw_mfma.h"

#include <algorithm>
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
// Three launches per call, whether the call covers one linear or all linears of a layer.  (1) k_adapter_down: U = X A_all^T on the matrix cores, all E*r down-projection rows of
// all experts at once (N = E*r is at most 256, so computing the unselected experts too costs nothing next to the
// traffic), the long contraction over `in` cut into slices whose partial sums go to Upart[slice][T][N].
// (2) k_adapter_gate: Z[t][e*r+rho] = scale * g(t,e) * sum_slices Upart (zero for experts token t did not select):
// the gather of the token's experts is a multiplication by a mostly-zero gate table.  (3) the matrix-core switch
// kernels in adapter mode: Y[T,out] <- rne(Y + Z B_all^T), rows = tokens, the row operand read from Z, the shared
// operand B^T packed like A (k_pack_A, transposed source).
//
// k_adapter_down.  X is bf16 and needs no split; A is split into bf16 high + low (two passes).  Inside a 64-column chunk u
// the contraction index is ordered  k-step s (0..3), lane half h, element i  <->  column 64u + 32h + 8s + i  (a lane's four
// k-steps are four consecutive 16-byte pieces of its token's row).  The A operand comes from a re-laid-out copy built once
// (k_pack_Atk):
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

// Token blocks of 32 per wave (RB).  1: a workgroup covers 128 tokens and keeps two LDS stages (64 KB at 64 down-projection
// rows), so two workgroups share a CU; 2: 256 tokens and three stages, one workgroup per CU, half the L2 traffic for A.
// Measured per 7B layer: 512 tokens equal, 1024: 76 against 82 us, 2048: 118 against 125, 4096: 200 against 221, 8192: 401
// against 404, 16384: 810 against 822, and one call per linear at 16384 tokens 1,297 against 1,105 us: small tiles up to 8192.
int adapter_token_blocks(int T, int N) { (void)N; return T <= 8192 ? 1 : 2; }

// 64-column chunks one workgroup contracts: about 128 workgroups per linear (a call usually covers the linears of a
// layer), at least 8 chunks each unless the matrix has fewer (every slice costs a set of partial sums)
int adapter_chunks_per_slice(int T, int in, int N) {
  const int nch = ceil_div(in, AD_CHUNK);
  const long long tiles = ceil_div(T, 128 * adapter_token_blocks(T, N));
  const long long cps = std::max<long long>(8, (nch * tiles + 127) / 128);
  return int(std::min<long long>(nch, cps));
}

int adapter_slices(int T, int in, int N) { return ceil_div(ceil_div(in, AD_CHUNK), adapter_chunks_per_slice(T, in, N)); }

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

// k_adapter_down.  A workgroup = 4 waves x RB blocks of 32 tokens x one slice of `in` (cps chunks of 64 columns).  Every
// wave owns its tokens and accumulates over the slice's chunks, so there is nothing to reduce across waves.
//
// Both operands reach the matrix cores through LDS, copied there by LDS-DMA (no registers), kAdStages chunks deep:
//   A: the chunk's NB * 4 * QP pieces of 1 KB are the same for all tokens; the four waves copy a quarter each, all read
//      them, so a chunk of A leaves L2 once per 128 * RB tokens.
//   X: a wave's 32 * RB token rows of the chunk (128 bytes each).  The matrix-core operand wants a lane to hold 16 bytes
//      of ITS token's row, and loading it that way makes every load instruction touch 32 different rows 16 bytes at a
//      time, which is what bounded this kernel (measured: 160 us against 57 us at 8192 tokens with the same bytes read
//      contiguously).  So the copy reads whole rows, 8 rows of 128 bytes per instruction, and the transposition happens on
//      the LDS side: row t keeps its 16-byte piece p at slot p ^ (t & 7), which the copy arranges by having the lane that
//      fills slot s read piece s ^ (t & 7), and which spreads the operand reads (32 rows, one slot each) over the banks.
// Token rows past T are read as row T-1 (their results are not written); pieces past the end of a row (in is a multiple
// of 8, not of 64) are read as piece 0 of the chunk: the packed A holds zeros there.
// One barrier per chunk.  One launch covers every linear of the call: workgroups jobs.first[i] .. jobs.first[i+1]-1 belong
// to linear i and are numbered (group of 4 row blocks, slice, token tile), the token tile fastest.
template <int NB, int QP, int RB>
constexpr int kAdStageSlots = NB * 4 * QP * 64 + 4 * RB * 256;       // 16-byte slots of one stage: A pieces, then the waves' X tiles
template <int NB, int QP, int RB>
constexpr int kAdStages = (RB > 1 && 3 * kAdStageSlots<NB, QP, RB> * 16 <= 144 * 1024) ? 3 : 2;     // RB = 1: two, so that two workgroups fit a CU

template <int NB, int QP, int RB>
__global__ __launch_bounds__(256) void k_adapter_down(AdJobs jobs, int N) {
  constexpr int kPieces = NB * 4 * QP;                 // 1 KB pieces of one chunk's A operand: [nb][k-step][part]
  constexpr int kStage = kAdStageSlots<NB, QP, RB>;
  constexpr int kStages = kAdStages<NB, QP, RB>;
  static_assert(kPieces % 4 == 0, "pieces divide among the four waves");
  const int lane = threadIdx.x & 63, wave = uniform(int(threadIdx.x >> 6)), n = lane & 31, h = lane >> 5;
  const int job = uniform(find_segment(jobs.first, jobs.n, int(blockIdx.x)));
  const uint16_t* __restrict__ X = uniform(jobs.X[job]);
  const uint16_t* __restrict__ Atk = uniform(jobs.Atk[job]);
  float* __restrict__ Upart = uniform(jobs.Upart[job]);
  const int T = jobs.T, in = uniform(jobs.in[job]), cps = uniform(jobs.cps[job]), n_slices = uniform(jobs.n_slices[job]);
  const int n_tiles = ceil_div(T, 128 * RB);
  const int local = uniform(int(blockIdx.x) - jobs.first[job]);
  const int tile = local % n_tiles, slice = (local / n_tiles) % n_slices, zgroup = local / (n_tiles * n_slices);
  const int nch = ceil_div(in, AD_CHUNK);
  const int u0 = slice * cps, u1 = min(nch, u0 + cps);
  const int tok0 = 128 * RB * tile + 32 * RB * wave;     // this wave's first token
  const int nb0 = zgroup * NB;           // N above 128: the 32-column blocks come in two groups of workgroups
  // piece (nb, s4, hl) of chunk u lies at q0 + (((nb * nch + u) * 4 + s4) * QP + hl) * 64 (16-byte units, + lane)
  const u32x4* q0 = reinterpret_cast<const u32x4*>(Atk) + (long long)nb0 * nch * 4 * QP * 64 + lane;
  // X copy: instruction i of block rb moves rows 8i .. 8i+7; this lane fills slot lane & 7 of row 8i + lane / 8
  const int xrow = lane >> 3, xslot = lane & 7;
  auto copy_chunk = [&](int u, int stage) {
    u32x4* base = wg_lds + stage * kStage;
#pragma unroll
    for (int i = 0; i < kPieces / 4; ++i) {                // this wave's quarter of the A pieces
      const int piece = wave * (kPieces / 4) + i;         // = (nb * 4 + s4) * QP + hl
      const int nb = piece / (4 * QP), rest = piece % (4 * QP);
      lds_dma16(q0 + ((long long)(nb * nch + u) * 4 * QP + rest) * 64, base + piece * 64);
    }
    const int pieces_in_row = min(8, (in - AD_CHUNK * u) >> 3);      // 16-byte pieces of this chunk that exist in a row
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 8 * i + xrow;                     // row of the block; its low three bits are those of xrow
        const int t = min(tok0 + 32 * rb + row, T - 1);
        int piece = xslot ^ (xrow & 7);
        piece = piece < pieces_in_row ? piece : 0;
        lds_dma16(X + (long long)t * in + AD_CHUNK * u + 8 * piece, base + kPieces * 64 + ((wave * RB + rb) * 32 + 8 * i) * 8);
      }
  };
  f32x16 acc[RB][NB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[rb][nb][v] = 0.0f;
  constexpr int kPerStep = kPieces / 4 + RB * 4;       // LDS copies a wave issues per chunk
  auto wait_and_meet = [&](int newer) {                // all but the `newer` youngest copies of this wave have landed; then the workgroup meets
    __builtin_amdgcn_sched_barrier(0);
    if (newer == 0) __builtin_amdgcn_s_waitcnt(0x0F70);
    else if (newer == kPerStep) __builtin_amdgcn_s_waitcnt(0x0F70 | (kPerStep & 15) | ((kPerStep >> 4) << 14));
    else __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * kPerStep) & 15) | (((2 * kPerStep) >> 4) << 14));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    __builtin_amdgcn_sched_barrier(0);
  };
  static_assert(2 * kPerStep < 64, "the wait counter has six bits");
  // prologue: the first kStages - 1 chunks are requested, the first one awaited
  int ahead = 0;                                       // chunks requested and not yet awaited, beyond the current one
  copy_chunk(u0, 0);
#pragma unroll
  for (int d = 1; d < kStages - 1; ++d)
    if (u0 + d < u1) { copy_chunk(u0 + d, d); ++ahead; }
  wait_and_meet(ahead * kPerStep);
  int stage = 0;
  for (int u = u0; u < u1; ++u) {                      // uniform over the workgroup
    // request chunk u + kStages - 1 into the stage that was read in step u - 1 (which ended in a barrier)
    const bool more = u + kStages - 1 < u1;
    if (more) copy_chunk(u + kStages - 1, (stage + kStages - 1) % kStages);
    const u32x4* ab = wg_lds + stage * kStage + lane;
    const u32x4* xb = wg_lds + stage * kStage + kPieces * 64 + (wave * RB * 32 + n) * 8;
    // Matrix work of the chunk as a flat list of NB * QP * 4 operand pieces of A, k-step outermost: i = (s4 * NB + nb) * QP
    // + (QP - 1 - hl), the small (low-part) products first.  kDepth LDS reads of A and the X operands of the next k-step
    // stay in flight ahead of the matrix instructions that use them.
    constexpr int kDepth = 4, kPerK = NB * QP;
    auto a_slot = [](int i) { const int s4 = i / kPerK, nb = (i % kPerK) / QP, hl = QP - 1 - i % QP; return ((nb * 4 + s4) * QP + hl) * 64; };
    u32x4 qr[kDepth], xr[2][RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) xr[0][rb] = xb[rb * 256 + ((4 * h + 0) ^ (n & 7))];
#pragma unroll
    for (int i = 0; i < kDepth; ++i) qr[i] = ab[a_slot(i)];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 4 * kPerK; ++i) {
      const int s4 = i / kPerK, nb = (i % kPerK) / QP;
      if (i % kPerK == 0 && s4 + 1 < 4) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) xr[(s4 + 1) & 1][rb] = xb[rb * 256 + ((4 * h + s4 + 1) ^ (n & 7))];
      }
      const bf16x8 q = __builtin_bit_cast(bf16x8, qr[i % kDepth]);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        acc[rb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xr[s4 & 1][rb]), q, acc[rb][nb], 0, 0, 0);
      if (i + kDepth < 4 * kPerK) qr[i % kDepth] = ab[a_slot(i + kDepth)];
      __builtin_amdgcn_sched_barrier(0);
    }
    // chunk u + 1 must have landed before the next step; what was requested after it may stay in flight
    const int left = u1 - 1 - u;                       // chunks after this one
    const int newer = left <= 1 ? 0 : min(left - 1, kStages - 2);
    wait_and_meet(newer * kPerStep);
    stage = (stage + 1) % kStages;
  }
  // acc[rb][nb][v] is U[token tok0 + 32*rb + 8*(v/4) + 4h + v%4][column 32*(nb0 + nb) + n]
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int col = 32 * (nb0 + nb) + n;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int t = tok0 + 32 * rb + 8 * (v >> 2) + 4 * h + (v & 3);
        if (t < T && col < N) Upart[((long long)slice * T + t) * N + col] = acc[rb][nb][v];
      }
    }
}

template <int NB, int QP, int RB>
static hipError_t launch_down(const AdJobs& jobs, int N, unsigned grid, hipStream_t s) {
  const size_t lds = size_t(kAdStages<NB, QP, RB>) * kAdStageSlots<NB, QP, RB> * sizeof(u32x4);
  static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_adapter_down<NB, QP, RB>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
  if (lds_ok != hipSuccess) return lds_ok;
  hipLaunchKernelGGL((k_adapter_down<NB, QP, RB>), dim3(grid), dim3(256), lds, s, jobs, N);
  return hipGetLastError();
}

hipError_t launch_adapter_down(const AdJobs& jobs_in, int N, int qp, hipStream_t s) {
  AdJobs jobs = jobs_in;
  const int nb = ceil_div(N, 32);
  const int zgroups = nb > 4 ? 2 : 1;
  const int nb_read = nb <= 1 ? 1 : nb <= 2 ? 2 : 4 * zgroups;       // blocks of Atk a workgroup row reads
  if (jobs.n < 1 || jobs.n > kAdMaxLin || nb > 8 || nb_read != adapter_blocks(N)) return hipErrorInvalidValue;   // never beyond what k_pack_Atk laid out
  const int rb = adapter_token_blocks(jobs.T, N);
  // Workgroups start in the order of their numbers and a linear's workgroups all take equally long (cps chunks): the
  // linears with the longest slices go first, so that the launch does not end with a few long workgroups on a half-empty chip.
  int order[kAdMaxLin];
  for (int i = 0; i < jobs.n; ++i) order[i] = i;
  std::stable_sort(order, order + jobs.n, [&](int a, int b) { return jobs_in.cps[a] > jobs_in.cps[b]; });
  for (int i = 0; i < jobs.n; ++i) {
    const int j = order[i];
    jobs.X[i] = jobs_in.X[j];
    jobs.Atk[i] = jobs_in.Atk[j];
    jobs.Upart[i] = jobs_in.Upart[j];
    jobs.Z[i] = jobs_in.Z[j];
    jobs.in[i] = jobs_in.in[j];
    jobs.cps[i] = jobs_in.cps[j];
    jobs.n_slices[i] = jobs_in.n_slices[j];
  }
  long long total = 0;
  for (int i = 0; i < jobs.n; ++i) {
    jobs.first[i] = int(total);
    total += (long long)ceil_div(jobs.T, 128 * rb) * jobs.n_slices[i] * zgroups;
    if (total > INT32_MAX) return hipErrorInvalidValue;
  }
  for (int i = jobs.n; i <= kAdMaxLin; ++i) jobs.first[i] = int(total);
  const unsigned grid = unsigned(total);
#define LSW_AD(NB_)                                                                                                       \
  do {                                                                                                                    \
    if (qp == 2) return rb == 1 ? launch_down<NB_, 2, 1>(jobs, N, grid, s) : launch_down<NB_, 2, 2>(jobs, N, grid, s);    \
    return rb == 1 ? launch_down<NB_, 1, 1>(jobs, N, grid, s) : launch_down<NB_, 1, 2>(jobs, N, grid, s);                 \
  } while (0)
  if (nb <= 1) LSW_AD(1);
  else if (nb <= 2) LSW_AD(2);
  else LSW_AD(4);                         // 3..4 blocks: one group of 4; 5..8: two groups of 4 (the layout is padded to whole groups)
#undef LSW_AD
}

// Z[t][col] = scale * g(t, expert of col) * sum over the slices of Upart[.][t][col]; columns N..z_stride-1 are zeroed.
// A token's list is checked as the switch's lists are: an id outside [0, E), a duplicate id or a non-finite gate
// raises the sticky error word (flag 2) and gives that token an all-zero row (its output stays what it was).
__global__ __launch_bounds__(256) void k_adapter_gate(AdJobs jobs, const int32_t* __restrict__ ids,
                                                      const float* __restrict__ gates, int k, int E, int r, float scale,
                                                      int z_stride, int32_t* __restrict__ err) {
  // one thread = four consecutive columns of one token (r is a multiple of 8: they belong to one expert)
  const int N = E * r, T = jobs.T, zq = z_stride >> 2;
  const long long per = (long long)T * zq, total = per * jobs.n;      // every linear of the call, one after the other
  for (long long gidx = (long long)blockIdx.x * blockDim.x + threadIdx.x; gidx < total; gidx += (long long)gridDim.x * blockDim.x) {
    const int job = int(gidx / per);
    const long long idx = gidx - job * per;
    const float* __restrict__ Upart = jobs.Upart[job];
    f32x4* __restrict__ Z = reinterpret_cast<f32x4*>(jobs.Z[job]);
    const int n_slices = jobs.n_slices[job];
    const int t = int(idx / zq), col = 4 * int(idx - (long long)t * zq);
    f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
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
        f32x4 u = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int s = 0; s < n_slices; ++s) u += *reinterpret_cast<const f32x4*>(Upart + ((long long)s * T + t) * N + col);
        z = coeff * u;
      }
    }
    Z[idx] = z;
  }
}

hipError_t launch_adapter_gate(const AdJobs& jobs, const int32_t* ids, const float* gates, int k, int E, int r,
                               float scale, int z_stride, int32_t* err, hipStream_t s) {
  const long long total = (long long)jobs.T * (z_stride / 4) * jobs.n;
  const int grid = int(std::min<long long>((total + 255) / 256, 1 << 16));
  hipLaunchKernelGGL(k_adapter_gate, dim3(grid), dim3(256), 0, s, jobs, ids, gates, k, E, r, scale, z_stride, err);
  return hipGetLastError();
}

}  // namespace lsw
