// liblsw device code (gfx950): the fused adapter switch on the matrix cores, fused rank up to 64, A streamed per step.
#include "lsw_device.h"
#include "lsw_mfma.h"

namespace lsw {

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

// One step of a wave: start the copy of the next step's Q quarter into the idle LDS buffer, store
// the previous step's tile, request the next tile into the freed registers, update the current
// tile, then drain and meet the workgroup.  Everything requested at the top has the whole compute
// phase to arrive.  Returns false after the last tile of the workgroup.
template <int NKS, int QP, bool PROBE>
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
  if constexpr (!PROBE) {   // (a finished workgroup re-reads its last block, which is harmless)
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

  if constexpr (PROBE) wg_probe_compute(wcur);
  else wg_compute<NKS, QP>(cur.p_hi, cur.p_lo, wg_lds + buf * kBufSlots + lane, wcur);

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
      mfma_load_item<NKS, QP, PROBE>(p, following, n, gpr, r, term_e, term_g, term_c, nxt, WG_ROWS, 32 * wave, p.flat ? walk.static_end : 0);
      if (p.flat) walk.step = mfma_item_units(nxt);
      walk_plan_after(walk, following, via_pool, wave, lane, claim);
    }
  }
  return true;
}

template <int NKS, int QP, bool PROBE>
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
  const bool flat = p.flat != 0;
  const int item0 = flat ? walk_init_flat(p, walk) : walk_init(p, p.xcd_remap == 2, walk);
  if (item0 >= walk.static_end) return; // uniform over the workgroup (never with a pool)
  const int flat_end = flat ? walk.static_end : 0;
  MfmaItem<NKS> cur, nxt;
  mfma_load_item<NKS, QP, PROBE>(p, item0, n, gpr, r, term_e, term_g, term_c, cur, WG_ROWS, 32 * wave, flat_end);
  if (flat) walk.step = mfma_item_units(cur);
  const int item1 = item0 + walk.step;
  bool have_nxt = item1 < walk.static_end;
  int claim = 0;
  if (have_nxt) {
    mfma_load_item<NKS, QP, PROBE>(p, item1, n, gpr, r, term_e, term_g, term_c, nxt, WG_ROWS, 32 * wave, flat_end);
    if (flat) walk.step = mfma_item_units(nxt);
    walk_plan_after(walk, item1, false, wave, lane, claim);
  } else {
    nxt = cur;
  }
  int cs = cur.col0;
  uint32_t lane_off = mfma_lane_offset<NKS>(cur, cs, n, h);
  u32x4 wa[16], wb[16];
  mfma_load_w<NKS>(cur, lane_off, wa);
#pragma unroll
  for (int v = 0; v < 16; ++v) wb[v] = u32x4{0u, 0u, 0u, 0u};
  if constexpr (!PROBE) wg_fetch_q<NKS, QP>(cur.Apk, cur.ncb, cs, n, gpr, wave, term_e, term_g, wg_lds);
  wg_drain_and_barrier();
  __amdgpu_buffer_rsrc_t prev_res = w_resource(cur.W, cur.wbytes);
  uint32_t prev_off = kOutOfRange, prev_stride = 0;

  bool a_is_cur = true;
  while (true) {
    if (!wg_step<NKS, QP, PROBE>(p, n, h, lane, wave, gpr, r, term_e, term_g, term_c, cur, nxt, have_nxt, walk, claim, cs, lane_off,
                      prev_res, prev_off, prev_stride, wa, wb, 0)) { a_is_cur = true; break; }
    if (!wg_step<NKS, QP, PROBE>(p, n, h, lane, wave, gpr, r, term_e, term_g, term_c, cur, nxt, have_nxt, walk, claim, cs, lane_off,
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

template <int NKS, int QP, bool PROBE = false>
static hipError_t launch_wg(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int grid, hipStream_t s) {
  // 16 KB per k-step and Q part, two buffers; the probe (few registers, no LDS use) asks for more than half a CU's LDS so
  // that, like the kernels it stands in for, exactly one workgroup runs per CU
  const size_t lds = PROBE ? size_t(kProbeLdsBytes) : size_t(2) * NKS * 8 * QP * 64 * sizeof(u32x4);
  // once per process (function-local statics are initialised exactly once, also under concurrent first calls)
  static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_switch_mfma<NKS, QP, PROBE>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
  if (lds_ok != hipSuccess) return lds_ok;
  hipLaunchKernelGGL((k_switch_mfma<NKS, QP, PROBE>), dim3(grid), dim3(64 * WG_WAVES), lds, s, p, t, t_dev, r);
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
  if (p.probe) return launch_wg<1, 2, true>(p, t, t_dev, r, grid, s);
  return qp == 2 ? launch_wg_qp<2>(p, t, t_dev, r, grid, s) : launch_wg_qp<1>(p, t, t_dev, r, grid, s);
}

}  // namespace lsw
