// liblsw device code (gfx950): the fused adapter switch on the matrix cores with one item's A resident in LDS.
#include "lsw_device.h"
#include "lsw_mfma.h"

namespace lsw {

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
  int out, in, ld;
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
  c.ld = uniform(Lp->ld);
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

template <int NKS, int QP, bool PROBE>
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
  const int nout = uniform(last ? nxt.out : cur.out), nin = uniform(last ? nxt.in : cur.in), nld = uniform(last ? nxt.ld : cur.ld);
  const __amdgpu_buffer_rsrc_t nres = w_resource(last ? nxt.Wsrc : cur.Wsrc, w_extent_bytes(nout, nin, nld));
  const uint32_t nstride = uint32_t(nld) * 2u;
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
  if constexpr (!PROBE) {
    if (boundary) res_load_b<NKS, QP>(nxt, wave, n, r, term_e, term_g, braw);
    wg_compute<NKS, QP>(p_hi, p_lo, wg_lds + ((cs - cur.col0) / MT_STEP) * kStepSlots + lane, wcur);
  } else {
    wg_probe_compute(wcur);
  }

  prev_res = w_resource(cur.W, w_extent_bytes(cur.out, cur.in, cur.ld));
  prev_off = lane_off;
  prev_stride = uint32_t(cur.ld) * 2u;
  lane_off = nlane_off;
  cs = ncs;
  if (last) {                      // item boundary (uniform over the workgroup: all four waves walk the same items)
    if (!have_nxt) return false;
    if constexpr (!PROBE) res_make_p<NKS>(nxt, wave, n, term_c, braw, p_hi, p_lo);
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
      if constexpr (!PROBE) res_fetch_q<NKS, QP>(p, cur, n, gpr, wave, term_e, term_g);
      wg_drain_and_barrier();      // the new one is complete (and every wave has read the claim)
    }
    if (have_nxt_io) walk_plan_after(walk, following, via_pool, wave, lane, claim);
  }
  return true;
}

template <int NKS, int QP, bool PROBE>
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
  if constexpr (!PROBE) {
    float braw[NKS][8];
    res_load_b<NKS, QP>(cur, wave, n, r, term_e, term_g, braw);
    res_make_p<NKS>(cur, wave, n, term_c, braw, p_hi, p_lo);
  }
  int cs = cur.col0;
  uint32_t lane_off = kOutOfRange;
  {
    const int col = cs + 8 * n;
    const uint32_t stride = uint32_t(cur.ld) * 2u;
    if (col < min(cur.in, cur.col0 + p.tile_cols))
      lane_off = uint32_t(cur.row0 + 32 * wave + 4 * h) * stride + uint32_t(col) * 2u;
  }
  u32x4 wa[16], wb[16];
  {
    const __amdgpu_buffer_rsrc_t res = w_resource(cur.Wsrc, w_extent_bytes(cur.out, cur.in, cur.ld));
#pragma unroll
    for (int v = 0; v < 16; ++v)
      wa[v] = __builtin_amdgcn_raw_buffer_load_b128(
          res, lane_off + uint32_t(8 * (v >> 2) + (v & 3)) * (uint32_t(cur.ld) * 2u), 0, kWLoadAux);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) wb[v] = u32x4{0u, 0u, 0u, 0u};
  if constexpr (!PROBE) res_fetch_q<NKS, QP>(p, cur, n, gpr, wave, term_e, term_g);
  wg_drain_and_barrier();
  __amdgpu_buffer_rsrc_t prev_res = w_resource(cur.W, w_extent_bytes(cur.out, cur.in, cur.ld));
  uint32_t prev_off = kOutOfRange, prev_stride = 0;

  bool a_is_cur = true;
  while (true) {
    if (!res_step<NKS, QP, PROBE>(p, n, h, lane, wave, gpr, r, term_e, term_g, term_c, cur, nxt, have_nxt, walk, claim, cs, lane_off,
                           prev_res, prev_off, prev_stride, p_hi, p_lo, wa, wb)) { a_is_cur = true; break; }
    if (!res_step<NKS, QP, PROBE>(p, n, h, lane, wave, gpr, r, term_e, term_g, term_c, cur, nxt, have_nxt, walk, claim, cs, lane_off,
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

template <int NKS, int QP, bool PROBE = false>
static hipError_t launch_res(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int grid, hipStream_t s) {
  size_t lds = size_t(p.tile_cols / MT_STEP) * NKS * 8 * QP * 64 * sizeof(u32x4);     // 8 KB per column step, k-step and Q part
  if (lds > size_t(kResidentLdsBytes) || p.Z != nullptr) return hipErrorInvalidValue;
  // the probe uses few registers and no LDS: it asks for more than half a CU's LDS so that, like the kernels it stands in
  // for, exactly one workgroup runs per CU (two on one CU would leave another CU idle)
  if (PROBE) lds = std::max(lds, size_t(kProbeLdsBytes));
  // once per process (function-local statics are initialised exactly once, also under concurrent first calls)
  static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_switch_mfma_res<NKS, QP, PROBE>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kResidentLdsBytes);
  if (lds_ok != hipSuccess) return lds_ok;
  hipLaunchKernelGGL((k_switch_mfma_res<NKS, QP, PROBE>), dim3(grid), dim3(64 * WG_WAVES), lds, s, p, t, t_dev, r);
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
  if (p.probe) return launch_res<1, 2, true>(p, t, t_dev, r, grid, s);
  return qp == 2 ? launch_res_qp<2>(p, t, t_dev, r, grid, s) : launch_res_qp<1>(p, t, t_dev, r, grid, s);
}

}  // namespace lsw
