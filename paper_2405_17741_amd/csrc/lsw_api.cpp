// Host side of liblsw: argument checks, the signed term list of a switch, the
// Softmax(TopK) router, the work decomposition, context state and kernel dispatch.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <vector>

#include "lsw_internal.h"

using namespace lsw;

// ---------------------------------------------------------------------------
// error reporting
// ---------------------------------------------------------------------------
static thread_local char g_err[512] = "";

static lsw_status fail(lsw_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

#define LSW_HIP(call)                                                                     \
  do {                                                                                    \
    hipError_t e_ = (call);                                                               \
    if (e_ != hipSuccess) {                                                               \
      lsw_status st_ = (e_ == hipErrorOutOfMemory) ? LSW_ERR_NOMEM : LSW_ERR_DEVICE;      \
      return fail(st_, "%s failed: %s", #call, hipGetErrorString(e_));                    \
    }                                                                                     \
  } while (0)

extern "C" const char* lsw_last_error(void) { return g_err; }

// ---------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------
struct PlanKey {
  int kernel;                 // 1 vector-ALU, 2 matrix-core
  int tile_cols;
  std::vector<int32_t> layers;  // empty = all
  bool operator<(const PlanKey& o) const {
    if (kernel != o.kernel) return kernel < o.kernel;
    if (tile_cols != o.tile_cols) return tile_cols < o.tile_cols;
    return layers < o.layers;
  }
};

struct DevicePlan {
  int32_t* d_sel = nullptr;   // one allocation: sel[n_sel] followed by first[n_sel+1]
  int32_t n_sel = 0;
  int32_t n_items = 0;
};

struct LayerState {
  int32_t k = 0;
  int32_t ids[LSW_MAX_K];
  float gates[LSW_MAX_K];
};

struct lsw_ctx {
  std::vector<lsw_linear> lin;
  std::vector<int32_t> layer_ids;            // sorted distinct layer numbers
  std::vector<LayerState> state;             // parallel to layer_ids
  int32_t E = 0, r = 0;
  int qp = 2;                                // Q parts: 2 = fp32-stored factors, 1 = bf16-stored factors
  float scale = 1.0f;
  int device = 0;
  int n_cu = 0;
  LinDesc* d_lin = nullptr;
  std::vector<LinDesc> desc;                 // host copy of the descriptor table
  bool have_base = false;                    // lsw_set_base has registered the base copies
  uint16_t* d_apk = nullptr;                 // packed A of all linears (r % 8 == 0 only)
  void* static_scratch = nullptr;            // this device's copy of the library's static workspace (lsw_adapter_forward_static)
  uint16_t* d_adapter = nullptr;             // adapter path: per linear the down-projection layout of A, then the packed B^T
  std::vector<size_t> atk_off, bpk_off;      // element offsets of the two parts of linear p inside d_adapter
  char* d_slots = nullptr;                   // the sticky error word (first kSlotBytes), then kLaunchSlots launch slots
  int32_t* d_err = nullptr;
  int slot_next = 0;                         // the slot the next switch launch takes
  int64_t owned_bytes = 0;
  int64_t x_elems = 0, y_elems = 0;          // sizes of the back-to-back x and y of lsw_merged_gemv_all
  std::map<PlanKey, DevicePlan> plans;
  int opt_kernel = 0, opt_strict = 0, opt_grid = 0, opt_tile_cols = kMfmaTileCols, opt_tile_cols_bigk = kMfmaBigkTileCols, opt_xcd = 3, opt_gemv_grid = 0, opt_one_pass = 1, opt_resident = 1, opt_pool = 1, opt_panel_group = -1;
  int last_kernel = 0, last_variant = 0, last_items = 0, last_grid = 0;
};

// What a switch launch WRITES besides the weights: the term list lsw_switch_dev builds on the device and the two
// counters of the item pool.  Every launch takes the next of kLaunchSlots slots in turn, so launches of one context
// that overlap on different streams (disjoint layer subsets) do not share them; a slot is reused after kLaunchSlots
// further launches.  The counters of a slot are zero whenever no launch is using it (the kernels leave them so).
struct LaunchSlot {
  Terms terms;
  int32_t pool[2];
};
constexpr int kLaunchSlots = 16;
constexpr size_t kSlotBytes = 256;
static_assert(sizeof(LaunchSlot) <= kSlotBytes, "slot size");

static LaunchSlot* take_slot(lsw_ctx* c) {
  LaunchSlot* s = reinterpret_cast<LaunchSlot*>(c->d_slots + kSlotBytes * size_t(1 + c->slot_next));
  c->slot_next = (c->slot_next + 1) % kLaunchSlots;
  return s;
}

static int layer_slot(const lsw_ctx* c, int32_t layer) {
  auto it = std::lower_bound(c->layer_ids.begin(), c->layer_ids.end(), layer);
  if (it == c->layer_ids.end() || *it != layer) return -1;
  return int(it - c->layer_ids.begin());
}

// ---------------------------------------------------------------------------
// step a1: router
// ---------------------------------------------------------------------------
extern "C" lsw_status lsw_route(const float* logits, int32_t E, int32_t k, int32_t* ids, float* gates) {
  if (!logits || E < 1) return fail(LSW_ERR_ARG, "lsw_route: logits null or E < 1");
  if (k < 0 || k > E) return fail(LSW_ERR_ARG, "lsw_route: k=%d outside 0..E=%d", k, E);
  if (k > 0 && (!ids || !gates)) return fail(LSW_ERR_ARG, "lsw_route: null output");
  for (int32_t i = 0; i < E; ++i)
    if (std::isnan(logits[i])) return fail(LSW_ERR_ARG, "lsw_route: logit %d is NaN", i);
  // selection: k passes, each taking the largest remaining logit; `>` keeps the lowest index on ties
  std::vector<char> taken(size_t(E), 0);
  for (int32_t c = 0; c < k; ++c) {
    int32_t best = -1;
    for (int32_t i = 0; i < E; ++i) {
      if (taken[i]) continue;
      if (best < 0 || logits[i] > logits[best]) best = i;
    }
    taken[best] = 1;
    ids[c] = best;
  }
  if (k == 0) return LSW_OK;
  const double top = double(logits[ids[0]]);
  std::vector<double> ex(size_t(k), 0.0);
  double sum = 0.0;
  for (int32_t c = 0; c < k; ++c) {
    ex[c] = std::exp(double(logits[ids[c]]) - top);
    sum += ex[c];
  }
  for (int32_t c = 0; c < k; ++c) gates[c] = float(ex[c] / sum);
  return LSW_OK;
}

// ---------------------------------------------------------------------------
// step a2: the signed term list
// ---------------------------------------------------------------------------
static lsw_status check_list(const char* which, const int32_t* ids, const float* gates, int32_t k, int32_t E) {
  if (k < 0 || k > LSW_MAX_K) return fail(LSW_ERR_ARG, "%s: k=%d outside 0..%d", which, k, int(LSW_MAX_K));
  if (k > E) return fail(LSW_ERR_ARG, "%s: k=%d exceeds E=%d", which, k, E);
  if (k > 0 && (!ids || !gates)) return fail(LSW_ERR_ARG, "%s: null list with k=%d", which, k);
  for (int32_t a = 0; a < k; ++a) {
    if (ids[a] < 0 || ids[a] >= E) return fail(LSW_ERR_ARG, "%s: id %d outside [0,%d)", which, ids[a], E);
    if (!std::isfinite(gates[a])) return fail(LSW_ERR_ARG, "%s: gate %d is not finite", which, a);
    for (int32_t b = 0; b < a; ++b)
      if (ids[b] == ids[a]) return fail(LSW_ERR_ARG, "%s: duplicate id %d", which, ids[a]);
  }
  return LSW_OK;
}

extern "C" lsw_status lsw_build_terms(const int32_t* old_ids, const float* old_gates, int32_t k_old,
                                      const int32_t* new_ids, const float* new_gates, int32_t k_new,
                                      int32_t E, float scale, int32_t* terms_ids, float* terms_coeff,
                                      int32_t* n_terms) {
  if (E < 1) return fail(LSW_ERR_ARG, "E < 1");
  if (!std::isfinite(scale)) return fail(LSW_ERR_ARG, "scale is not finite");
  if (!n_terms) return fail(LSW_ERR_ARG, "n_terms is null");
  lsw_status st = check_list("old", old_ids, old_gates, k_old, E);
  if (st != LSW_OK) return st;
  st = check_list("new", new_ids, new_gates, k_new, E);
  if (st != LSW_OK) return st;
  if (k_old + k_new > 0 && (!terms_ids || !terms_coeff)) return fail(LSW_ERR_ARG, "null term output");
  int32_t n = 0;
  for (int32_t a = 0; a < k_new; ++a) {
    float coeff = scale * new_gates[a];
    for (int32_t b = 0; b < k_old; ++b)
      if (old_ids[b] == new_ids[a]) coeff = scale * new_gates[a] - scale * old_gates[b];
    if (coeff != 0.0f) { terms_ids[n] = new_ids[a]; terms_coeff[n] = coeff; ++n; }
  }
  for (int32_t b = 0; b < k_old; ++b) {
    bool also_new = false;
    for (int32_t a = 0; a < k_new; ++a) also_new |= (new_ids[a] == old_ids[b]);
    if (also_new) continue;
    float coeff = -(scale * old_gates[b]);
    if (coeff != 0.0f) { terms_ids[n] = old_ids[b]; terms_coeff[n] = coeff; ++n; }
  }
  *n_terms = n;
  return LSW_OK;
}

// ---------------------------------------------------------------------------
// work decomposition (host view; the kernels use the same decode routines)
// ---------------------------------------------------------------------------
static bool shapes_ok(const int32_t* out, const int32_t* in, int32_t n_lin, int32_t tr, int32_t tc) {
  if (!out || !in || n_lin < 1 || tr < 1 || tc < 1) return false;
  for (int32_t p = 0; p < n_lin; ++p)
    if (out[p] < 1 || in[p] < 1) return false;
  return true;
}

extern "C" int64_t lsw_worklist_size(const int32_t* out, const int32_t* in, int32_t n_lin,
                                     int32_t tile_rows, int32_t tile_cols) {
  if (!shapes_ok(out, in, n_lin, tile_rows, tile_cols)) {
    fail(LSW_ERR_ARG, "lsw_worklist_size: bad argument");
    return -1;
  }
  int64_t n = 0;
  for (int32_t p = 0; p < n_lin; ++p)
    n += int64_t(ceil_div(out[p], tile_rows)) * ceil_div(in[p], tile_cols);
  return n;
}

extern "C" lsw_status lsw_worklist_item_grouped(const int32_t* out, const int32_t* in, int32_t n_lin,
                                                int32_t tile_rows, int32_t tile_cols, int32_t panel_group, int64_t item,
                                                int32_t* lin, int32_t* row0, int32_t* n_rows, int32_t* col0,
                                                int32_t* n_cols) {
  if (!shapes_ok(out, in, n_lin, tile_rows, tile_cols) || panel_group < 0 || !lin || !row0 || !n_rows || !col0 || !n_cols)
    return fail(LSW_ERR_ARG, "lsw_worklist_item: bad argument");
  std::vector<int32_t> first(size_t(n_lin) + 1, 0);
  int64_t total = 0;
  for (int32_t p = 0; p < n_lin; ++p) {
    total += int64_t(ceil_div(out[p], tile_rows)) * ceil_div(in[p], tile_cols);
    if (total > INT32_MAX) return fail(LSW_ERR_SHAPE, "more than 2^31 work items");
    first[p + 1] = int32_t(total);
  }
  if (item < 0 || item >= total) return fail(LSW_ERR_ARG, "item %lld outside [0,%lld)", (long long)item, (long long)total);
  int32_t s = find_segment(first.data(), n_lin, int32_t(item));
  int32_t r0, c0;
  decode_item(int32_t(item) - first[s], out[s], in[s], tile_rows, tile_cols, panel_group, &r0, &c0);
  *lin = s;
  *row0 = r0;
  *col0 = c0;
  *n_rows = std::min(tile_rows, out[s] - r0);
  *n_cols = std::min(tile_cols, in[s] - c0);
  return LSW_OK;
}

extern "C" lsw_status lsw_walk_share(int32_t n_items, int32_t grid, int32_t block, int32_t pool_div, int32_t share[5]) {
  if (n_items < 0 || grid <= 0 || grid % 8 != 0 || block < 0 || block >= grid || !share)
    return fail(LSW_ERR_ARG, "lsw_walk_share: bad argument");
  const WalkShare w = walk_share(n_items, grid, block, pool_div > 0, pool_div);
  share[0] = w.first;
  share[1] = w.step;
  share[2] = w.static_end;
  share[3] = w.per;
  share[4] = w.pool_len;
  return LSW_OK;
}

extern "C" int32_t lsw_walk_pool_item(int32_t n_items, int32_t grid, int32_t pool_div, int32_t claim) {
  if (n_items < 0 || grid <= 0 || grid % 8 != 0) return -1;
  const WalkShare w = walk_share(n_items, grid, 0, pool_div > 0, pool_div);
  return walk_pool_item(n_items, w.per, w.pool_len, claim);
}

extern "C" lsw_status lsw_flat_item(const int32_t* rows, const int32_t* cols, int32_t n_mat, int32_t grid, int32_t block,
                                    int64_t unit, int32_t* mat, int32_t* row0, int32_t* col0, int32_t* n_cols, int64_t* next_unit) {
  if (!shapes_ok(rows, cols, n_mat, kMfmaTileRows, kApkBlockCols) || grid <= 0 || grid % 8 != 0 || block < 0 || block >= grid ||
      !mat || !row0 || !col0 || !n_cols || !next_unit)
    return fail(LSW_ERR_ARG, "lsw_flat_item: bad argument");
  std::vector<int32_t> first(size_t(n_mat) + 1, 0);
  int64_t total = 0;
  for (int32_t i = 0; i < n_mat; ++i) {
    first[size_t(i)] = int32_t(total);
    total += int64_t(ceil_div(rows[i], kMfmaTileRows)) * ceil_div(cols[i], kApkBlockCols);
    if (total > INT32_MAX) return fail(LSW_ERR_SHAPE, "lsw_flat_item: more than 2^31 - 1 units");
  }
  first[size_t(n_mat)] = int32_t(total);
  int32_t lo, hi;
  flat_range(int32_t(total), grid, block, &lo, &hi);
  if (unit < 0) unit = lo;                                 // the range's first item
  if (unit < lo || unit >= hi) { *next_unit = -1; *mat = -1; *row0 = *col0 = *n_cols = 0; return LSW_OK; }   // empty range, or past its end
  const int32_t seg = find_segment(first.data(), n_mat, int32_t(unit));
  int32_t r0, c0;
  decode_item(int32_t(unit) - first[size_t(seg)], rows[seg], cols[seg], kMfmaTileRows, kApkBlockCols, 0, &r0, &c0);
  const int32_t len = flat_item_units(cols[seg], c0, int32_t(unit), hi);
  *mat = seg;
  *row0 = r0;
  *col0 = c0;
  *n_cols = std::min(cols[seg], c0 + kApkBlockCols * len) - c0;
  *next_unit = unit + len < hi ? unit + len : -1;
  return LSW_OK;
}

extern "C" lsw_status lsw_worklist_item(const int32_t* out, const int32_t* in, int32_t n_lin,
                                        int32_t tile_rows, int32_t tile_cols, int64_t item,
                                        int32_t* lin, int32_t* row0, int32_t* n_rows, int32_t* col0,
                                        int32_t* n_cols) {
  return lsw_worklist_item_grouped(out, in, n_lin, tile_rows, tile_cols, 0, item, lin, row0, n_rows, col0, n_cols);
}

// ---------------------------------------------------------------------------
// create / destroy
// ---------------------------------------------------------------------------
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" lsw_status lsw_create_adapters(const lsw_linear* lin, int32_t n_lin, int32_t E, int32_t r,
                                          float scale, lsw_ctx** out) {
  return lsw_create_adapters_ex(lin, n_lin, E, r, scale, LSW_FACTOR_F32, out);
}

extern "C" lsw_status lsw_create_adapters_ex(const lsw_linear* lin, int32_t n_lin, int32_t E, int32_t r,
                                             float scale, int32_t factor_dtype, lsw_ctx** out) {
  if (!out) return fail(LSW_ERR_ARG, "out is null");
  *out = nullptr;
  if (factor_dtype != LSW_FACTOR_F32 && factor_dtype != LSW_FACTOR_BF16) return fail(LSW_ERR_ARG, "unknown factor dtype %d", factor_dtype);
  const int qp = factor_dtype == LSW_FACTOR_BF16 ? 1 : 2;
  if (qp == 1 && r % 8 != 0) return fail(LSW_ERR_SHAPE, "bf16 factors need r %% 8 == 0 (rows of B stay 16-byte aligned)");
  if (!lin || n_lin < 1) return fail(LSW_ERR_ARG, "lin is null or n_lin < 1");
  if (E < 1 || E > 4096) return fail(LSW_ERR_ARG, "E=%d outside 1..4096", E);
  if (r < 1 || r > 512) return fail(LSW_ERR_ARG, "r=%d outside 1..512", r);
  if (!std::isfinite(scale)) return fail(LSW_ERR_ARG, "scale is not finite");
  int64_t items_valu = 0, items_mfma = 0;
  for (int32_t p = 0; p < n_lin; ++p) {
    const lsw_linear& L = lin[p];
    if (!L.W || !L.A || !L.B) return fail(LSW_ERR_ARG, "linear %d: null tensor", p);
    if (L.layer < 0) return fail(LSW_ERR_ARG, "linear %d: layer %d < 0", p, L.layer);
    if (L.out < 1) return fail(LSW_ERR_SHAPE, "linear %d: out=%d < 1", p, L.out);
    if (L.in < 8 || L.in % 8 != 0) return fail(LSW_ERR_SHAPE, "linear %d: in=%d is not a positive multiple of 8", p, L.in);
    if (L.ld != 0 && (L.ld < L.in || L.ld % 8 != 0))
      return fail(LSW_ERR_SHAPE, "linear %d: ld=%d must be 0 (dense) or a multiple of 8 that is at least in=%d", p, L.ld, L.in);
    // 32-bit byte offsets inside one W, including the rows a 128-row work item may reach past the end
    if (int64_t(ceil_div(L.out, kMfmaTileRows)) * kMfmaTileRows * (L.ld ? L.ld : L.in) * 2 >= (int64_t(1) << 31))
      return fail(LSW_ERR_SHAPE, "linear %d: W (rows rounded up to %d, at its leading dimension) must stay below 2^31 bytes", p, kMfmaTileRows);
    // 32-bit byte offsets inside one linear's packed A (E * r * padded in * 4 bytes)
    if (r % 8 == 0 && int64_t(E) * r * ceil_div(L.in, kApkBlockCols) * kApkBlockCols * 2 * qp >= (int64_t(1) << 31))
      return fail(LSW_ERR_SHAPE, "linear %d: E * r * in * 4 must stay below 2^31 bytes", p);
    if (!aligned16(L.W) || !aligned16(L.A) || !aligned16(L.B))
      return fail(LSW_ERR_SHAPE, "linear %d: tensor not 16-byte aligned", p);
    items_valu += int64_t(ceil_div(L.out, kValuTileRows)) * ceil_div(L.in, kValuTileCols);
    items_mfma += int64_t(ceil_div(L.out, kMfmaTileRows)) * ceil_div(L.in, kMfmaTileCols);
  }
  if (items_valu > INT32_MAX || items_mfma > INT32_MAX) return fail(LSW_ERR_SHAPE, "more than 2^31 work items");

  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) {
    (void)hipGetLastError();
    return fail(LSW_ERR_DEVICE, "no HIP device available");
  }

  std::unique_ptr<lsw_ctx> c(new (std::nothrow) lsw_ctx);
  if (!c) return fail(LSW_ERR_NOMEM, "host allocation failed");
  c->lin.assign(lin, lin + n_lin);
  c->E = E;
  c->r = r;
  c->scale = scale;
  c->qp = qp;
  for (int32_t p = 0; p < n_lin; ++p) c->layer_ids.push_back(lin[p].layer);
  std::sort(c->layer_ids.begin(), c->layer_ids.end());
  c->layer_ids.erase(std::unique(c->layer_ids.begin(), c->layer_ids.end()), c->layer_ids.end());
  c->state.assign(c->layer_ids.size(), LayerState());

  LSW_HIP(hipGetDevice(&c->device));
  hipDeviceProp_t prop;
  LSW_HIP(hipGetDeviceProperties(&prop, c->device));
  c->n_cu = prop.multiProcessorCount;

  // packed copy of A for the matrix-core kernel
  std::vector<LinDesc> desc(static_cast<size_t>(n_lin));
  const bool pack = (r % 8 == 0);
  size_t apk_elems = 0;
  std::vector<size_t> apk_off(size_t(n_lin), 0);
  for (int32_t p = 0; p < n_lin; ++p) {
    apk_off[p] = apk_elems;
    apk_elems += size_t(E) * size_t(r) * size_t(ceil_div(lin[p].in, kApkBlockCols) * kApkBlockCols) * size_t(qp);   // bf16 high (+ low) part per element, columns padded to the block
  }
  lsw_ctx* raw = c.get();
  auto cleanup = [raw]() {
    if (raw->d_apk) (void)hipFree(raw->d_apk);
    if (raw->d_lin) (void)hipFree(raw->d_lin);
    if (raw->d_slots) (void)hipFree(raw->d_slots);
    raw->d_apk = nullptr;
    raw->d_lin = nullptr;
    raw->d_slots = nullptr;
  };
  if (pack) {
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->d_apk), apk_elems * sizeof(uint16_t));
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(LSW_ERR_NOMEM, "hipMalloc of %zu bytes for packed A failed", apk_elems * 2); }
    c->owned_bytes += int64_t(apk_elems * sizeof(uint16_t));
    for (int32_t p = 0; p < n_lin; ++p) {
      e = launch_pack_A(lin[p].A, c->d_apk + apk_off[p], E, r, lin[p].in, qp, 0, nullptr);
      if (e != hipSuccess) { cleanup(); return fail(LSW_ERR_DEVICE, "pack kernel launch failed: %s", hipGetErrorString(e)); }
    }
  }
  for (int32_t p = 0; p < n_lin; ++p) {
    desc[p].W = static_cast<uint16_t*>(lin[p].W);
    desc[p].A = lin[p].A;
    desc[p].B = lin[p].B;
    desc[p].Apk = pack ? c->d_apk + apk_off[p] : nullptr;
    desc[p].Wbase = nullptr;
    desc[p].out = lin[p].out;
    desc[p].in = lin[p].in;
    desc[p].ld = lin[p].ld ? lin[p].ld : lin[p].in;
    desc[p].x_off = c->x_elems;
    desc[p].y_off = c->y_elems;
    c->x_elems += lin[p].in;
    c->y_elems += lin[p].out;
  }
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->d_lin), desc.size() * sizeof(LinDesc));
  if (e != hipSuccess) { (void)hipGetLastError(); cleanup(); return fail(LSW_ERR_NOMEM, "hipMalloc of the descriptor table failed"); }
  c->owned_bytes += int64_t(desc.size() * sizeof(LinDesc));
  const size_t slot_bytes = kSlotBytes * size_t(1 + kLaunchSlots);
  e = hipMalloc(reinterpret_cast<void**>(&c->d_slots), slot_bytes);
  if (e != hipSuccess) { (void)hipGetLastError(); cleanup(); return fail(LSW_ERR_NOMEM, "hipMalloc of the launch slots failed"); }
  c->d_err = reinterpret_cast<int32_t*>(c->d_slots);
  c->owned_bytes += int64_t(slot_bytes);
  e = hipMemset(c->d_slots, 0, slot_bytes);
  if (e != hipSuccess) { cleanup(); return fail(LSW_ERR_DEVICE, "clearing the launch slots failed: %s", hipGetErrorString(e)); }
  e = hipMemcpy(c->d_lin, desc.data(), desc.size() * sizeof(LinDesc), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipDeviceSynchronize();   // the pack kernels have read A
  if (e != hipSuccess) { cleanup(); return fail(LSW_ERR_DEVICE, "descriptor upload / pack failed: %s", hipGetErrorString(e)); }
  c->desc = std::move(desc);
  *out = c.release();
  return LSW_OK;
}

extern "C" void lsw_destroy(lsw_ctx* c) {
  if (!c) return;
  for (auto& kv : c->plans)
    if (kv.second.d_sel) (void)hipFree(kv.second.d_sel);
  if (c->d_apk) (void)hipFree(c->d_apk);
  if (c->d_adapter) (void)hipFree(c->d_adapter);
  if (c->d_lin) (void)hipFree(c->d_lin);
  if (c->d_slots) (void)hipFree(c->d_slots);
  delete c;
}

// ---------------------------------------------------------------------------
// plans: which linears a launch covers and where each one's items start
constexpr size_t kMaxPlans = 256;
// ---------------------------------------------------------------------------
static lsw_status get_plan(lsw_ctx* c, int kernel, int tc, const std::vector<int32_t>& layers_sorted, DevicePlan** out) {
  PlanKey key{kernel, tc, layers_sorted};
  auto it = c->plans.find(key);
  if (it != c->plans.end()) { *out = &it->second; return LSW_OK; }
  // A table stays where it is for as long as the context lives unless the caller drops them all (lsw_drop_subset_tables):
  // launches in flight and recorded HIP graphs hold its address.  A caller that walks through very many different layer
  // subsets therefore meets a limit, not a silent eviction.
  if (c->plans.size() >= kMaxPlans)
    return fail(LSW_ERR_STATE, "%zu layer-subset tables are in use (the limit per context); lsw_drop_subset_tables frees them", c->plans.size());
  const int32_t tr = kernel == 4 ? kGemvRows : kernel == 3 ? 32 : kernel == 2 ? kMfmaTileRows : kValuTileRows;   // 3 = bandwidth probe, 4 = merged decode
  std::vector<int32_t> sel, first(1, 0);
  int64_t total = 0;
  for (size_t p = 0; p < c->lin.size(); ++p) {
    if (!layers_sorted.empty() && !std::binary_search(layers_sorted.begin(), layers_sorted.end(), c->lin[p].layer))
      continue;
    sel.push_back(int32_t(p));
    total += int64_t(ceil_div(c->lin[p].out, tr)) * ceil_div(c->lin[p].in, tc);
    first.push_back(int32_t(total));
  }
  if (total > INT32_MAX) return fail(LSW_ERR_SHAPE, "more than 2^31 work items");
  DevicePlan dp;
  dp.n_sel = int32_t(sel.size());
  dp.n_items = int32_t(total);
  std::vector<int32_t> blob(sel);
  blob.insert(blob.end(), first.begin(), first.end());
  LSW_HIP(hipMalloc(reinterpret_cast<void**>(&dp.d_sel), blob.size() * sizeof(int32_t)));
  hipError_t e = hipMemcpy(dp.d_sel, blob.data(), blob.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e != hipSuccess) { (void)hipFree(dp.d_sel); return fail(LSW_ERR_DEVICE, "plan upload failed: %s", hipGetErrorString(e)); }
  c->owned_bytes += int64_t(blob.size() * sizeof(int32_t));
  auto ins = c->plans.emplace(std::move(key), dp);
  *out = &ins.first->second;
  return LSW_OK;
}

extern "C" lsw_status lsw_drop_subset_tables(lsw_ctx* c) {
  if (!c) return fail(LSW_ERR_ARG, "ctx is null");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != c->device) { (void)hipGetLastError(); return fail(LSW_ERR_STATE, "the context's device is not current"); }
  LSW_HIP(hipDeviceSynchronize());              // no launch may still be reading a table
  for (auto& kv : c->plans) {
    (void)hipFree(kv.second.d_sel);
    c->owned_bytes -= int64_t(size_t(2 * kv.second.n_sel + 1) * sizeof(int32_t));
  }
  c->plans.clear();
  return LSW_OK;
}

// the launch description over the linears of a plan, everything else zero
static LaunchPlan plan_of(const lsw_ctx* c, const DevicePlan* dp, int tile_cols, int xcd_remap) {
  LaunchPlan lp{};
  lp.lin = c->d_lin;
  lp.sel = dp->d_sel;
  lp.first = dp->d_sel + dp->n_sel;
  lp.n_sel = dp->n_sel;
  lp.n_items = dp->n_items;
  lp.tile_cols = tile_cols;
  lp.xcd_remap = xcd_remap;
  return lp;
}

// A context belongs to the device that was current when it was created; its launches and copies must run there.
static lsw_status ctx_ready(const lsw_ctx* c) {
  if (!c) return fail(LSW_ERR_ARG, "ctx is null");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return fail(LSW_ERR_DEVICE, "no current HIP device"); }
  if (dev != c->device) return fail(LSW_ERR_STATE, "the context belongs to device %d, the calling thread's current device is %d", c->device, dev);
  return LSW_OK;
}

// ---------------------------------------------------------------------------
// the switch
// ---------------------------------------------------------------------------
// layer list of a call -> sorted selection (empty = every layer)
static lsw_status select_layers(lsw_ctx* c, const int32_t* layers, int32_t n_layers, std::vector<int32_t>* sel) {
  if (n_layers < 0 || (n_layers > 0 && !layers)) return fail(LSW_ERR_ARG, "bad layer list");
  sel->clear();
  if (n_layers > 0) {
    sel->assign(layers, layers + n_layers);
    std::sort(sel->begin(), sel->end());
    for (int32_t a = 0; a < n_layers; ++a) {
      if (layer_slot(c, (*sel)[a]) < 0) return fail(LSW_ERR_ARG, "unknown layer %d", (*sel)[a]);
      if (a > 0 && (*sel)[a] == (*sel)[a - 1]) return fail(LSW_ERR_ARG, "duplicate layer %d", (*sel)[a]);
    }
    if (sel->size() == c->layer_ids.size()) sel->clear();   // every layer: the common plan
  }
  return LSW_OK;
}

// One launch over the selected layers.  t.n sizes the launch; with t_dev the kernel reads the list from device memory.
static lsw_status launch_switch(lsw_ctx* c, const std::vector<int32_t>& sel_layers, const Terms& t, LaunchSlot* slot, bool terms_on_device,
                                hipStream_t s, bool from_base = false, bool probe = false) {
  const Terms* t_dev = terms_on_device ? &slot->terms : nullptr;
  // the matrix-core kernels keep the fused rank (terms x r) in registers: up to 64 in the streaming
  // kernel, up to 256 in the chunked one
  const int n_groups = (c->r % 8 == 0) ? t.n * (c->r / 8) : 0;
  const bool mfma_fits = (c->r % 8 == 0) && n_groups <= 32;
  const bool bigk = n_groups > 8;
  int kernel = c->opt_kernel;
  if (kernel == 0) kernel = mfma_fits ? 2 : 1;
  if (kernel >= 2 && !mfma_fits)
    return fail(LSW_ERR_ARG, "matrix-core kernel needs r %% 8 == 0 and a fused rank <= 256 (r=%d, terms=%d)", c->r, t.n);
  c->last_kernel = 0;
  c->last_variant = 0;
  c->last_items = 0;
  c->last_grid = 0;
  if (t.n > 0) {
    DevicePlan* dp = nullptr;
    int tc = kernel >= 2 ? (bigk ? c->opt_tile_cols_bigk : c->opt_tile_cols) : kValuTileCols;
    int grid = c->opt_grid;
    if (grid <= 0) grid = (kernel == 2) ? c->n_cu : c->n_cu * 2;   // matrix-core: one workgroup per CU
    grid = std::max(8, (grid / 8) * 8);     // a multiple of the 8 XCDs (the kernels' block remap assumes it)
    // Per-XCD order (each XCD walks its own eighth of the item list, the tail of every eighth dealt through the pool)
    // pays where at least half of the selected weights lie in linears whose column panels per row block divide the
    // workgroups of one XCD (32): a workgroup's consecutive items then lie in the same panel, the region an XCD updates
    // stays compact, and each packed A is fetched into one L2 instead of eight.  Measured: 70B shape 47.4 against
    // 50.2 ms, 7B with bf16-stored factors 4,076 against 4,121 us; 13B shape (5 and 13.5 panels) 9,300 against 9,180 us
    // on a fresh machine, so it keeps the round-wise order.
    // Item order inside wide matrices (LSW_OPT_PANEL_GROUP): rows outermost, unless the launch runs in per-XCD order and
    // the packed A a row of items needs (fused rank x in x 2 bytes x Q parts) exceeds 1.5 MB in some matrix: then an XCD's
    // 32 concurrent items would pull more of it through the 4 MB L2 per round than survives next to the W stream (the
    // 70B `down`, 28 panels of 256 KB at 4 terms, fetched 3.57 GB where 1.92 GB are needed), and the panels are taken
    // in groups of 4.  Measured on the 70B shape: 4-term launches 48.4 against 50.0 ms.  Not for smaller operands (7B:
    // 0.8 % slower) and not in the round-wise order (13B: 2-4 % slower).
    bool per_xcd = false;
    int panel_group = 0;
    int64_t widest_q = 0;
    auto per_xcd_at = [&](int cols) {
      int64_t reuse = 0, total = 0;
      widest_q = 0;
      for (const lsw_linear& L : c->lin) {
        if (!sel_layers.empty() && !std::binary_search(sel_layers.begin(), sel_layers.end(), L.layer)) continue;
        const int64_t w = int64_t(L.out) * L.in;
        total += w;
        if ((grid / 8) % ceil_div(L.in, cols) == 0) reuse += w;
        widest_q = std::max(widest_q, int64_t(n_groups) * 8 * L.in * 2 * c->qp);
      }
      return 2 * reuse >= total;
    };
    auto q_fits = [&](int cols) { return (cols / kApkBlockCols) * ((n_groups + 1) / 2) * 8 * c->qp * 1024 <= kResidentLdsBytes; };
    if (kernel == 2 && !bigk) per_xcd = per_xcd_at(tc);
    // The resident-Q kernel on top of that where the Q of one item (8 KB per 256 columns, k-step and Q part) fits LDS.
    // fp32-stored factors only: with bf16-stored ones (half the Q bytes) the streaming kernel is as fast or faster.
    // At 3 k-steps (fused ranks 40-48) the Q of a full-width item does not fit but that of a half-width one does:
    // measured on the 70B shape 44.5 against 45.5 ms for the streaming kernel, so those launches run at half width.  Not
    // at 4 k-steps: there the resident kernel spills registers (52.9, or 50.5 with the B rows of the next item loaded
    // after the tile update, against 48.5 ms).
    bool resident = per_xcd && c->opt_resident && c->qp == 2 && q_fits(tc);
    if (kernel == 2 && !bigk && !resident && c->opt_resident && c->qp == 2 && (n_groups + 1) / 2 == 3 && tc % (2 * kApkBlockCols) == 0 &&
        q_fits(tc / 2) && per_xcd_at(tc / 2)) {
      tc /= 2;
      per_xcd = resident = true;
    } else if (kernel == 2 && !bigk) {
      per_xcd = per_xcd_at(tc);       // (widest_q of the width in use)
    }
    if (kernel == 2 && !bigk)
      panel_group = c->opt_panel_group >= 0 ? c->opt_panel_group : (per_xcd && widest_q > (3 << 19)) ? 4 : 0;
    // LSW_OPT_XCD_REMAP: 3 = automatic
    const int xcd_mode = c->opt_xcd == 3 ? (bigk || kernel != 2 ? 1 : per_xcd ? 2 : 1) : c->opt_xcd;
    lsw_status st = get_plan(c, kernel, tc, sel_layers, &dp);
    if (st != LSW_OK) return st;
    LaunchPlan lp = plan_of(c, dp, tc, xcd_mode);
    lp.from_base = from_base ? 1 : 0;
    lp.exact_one_pass = c->opt_one_pass;
    lp.pool = c->opt_pool ? slot->pool : nullptr;
    lp.pool_div = c->opt_pool == 1 ? 16 : c->opt_pool;
    lp.panel_group = panel_group;
    lp.probe = probe ? 1 : 0;
    if (probe && kernel != 2) return fail(LSW_ERR_ARG, "the switch-pattern probe needs the matrix-core kernels (r %% 8 == 0)");
    hipError_t e = (kernel == 2) ? (bigk && !probe ? launch_switch_mfma_bigk(lp, t, t_dev, c->r, c->qp, grid, s)
                                  : resident ? launch_switch_mfma_res(lp, t, t_dev, c->r, c->qp, grid, s)
                                             : launch_switch_mfma(lp, t, t_dev, c->r, c->qp, grid, s))
                                 : launch_switch_valu(lp, t, t_dev, c->r, c->qp, grid, s);
    if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "switch launch failed: %s", hipGetErrorString(e));
    c->last_kernel = kernel;
    c->last_variant = kernel == 2 ? (bigk ? 3 : resident ? 2 : 1) : 0;
    c->last_items = dp->n_items;
    c->last_grid = grid;
  }
  return LSW_OK;
}

extern "C" lsw_status lsw_switch(lsw_ctx* c, const int32_t* layers, int32_t n_layers,
                                 const int32_t* old_ids, const float* old_gates, int32_t k_old,
                                 const int32_t* new_ids, const float* new_gates, int32_t k_new,
                                 void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  std::vector<int32_t> sel_layers;
  lsw_status st = select_layers(c, layers, n_layers, &sel_layers);
  if (st != LSW_OK) return st;
  Terms t;
  std::memset(&t, 0, sizeof(t));
  st = lsw_build_terms(old_ids, old_gates, k_old, new_ids, new_gates, k_new, c->E, c->scale, t.e, t.coeff, &t.n);
  if (st != LSW_OK) return st;

  const std::vector<int32_t>& touched = sel_layers.empty() ? c->layer_ids : sel_layers;
  if (c->opt_strict) {
    for (int32_t layer : touched) {
      const LayerState& s = c->state[size_t(layer_slot(c, layer))];
      if (s.k < 0) return fail(LSW_ERR_STATE, "layer %d: the merged set lives on the device (lsw_switch_dev)", layer);
      bool same = (s.k == k_old);
      for (int32_t a = 0; same && a < k_old; ++a) {
        bool found = false;
        for (int32_t b = 0; b < s.k; ++b)
          found |= (s.ids[b] == old_ids[a] && std::memcmp(&s.gates[b], &old_gates[a], sizeof(float)) == 0);
        same = found;
      }
      if (!same) return fail(LSW_ERR_STATE, "layer %d: `old` differs from the merged state", layer);
    }
  }
  st = launch_switch(c, sel_layers, t, take_slot(c), false, static_cast<hipStream_t>(hip_stream));
  if (st != LSW_OK) return st;
  for (int32_t layer : touched) {
    LayerState& s = c->state[size_t(layer_slot(c, layer))];
    s.k = k_new;
    for (int32_t a = 0; a < k_new; ++a) { s.ids[a] = new_ids[a]; s.gates[a] = new_gates[a]; }
  }
  return LSW_OK;
}

// ---------------------------------------------------------------------------
// drift control: re-base the merged weights on a caller-kept copy of the base weights
// ---------------------------------------------------------------------------
extern "C" lsw_status lsw_set_base(lsw_ctx* c, const void* const* W_base, int32_t n_lin) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (!W_base || n_lin != int32_t(c->lin.size())) return fail(LSW_ERR_ARG, "W_base is null or n_lin differs from the %zu registered linears", c->lin.size());
  for (int32_t p = 0; p < n_lin; ++p) {
    if (!W_base[p]) return fail(LSW_ERR_ARG, "linear %d: null base copy", p);
    if (!aligned16(W_base[p])) return fail(LSW_ERR_SHAPE, "linear %d: base copy not 16-byte aligned", p);
    if (W_base[p] == c->lin[size_t(p)].W) return fail(LSW_ERR_ARG, "linear %d: the base copy is the merged weight itself", p);
  }
  for (int32_t p = 0; p < n_lin; ++p) c->desc[size_t(p)].Wbase = static_cast<const uint16_t*>(W_base[p]);
  LSW_HIP(hipDeviceSynchronize());     // no launch may be reading the table while it changes
  LSW_HIP(hipMemcpy(c->d_lin, c->desc.data(), c->desc.size() * sizeof(LinDesc), hipMemcpyHostToDevice));
  c->have_base = true;
  return LSW_OK;
}

extern "C" lsw_status lsw_rebase(lsw_ctx* c, const int32_t* layers, int32_t n_layers,
                                 const int32_t* ids, const float* gates, int32_t k, void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (!c->have_base) return fail(LSW_ERR_STATE, "lsw_rebase: no base copies registered (lsw_set_base)");
  std::vector<int32_t> sel_layers;
  lsw_status st = select_layers(c, layers, n_layers, &sel_layers);
  if (st != LSW_OK) return st;
  Terms t;
  std::memset(&t, 0, sizeof(t));
  st = lsw_build_terms(nullptr, nullptr, 0, ids, gates, k, c->E, c->scale, t.e, t.coeff, &t.n);
  if (st != LSW_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const std::vector<int32_t>& touched = sel_layers.empty() ? c->layer_ids : sel_layers;
  if (t.n == 0) {          // nothing to merge: the base weights themselves
    c->last_kernel = 0;
    c->last_items = 0;
    c->last_grid = 0;
    DevicePlan* dp = nullptr;                  // one launch: the probe's walk over the selected linears, reading the base copy
    st = get_plan(c, 3, c->opt_tile_cols, sel_layers, &dp);
    if (st != LSW_OK) return st;
    LaunchPlan lp = plan_of(c, dp, c->opt_tile_cols, c->opt_xcd ? 1 : 0);
    lp.from_base = 1;
    hipError_t e = launch_probe_inplace(lp, c->n_cu * 4, s);
    if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "copy launch failed: %s", hipGetErrorString(e));
  } else {
    st = launch_switch(c, sel_layers, t, take_slot(c), false, s, /*from_base*/ true);
    if (st != LSW_OK) return st;
  }
  for (int32_t layer : touched) {
    LayerState& ls = c->state[size_t(layer_slot(c, layer))];
    ls.k = k;
    for (int32_t a = 0; a < k; ++a) { ls.ids[a] = ids[a]; ls.gates[a] = gates[a]; }
  }
  return LSW_OK;
}

// ---------------------------------------------------------------------------
// device-resident routing: no value of the token's (ids, gates) ever visits the host
// ---------------------------------------------------------------------------
extern "C" lsw_status lsw_route_dev(lsw_ctx* c, const float* logits_dev, int32_t k, int32_t* ids_dev, float* gates_dev,
                                    void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (k < 0 || k > LSW_MAX_K || k > c->E) return fail(LSW_ERR_ARG, "lsw_route_dev: k=%d outside 0..min(%d, E=%d)", k, int(LSW_MAX_K), c->E);
  if (!logits_dev || (k > 0 && (!ids_dev || !gates_dev))) return fail(LSW_ERR_ARG, "lsw_route_dev: null pointer");
  if (k == 0) return LSW_OK;
  hipError_t e = launch_route(logits_dev, 1, c->E, k, ids_dev, gates_dev, c->d_err, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "route launch failed: %s", hipGetErrorString(e));
  return LSW_OK;
}

extern "C" lsw_status lsw_switch_dev(lsw_ctx* c, const int32_t* layers, int32_t n_layers,
                                     const int32_t* old_ids_dev, const float* old_gates_dev, int32_t k_old,
                                     const int32_t* new_ids_dev, const float* new_gates_dev, int32_t k_new,
                                     void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (c->opt_strict) return fail(LSW_ERR_STATE, "lsw_switch_dev: the host cannot check device-resident lists (strict mode is on)");
  if (k_old < 0 || k_old > LSW_MAX_K || k_old > c->E) return fail(LSW_ERR_ARG, "old: k=%d out of range", k_old);
  if (k_new < 0 || k_new > LSW_MAX_K || k_new > c->E) return fail(LSW_ERR_ARG, "new: k=%d out of range", k_new);
  if ((k_old > 0 && (!old_ids_dev || !old_gates_dev)) || (k_new > 0 && (!new_ids_dev || !new_gates_dev)))
    return fail(LSW_ERR_ARG, "null list with k > 0");
  std::vector<int32_t> sel_layers;
  lsw_status st = select_layers(c, layers, n_layers, &sel_layers);
  if (st != LSW_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Terms t;
  std::memset(&t, 0, sizeof(t));
  t.n = k_old + k_new;                       // the launch is sized for the longest list the device may build
  LaunchSlot* slot = take_slot(c);
  if (t.n > 0) {
    hipError_t e = launch_build_terms(old_ids_dev, old_gates_dev, k_old, new_ids_dev, new_gates_dev, k_new, c->E, c->scale,
                                      &slot->terms, c->d_err, s);
    if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "term builder launch failed: %s", hipGetErrorString(e));
  }
  st = launch_switch(c, sel_layers, t, slot, true, s);
  if (st != LSW_OK) return st;
  const std::vector<int32_t>& touched = sel_layers.empty() ? c->layer_ids : sel_layers;
  for (int32_t layer : touched) c->state[size_t(layer_slot(c, layer))].k = -1;     // known to the device only
  return LSW_OK;
}

extern "C" lsw_status lsw_route_batch_dev(lsw_ctx* c, const float* logits_dev, int32_t n_tokens, int32_t k, int32_t* ids_dev,
                                          float* gates_dev, void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (n_tokens < 1 || n_tokens > (1 << 24)) return fail(LSW_ERR_ARG, "lsw_route_batch_dev: n_tokens=%d outside 1..2^24", n_tokens);
  if (k < 0 || k > LSW_MAX_K || k > c->E) return fail(LSW_ERR_ARG, "lsw_route_batch_dev: k=%d outside 0..min(%d, E=%d)", k, int(LSW_MAX_K), c->E);
  if (!logits_dev || (k > 0 && (!ids_dev || !gates_dev))) return fail(LSW_ERR_ARG, "lsw_route_batch_dev: null pointer");
  if (k == 0) return LSW_OK;
  hipError_t e = launch_route(logits_dev, n_tokens, c->E, k, ids_dev, gates_dev, c->d_err, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "route launch failed: %s", hipGetErrorString(e));
  return LSW_OK;
}

// ---------------------------------------------------------------------------
// un-merged adapter path over many tokens (Eq. 2)
// ---------------------------------------------------------------------------
static int z_stride_of(const lsw_ctx* c) { return ceil_div(c->E * c->r, 16) * 16; }   // whole k-steps of 16: the pad columns hold zeros

extern "C" lsw_status lsw_enable_adapter_path(lsw_ctx* c) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (c->d_adapter) return LSW_OK;
  {   // the address of the static workspace on this device (the context's device is current: ctx_ready)
    hipError_t se = adapter_static_scratch(c->device, &c->static_scratch);
    if (se != hipSuccess) { c->static_scratch = nullptr; return fail(LSW_ERR_DEVICE, "address of the static workspace: %s", hipGetErrorString(se)); }
  }
  if (c->r % 8 != 0 || c->E * c->r > 256)
    return fail(LSW_ERR_SHAPE, "the adapter path needs r %% 8 == 0 and E * r <= 256 (E=%d, r=%d)", c->E, c->r);
  const size_t n_lin = c->lin.size();
  size_t elems = 0;
  c->atk_off.assign(n_lin, 0);
  c->bpk_off.assign(n_lin, 0);
  for (size_t p = 0; p < n_lin; ++p) {
    const lsw_linear& L = c->lin[p];
    if (L.out % 8 != 0) return fail(LSW_ERR_SHAPE, "linear %zu: the adapter path needs out %% 8 == 0 (out=%d)", p, L.out);
    if (int64_t(c->E) * c->r * ceil_div(L.out, kApkBlockCols) * kApkBlockCols * 2 * c->qp >= (int64_t(1) << 31))
      return fail(LSW_ERR_SHAPE, "linear %zu: E * r * out * 4 must stay below 2^31 bytes", p);
    c->atk_off[p] = elems;
    elems += size_t(adapter_atk_elems(c->E, c->r, L.in, c->qp));
    c->bpk_off[p] = elems;
    elems += size_t(c->E) * size_t(c->r) * size_t(ceil_div(L.out, kApkBlockCols) * kApkBlockCols) * size_t(c->qp);
  }
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->d_adapter), elems * sizeof(uint16_t));
  if (e != hipSuccess) { (void)hipGetLastError(); c->d_adapter = nullptr; return fail(LSW_ERR_NOMEM, "hipMalloc of %zu bytes for the adapter path failed", elems * 2); }
  for (size_t p = 0; p < n_lin && e == hipSuccess; ++p) {
    const lsw_linear& L = c->lin[p];
    e = launch_pack_Atk(L.A, c->d_adapter + c->atk_off[p], c->E, c->r, L.in, c->qp, nullptr);
    if (e == hipSuccess) e = launch_pack_A(L.B, c->d_adapter + c->bpk_off[p], c->E, c->r, L.out, c->qp, 1, nullptr);
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    (void)hipFree(c->d_adapter);
    c->d_adapter = nullptr;
    return fail(LSW_ERR_DEVICE, "packing the adapter-path operands failed: %s", hipGetErrorString(e));
  }
  c->owned_bytes += int64_t(elems * sizeof(uint16_t));
  return LSW_OK;
}

static int64_t adapter_ws_bytes(const lsw_ctx* c, size_t lin_index, int32_t T) {
  const int64_t N = int64_t(c->E) * c->r;
  return 4 * (int64_t(adapter_slices(T, c->lin[lin_index].in, int(N))) * T * N + int64_t(T) * z_stride_of(c));
}

extern "C" int64_t lsw_adapter_workspace_bytes(const lsw_ctx* c, int32_t lin_index, int32_t T) {
  if (!c || lin_index < 0 || size_t(lin_index) >= c->lin.size() || T < 1) {
    fail(LSW_ERR_ARG, "lsw_adapter_workspace_bytes: bad argument");
    return -1;
  }
  return adapter_ws_bytes(c, size_t(lin_index), T);
}

// the linears of `layer` in registration order (at most kAdMaxLin)
static lsw_status layer_linears(const lsw_ctx* c, int32_t layer, std::vector<int32_t>* idx) {
  idx->clear();
  for (size_t p = 0; p < c->lin.size(); ++p)
    if (c->lin[p].layer == layer) idx->push_back(int32_t(p));
  if (idx->empty()) return fail(LSW_ERR_ARG, "unknown layer %d", layer);
  if (idx->size() > size_t(kAdMaxLin)) return fail(LSW_ERR_SHAPE, "layer %d has %zu linears, one call covers at most %d", layer, idx->size(), kAdMaxLin);
  return LSW_OK;
}

extern "C" int64_t lsw_adapter_layer_workspace_bytes(const lsw_ctx* c, int32_t layer, int32_t T) {
  std::vector<int32_t> idx;
  if (!c || T < 1 || layer_linears(c, layer, &idx) != LSW_OK) {
    if (!c || T < 1) fail(LSW_ERR_ARG, "lsw_adapter_layer_workspace_bytes: bad argument");
    return -1;
  }
  int64_t total = 0;
  for (int32_t p : idx) total += adapter_ws_bytes(c, size_t(p), T);
  return total;
}

// Eq. 2's adapter sum for n linears that see the same T tokens: three launches in all (down-projections, gate tables,
// up-projections), the workspace cut into one block per linear in the given order.
static lsw_status adapter_run(lsw_ctx* c, const int32_t* lin_idx, int n, const void* const* X, int32_t T, const int32_t* ids_dev,
                              const float* gates_dev, int32_t k, void* const* Y, void* workspace, hipStream_t s) {
  if (!c->d_adapter) return fail(LSW_ERR_STATE, "the adapter path is not enabled: call lsw_enable_adapter_path first");
  if (T < 1) return fail(LSW_ERR_ARG, "T=%d < 1", T);
  if (k < 0 || k > LSW_MAX_K || k > c->E) return fail(LSW_ERR_ARG, "k=%d outside 0..min(%d, E=%d)", k, int(LSW_MAX_K), c->E);
  if (!X || !Y || !workspace || (k > 0 && (!ids_dev || !gates_dev))) return fail(LSW_ERR_ARG, "null pointer");
  if (!aligned16(workspace)) return fail(LSW_ERR_SHAPE, "the workspace is not 16-byte aligned");
  const int N = c->E * c->r, zs = z_stride_of(c);
  const int n_groups = c->E * (c->r / 8);
  const bool bigk = n_groups > 8;
  // Up-projection items: 128 tokens x some output columns.  The row operand (a token block's rows of Z, split) is set up
  // once per item, so wide items are cheaper per byte: the work is numbered in single column steps and every workgroup
  // takes one contiguous, equally long range of it (LaunchPlan::flat), cut into items only where a row of steps ends.
  const int grid = std::max(8, (c->n_cu / 8) * 8);
  const int tc = kApkBlockCols;
  AdJobs jobs{};
  jobs.n = n;
  jobs.T = T;
  LaunchPlan lp{};
  lp.n_sel = n;
  lp.tile_cols = tc;
  lp.xcd_remap = c->opt_xcd ? 1 : 0;
  lp.flat = 1;
  lp.z_stride = zs;
  char* ws = static_cast<char*>(workspace);
  int64_t n_items = 0;
  for (int i = 0; i < n; ++i) {
    const size_t p = size_t(lin_idx[i]);
    const lsw_linear& L = c->lin[p];
    if (!X[i] || !Y[i]) return fail(LSW_ERR_ARG, "linear %zu: null X or Y", p);
    if (!aligned16(X[i]) || !aligned16(Y[i])) return fail(LSW_ERR_SHAPE, "linear %zu: X or Y is not 16-byte aligned", p);
    if (int64_t(T) * L.in * 2 >= (int64_t(1) << 31) || int64_t(ceil_div(T, kMfmaTileRows)) * kMfmaTileRows * L.out * 2 >= (int64_t(1) << 31))
      return fail(LSW_ERR_SHAPE, "T=%d: X and Y (rows rounded up to %d) must stay below 2^31 bytes each", T, kMfmaTileRows);
    jobs.X[i] = static_cast<const uint16_t*>(X[i]);
    jobs.Atk[i] = c->d_adapter + c->atk_off[p];
    jobs.in[i] = L.in;
    jobs.cps[i] = adapter_chunks_per_slice(T, L.in, N);
    jobs.n_slices[i] = adapter_slices(T, L.in, N);
    jobs.Upart[i] = reinterpret_cast<float*>(ws);
    jobs.Z[i] = jobs.Upart[i] + size_t(jobs.n_slices[i]) * size_t(T) * size_t(N);
    ws += adapter_ws_bytes(c, p, T);
    LinDesc& d = lp.ad[i];
    d.W = static_cast<uint16_t*>(Y[i]);
    d.B = jobs.Z[i];
    d.Apk = c->d_adapter + c->bpk_off[p];
    d.out = T;
    d.in = L.out;
    d.ld = L.out;
    lp.ad_first[i] = int32_t(n_items);
    n_items += int64_t(ceil_div(T, kMfmaTileRows)) * ceil_div(L.out, tc);
    if (n_items > INT32_MAX) return fail(LSW_ERR_SHAPE, "more than 2^31 work items");
  }
  for (int i = n; i <= kAdMaxLin; ++i) lp.ad_first[i] = int32_t(n_items);
  lp.n_items = int32_t(n_items);
  lp.Z = jobs.Z[0];
  if (k == 0) return LSW_OK;                  // no expert selected: nothing to add
  hipError_t e = launch_adapter_down(jobs, N, c->qp, s);
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "down-projection launch failed: %s", hipGetErrorString(e));
  e = launch_adapter_gate(jobs, ids_dev, gates_dev, k, c->E, c->r, c->scale, zs, c->d_err, s);
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "gate launch failed: %s", hipGetErrorString(e));
  // the up-projections: the matrix-core switch kernels with rows = tokens and the row operand read from Z
  Terms t;
  std::memset(&t, 0, sizeof(t));
  t.n = c->E;                                // sizes the launch: E * r / 8 groups of the fused rank
  e = bigk ? launch_switch_mfma_bigk(lp, t, nullptr, c->r, c->qp, grid, s) : launch_switch_mfma(lp, t, nullptr, c->r, c->qp, grid, s);
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "up-projection launch failed: %s", hipGetErrorString(e));
  return LSW_OK;
}

extern "C" lsw_status lsw_adapter_forward(lsw_ctx* c, int32_t lin_index, const void* X_bf16, int32_t T,
                                          const int32_t* ids_dev, const float* gates_dev, int32_t k,
                                          void* Y_bf16, void* workspace, void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (!c->d_adapter) return fail(LSW_ERR_STATE, "lsw_adapter_forward: call lsw_enable_adapter_path first");
  if (lin_index < 0 || size_t(lin_index) >= c->lin.size()) return fail(LSW_ERR_ARG, "lin_index %d out of range", lin_index);
  return adapter_run(c, &lin_index, 1, &X_bf16, T, ids_dev, gates_dev, k, &Y_bf16, workspace, static_cast<hipStream_t>(hip_stream));
}

extern "C" lsw_status lsw_adapter_forward_layer(lsw_ctx* c, int32_t layer, const void* const* X_bf16, int32_t T,
                                                const int32_t* ids_dev, const float* gates_dev, int32_t k,
                                                void* const* Y_bf16, void* workspace, void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (!c->d_adapter) return fail(LSW_ERR_STATE, "lsw_adapter_forward_layer: call lsw_enable_adapter_path first");
  std::vector<int32_t> idx;
  if (lsw_status st = layer_linears(c, layer, &idx)) return st;
  return adapter_run(c, idx.data(), int(idx.size()), X_bf16, T, ids_dev, gates_dev, k, Y_bf16, workspace, static_cast<hipStream_t>(hip_stream));
}

extern "C" lsw_status lsw_adapter_forward_static(lsw_ctx* c, int32_t lin_index, const void* X_bf16, int32_t T,
                                                 const int32_t* ids_dev, const float* gates_dev, int32_t k,
                                                 void* Y_bf16, void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (!c->d_adapter || !c->static_scratch) return fail(LSW_ERR_STATE, "lsw_adapter_forward_static: call lsw_enable_adapter_path first");
  if (lin_index < 0 || size_t(lin_index) >= c->lin.size()) return fail(LSW_ERR_ARG, "lin_index %d out of range", lin_index);
  if (T < 1) return fail(LSW_ERR_ARG, "T=%d < 1", T);
  const int64_t need = lsw_adapter_workspace_bytes(c, lin_index, T);
  if (need < 0 || need > int64_t(kStaticScratchBytes))
    return fail(LSW_ERR_SHAPE, "T=%d tokens need %lld bytes of workspace, the static one holds %lld: use lsw_adapter_forward with a workspace of the caller's",
                T, (long long)need, (long long)kStaticScratchBytes);
  // same checks, same three launches; the kernels get the device address looked up at lsw_enable_adapter_path
  return lsw_adapter_forward(c, lin_index, X_bf16, T, ids_dev, gates_dev, k, Y_bf16, c->static_scratch, hip_stream);
}

extern "C" lsw_status lsw_dev_status(lsw_ctx* c, int32_t* flags) {
  if (!flags) return fail(LSW_ERR_ARG, "null argument");
  if (lsw_status ready = ctx_ready(c)) return ready;
  LSW_HIP(hipMemcpy(flags, c->d_err, sizeof(int32_t), hipMemcpyDeviceToHost));     // waits for earlier work on the null stream only
  return LSW_OK;
}

extern "C" lsw_status lsw_gemv_bf16(const void* W_bf16, const void* x_bf16, float* y_fp32, int32_t out, int32_t in,
                                    void* hip_stream) {
  if (!W_bf16 || !x_bf16 || !y_fp32) return fail(LSW_ERR_ARG, "null pointer");
  if (out < 1 || in < 8 || in % 8 != 0) return fail(LSW_ERR_SHAPE, "out=%d, in=%d: in must be a positive multiple of 8", out, in);
  if (!aligned16(W_bf16) || !aligned16(x_bf16)) return fail(LSW_ERR_SHAPE, "W or x is not 16-byte aligned");
  hipError_t e = launch_gemv(static_cast<const uint16_t*>(W_bf16), static_cast<const uint16_t*>(x_bf16), y_fp32, out, in, in, 512,
                             static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "gemv launch failed: %s", hipGetErrorString(e));
  return LSW_OK;
}

// ---------------------------------------------------------------------------
// bandwidth probe over the registered weights
// ---------------------------------------------------------------------------
extern "C" lsw_status lsw_probe_inplace(lsw_ctx* c, int32_t waves_per_cu, void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (waves_per_cu < 0 || waves_per_cu > 16) return fail(LSW_ERR_ARG, "waves_per_cu=%d outside 0..16", waves_per_cu);
  if (waves_per_cu == 0) {          // the switch kernel's own launch for a token with two old and two new experts, work taken out
    Terms t;
    std::memset(&t, 0, sizeof(t));
    t.n = std::min(4, c->E);
    return launch_switch(c, std::vector<int32_t>(), t, take_slot(c), false, static_cast<hipStream_t>(hip_stream), false, true);
  }
  DevicePlan* dp = nullptr;
  lsw_status st = get_plan(c, 3, c->opt_tile_cols, std::vector<int32_t>(), &dp);
  if (st != LSW_OK) return st;
  const LaunchPlan lp = plan_of(c, dp, c->opt_tile_cols, c->opt_xcd ? 1 : 0);
  hipError_t e = launch_probe_inplace(lp, c->n_cu * waves_per_cu, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "probe launch failed: %s", hipGetErrorString(e));
  return LSW_OK;
}

extern "C" lsw_status lsw_probe_matrix_loop(int32_t iters, int32_t launches, int32_t copies_per_group, int32_t zero_operands, double* ns_per_group) {
  if (!ns_per_group || iters < 1 || iters > (1 << 20) || launches < 1 || launches > 1000 || copies_per_group < 0 || copies_per_group > 2)
    return fail(LSW_ERR_ARG, "lsw_probe_matrix_loop: bad argument");
  int dev = 0;
  hipDeviceProp_t prop;
  LSW_HIP(hipGetDevice(&dev));
  LSW_HIP(hipGetDeviceProperties(&prop, dev));
  const int grid = prop.multiProcessorCount;
  void *out = nullptr, *pin = nullptr, *qsrc = nullptr;
  hipEvent_t a = nullptr, b = nullptr;
  auto release = [&]() {
    if (out) (void)hipFree(out);
    if (pin) (void)hipFree(pin);
    if (qsrc) (void)hipFree(qsrc);
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
  };
  std::vector<uint32_t> hp(32 * 64 * 4);
  for (size_t i = 0; i < hp.size(); ++i) hp[i] = ((uint32_t(i + 1) * 2246822519u) & 0x0fff0fffu) | 0x3c00bc00u;     // bf16 pairs near +-1
  hipError_t e = hipMalloc(&out, size_t(grid) * 256 * 16);
  if (e == hipSuccess) e = hipMalloc(&pin, hp.size() * 4);
  if (e == hipSuccess) e = hipMalloc(&qsrc, size_t(4) << 20);
  if (e != hipSuccess) { (void)hipGetLastError(); release(); return fail(LSW_ERR_NOMEM, "lsw_probe_matrix_loop: device allocation failed"); }
  e = hipMemcpy(pin, hp.data(), hp.size() * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemset(qsrc, 0x3c, size_t(4) << 20);
  if (e == hipSuccess) e = hipEventCreate(&a);
  if (e == hipSuccess) e = hipEventCreate(&b);
  for (int i = 0; i < 2 && e == hipSuccess; ++i) e = launch_probe_matrix_loop(out, pin, qsrc, grid, iters, copies_per_group, zero_operands, nullptr);
  if (e == hipSuccess) e = hipEventRecord(a, nullptr);
  for (int i = 0; i < launches && e == hipSuccess; ++i) e = launch_probe_matrix_loop(out, pin, qsrc, grid, iters, copies_per_group, zero_operands, nullptr);
  if (e == hipSuccess) e = hipEventRecord(b, nullptr);
  if (e == hipSuccess) e = hipEventSynchronize(b);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
  release();
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "lsw_probe_matrix_loop: %s", hipGetErrorString(e));
  *ns_per_group = double(ms) * 1e6 / (double(launches) * iters * 64.0);
  return LSW_OK;
}

// ---------------------------------------------------------------------------
// merged decode, state, options
// ---------------------------------------------------------------------------
extern "C" lsw_status lsw_merged_gemv(lsw_ctx* c, int32_t lin_index, const void* x_bf16, float* y_fp32,
                                      void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (lin_index < 0 || size_t(lin_index) >= c->lin.size()) return fail(LSW_ERR_ARG, "lin_index %d out of range", lin_index);
  if (!x_bf16 || !y_fp32) return fail(LSW_ERR_ARG, "null vector");
  if (!aligned16(x_bf16)) return fail(LSW_ERR_SHAPE, "x is not 16-byte aligned");
  const lsw_linear& L = c->lin[size_t(lin_index)];
  hipError_t e = launch_gemv(static_cast<const uint16_t*>(L.W), static_cast<const uint16_t*>(x_bf16), y_fp32,
                             L.out, L.in, c->desc[size_t(lin_index)].ld, c->opt_gemv_grid > 0 ? c->opt_gemv_grid : c->n_cu * 2,
                             static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "gemv launch failed: %s", hipGetErrorString(e));
  return LSW_OK;
}

extern "C" lsw_status lsw_merged_gemv_all(lsw_ctx* c, const void* x_all_bf16, float* y_all_fp32, void* hip_stream) {
  if (lsw_status ready = ctx_ready(c)) return ready;
  if (!x_all_bf16 || !y_all_fp32) return fail(LSW_ERR_ARG, "null vector");
  if (!aligned16(x_all_bf16)) return fail(LSW_ERR_SHAPE, "x is not 16-byte aligned");
  DevicePlan* dp = nullptr;
  lsw_status st = get_plan(c, 4, 1 << 30, std::vector<int32_t>(), &dp);   // items: blocks of rows, whole rows wide
  if (st != LSW_OK) return st;
  const LaunchPlan lp = plan_of(c, dp, 1 << 30, c->opt_xcd ? 1 : 0);
  int grid = c->opt_gemv_grid > 0 ? c->opt_gemv_grid : c->n_cu * 2;
  grid = std::max(8, (grid / 8) * 8);
  hipError_t e = launch_gemv_all(lp, static_cast<const uint16_t*>(x_all_bf16), y_all_fp32, grid,
                                 static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(LSW_ERR_DEVICE, "gemv launch failed: %s", hipGetErrorString(e));
  return LSW_OK;
}

extern "C" lsw_status lsw_get_state(const lsw_ctx* c, int32_t layer, int32_t* ids, float* gates, int32_t* k) {
  if (!c || !k) return fail(LSW_ERR_ARG, "null argument");
  int slot = layer_slot(c, layer);
  if (slot < 0) return fail(LSW_ERR_ARG, "unknown layer %d", layer);
  const LayerState& s = c->state[size_t(slot)];
  if (s.k < 0) return fail(LSW_ERR_STATE, "layer %d: the merged set lives on the device (lsw_switch_dev)", layer);
  if (s.k > 0 && (!ids || !gates)) return fail(LSW_ERR_ARG, "null output");
  *k = s.k;
  for (int32_t a = 0; a < s.k; ++a) { ids[a] = s.ids[a]; gates[a] = s.gates[a]; }
  return LSW_OK;
}

extern "C" lsw_status lsw_set_option(lsw_ctx* c, int32_t option, int64_t value) {
  if (!c) return fail(LSW_ERR_ARG, "ctx is null");
  switch (option) {
    case LSW_OPT_KERNEL:
      if (value < 0 || value > 2) return fail(LSW_ERR_ARG, "kernel option %lld outside 0..2", (long long)value);
      if (value >= 2 && c->r % 8 != 0) return fail(LSW_ERR_ARG, "matrix-core kernel needs r %% 8 == 0");
      c->opt_kernel = int(value);
      return LSW_OK;
    case LSW_OPT_STRICT_STATE:
      c->opt_strict = value != 0;
      return LSW_OK;
    case LSW_OPT_GRID:
      if (value < 0 || value > (1 << 20)) return fail(LSW_ERR_ARG, "grid option out of range");
      c->opt_grid = int(value);
      return LSW_OK;
    case LSW_OPT_TILE_COLS:
      if (value < kApkBlockCols || value > (1 << 20) || value % kApkBlockCols != 0)
        return fail(LSW_ERR_ARG, "tile columns must be a multiple of %d", kApkBlockCols);
      c->opt_tile_cols = int(value);
      c->opt_tile_cols_bigk = int(value);
      return LSW_OK;
    case LSW_OPT_XCD_REMAP:
      if (value < 0 || value > 3) return fail(LSW_ERR_ARG, "XCD order must be 0..3");
      c->opt_xcd = int(value);
      return LSW_OK;
    case LSW_OPT_RESIDENT_Q:
      c->opt_resident = value != 0;
      return LSW_OK;
    case LSW_OPT_PANEL_GROUP:
      if (value < -1 || value > 1024) return fail(LSW_ERR_ARG, "panel group out of range");
      c->opt_panel_group = int(value);
      return LSW_OK;
    case LSW_OPT_XCD_POOL:
      if (value < 0 || value > (1 << 20)) return fail(LSW_ERR_ARG, "pool option out of range");
      c->opt_pool = int(value);
      return LSW_OK;
    case LSW_OPT_ONE_PASS:
      c->opt_one_pass = value != 0;
      return LSW_OK;
    case LSW_OPT_GEMV_GRID:
      if (value < 0 || value > (1 << 20)) return fail(LSW_ERR_ARG, "grid option out of range");
      c->opt_gemv_grid = int(value);
      return LSW_OK;
    default:
      return fail(LSW_ERR_ARG, "unknown option %d", option);
  }
}

extern "C" int64_t lsw_query(const lsw_ctx* c, int32_t what) {
  if (!c) return -1;
  switch (what) {
    case LSW_Q_N_LINEARS: return int64_t(c->lin.size());
    case LSW_Q_N_LAYERS: return int64_t(c->layer_ids.size());
    case LSW_Q_LAST_KERNEL: return c->last_kernel;
    case LSW_Q_LAST_ITEMS: return c->last_items;
    case LSW_Q_LAST_GRID: return c->last_grid;
    case LSW_Q_PACKED_BYTES: return c->owned_bytes;
    case LSW_Q_GEMV_X_ELEMS: return c->x_elems;
    case LSW_Q_GEMV_Y_ELEMS: return c->y_elems;
    case LSW_Q_LAST_VARIANT: return c->last_variant;
    default: return -1;
  }
}
