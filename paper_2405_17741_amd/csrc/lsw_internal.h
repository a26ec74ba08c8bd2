// Internal declarations shared by the host side and the kernels of liblsw.
#ifndef LSW_INTERNAL_H
#define LSW_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lsw.h"
#include "lsw_tuning.h"

#if defined(__HIPCC__) || defined(__HIP__)
#define LSW_HD __host__ __device__
#else
#define LSW_HD
#endif

namespace lsw {

constexpr int kMaxTerms = 2 * LSW_MAX_K;  // old + new lists

// Device-side descriptor of one adapted linear.
struct LinDesc {
  uint16_t*       W;      // bf16 [out, in]
  const void*     A;      // fp32 or bf16 [E, r, in]
  const void*     B;      // fp32 or bf16 [E, out, r]
  const uint16_t* Apk;    // packed A for the matrix-core kernel (see pack kernel), or null
  const uint16_t* Wbase;  // caller-kept copy of the weights with nothing merged (lsw_set_base), or null
  int32_t         out;
  int32_t         in;
  int32_t         ld;     // elements between the starts of consecutive rows of W (and of Wbase), >= in
  int64_t         x_off;  // element offset of this linear's input in the back-to-back x of lsw_merged_gemv_all
  int64_t         y_off;  // element offset of its output in the back-to-back y
};

// The fused low-rank update of one switch: sum over n terms of coeff * B[e] @ A[e].
// Passed to the kernel by value (no device write, no host sync per token).
struct Terms {
  int32_t n;
  int32_t e[kMaxTerms];
  float   coeff[kMaxTerms];
};

// Work decomposition.  The selected linears are listed in `sel` (index into the
// descriptor table); first[s] is the number of the first item of sel[s] and
// first[n_sel] the total.  Linear p has ceil(out/TM) x ceil(in/CW) items, rows outermost.
struct Item {
  int32_t lin;    // index into the descriptor table
  int32_t row0;
  int32_t col0;
};

LSW_HD inline int32_t ceil_div(int32_t a, int32_t b) { return a / b + (a % b != 0); }   // a >= 0, b > 0; no overflow near 2^31

// Bytes from the first element of a [out, in] matrix with leading dimension ld to the end of its last row: what the
// kernels give the hardware as the size of the buffer, so that rows past the end fall outside it.  Below 2^31 (checked
// when the linear is registered).
LSW_HD inline int32_t w_extent_bytes(int32_t out, int32_t in, int32_t ld) { return ((out - 1) * ld + in) * 2; }

// Largest s with first[s] <= item  (first[] is non-decreasing, first[0] == 0, item < first[n_sel]).
LSW_HD inline int32_t find_segment(const int32_t* first, int32_t n_sel, int32_t item) {
  int32_t lo = 0, hi = n_sel;          // invariant: first[lo] <= item < first[hi]
  while (hi - lo > 1) {
    int32_t mid = (lo + hi) >> 1;
    if (first[mid] <= item) lo = mid; else hi = mid;
  }
  return lo;
}

// Item `local` of a linear -> its first row and column.  Row-major over (row block, column panel) by default.  With
// group > 0 and more than `group` column panels the panels are taken in groups of `group` (the last one may be
// narrower): all row blocks of one group, row-major, before the next group, so that the part of the packed A operand
// a run of consecutive items needs stays small.
LSW_HD inline void decode_item(int32_t local, int32_t out, int32_t in, int32_t tile_rows, int32_t tile_cols, int32_t group,
                               int32_t* row0, int32_t* col0) {
  const int32_t ncc = ceil_div(in, tile_cols);
  if (group <= 0 || ncc <= group) {
    *row0 = (local / ncc) * tile_rows;
    *col0 = (local % ncc) * tile_cols;
    return;
  }
  const int32_t per_group = ceil_div(out, tile_rows) * group;      // items of a full group
  const int32_t g = local / per_group;
  const int32_t width = (ncc - g * group < group) ? ncc - g * group : group;
  const int32_t l = local - g * per_group;
  *row0 = (l / width) * tile_rows;
  *col0 = (g * group + l % width) * tile_cols;
}

// Per-XCD order of a matrix-core launch: XCD x (workgroups x, x + 8, ...: the hardware deals workgroups round-robin)
// owns items [x * per, (x + 1) * per); its grid / 8 workgroups take consecutive items per round, except that the last
// pool_len items of every range form a pool dealt out one by one through an atomic counter (claim g -> walk_pool_item).
// A pool only where every workgroup of every XCD keeps at least two static items (the same answer in all workgroups).
struct WalkShare {
  int32_t first;        // the workgroup's first item (none if it is not below static_end: never with a pool)
  int32_t step;         // distance of its consecutive static items
  int32_t static_end;   // end of the statically dealt part of its XCD's range
  int32_t per;          // items per range (the last range may be shorter)
  int32_t pool_len;     // items every range gives to the pool (its last ones); 0 = no pool
};

LSW_HD inline WalkShare walk_share(int32_t n_items, int32_t grid, int32_t block, bool pool, int32_t pool_div) {
  WalkShare w;
  w.step = grid >> 3;
  w.per = ceil_div(n_items, 8);
  w.pool_len = w.per / (pool_div > 1 ? pool_div : 1);
  if (!pool || n_items - 7 * w.per - w.pool_len < 2 * w.step) w.pool_len = 0;
  const int32_t xcd = block & 7;
  const int32_t range_end = (xcd + 1) * w.per < n_items ? (xcd + 1) * w.per : n_items;
  w.static_end = range_end - w.pool_len;
  w.first = xcd * w.per + (block >> 3);
  return w;
}

// pool claim g -> item: claims go round the eight ranges, position g / 8 of the range's pool part; -1 when the pool is empty
LSW_HD inline int32_t walk_pool_item(int32_t n_items, int32_t per, int32_t pool_len, int32_t g) {
  if (g < 0 || g >= 8 * pool_len) return -1;
  const int32_t range_end = ((g & 7) + 1) * per < n_items ? ((g & 7) + 1) * per : n_items;
  return range_end - pool_len + (g >> 3);
}

constexpr int kResidentLdsBytes = 128 * 1024;   // LDS the resident-Q matrix-core kernel may use for one item's Q
constexpr int kProbeLdsBytes = 96 * 1024;       // LDS the switch-pattern probe reserves: more than half of a CU's 160 KB

// Tile shapes of the two switch kernels (rows x columns of one work item).
constexpr int kValuTileRows = 64,  kValuTileCols = 128;
constexpr int kMfmaTileRows = 128, kMfmaTileCols = 1024;   // 4 waves x 32 rows; default item width (LSW_OPT_TILE_COLS overrides)
constexpr int kMfmaBigkTileCols = 4096;                     // default item width of the chunked (fused rank > 64) matrix-core kernel
constexpr int kGemvRows = 4;                                // rows of one wave's block in the merged-decode kernels
constexpr int kApkBlockCols = 256;   // column block of the packed A layout = columns per matrix-core step

// Flat order (LaunchPlan::flat): the work is numbered in units of one column step; the workgroup at place i of the
// XCD-contiguous order (XCD x = workgroups x, x + 8, ...: place = (block % 8) * (grid / 8) + block / 8) takes the units
// [n * i / grid, n * (i + 1) / grid): all ranges equal to within one unit, XCD x on the x-th eighth of the numbering.
LSW_HD inline void flat_range(int32_t n_units, int32_t grid, int32_t block, int32_t* first, int32_t* end) {
  const long long place = (long long)(block & 7) * (grid >> 3) + (block >> 3);
  *first = int32_t((long long)n_units * place / grid);
  *end = int32_t((long long)n_units * (place + 1) / grid);
}
// A range is worked off as items: the item that starts at unit `unit` (column col0 of a matrix with `in` columns) takes
// every unit up to the end of its row of units or of the range, whichever comes first.  Returns its length in units.
LSW_HD inline int32_t flat_item_units(int32_t in, int32_t col0, int32_t unit, int32_t range_end) {
  const int32_t to_row_end = ceil_div(in - col0, kApkBlockCols), to_range_end = range_end - unit;
  return to_row_end < to_range_end ? to_row_end : to_range_end;
}

constexpr int kAdMaxLin = 8;    // linears one launch of the adapter path (lsw_adapter_forward_layer) covers at most

struct LaunchPlan {             // device pointers + counts for one launch
  const LinDesc* lin;
  const int32_t* sel;
  const int32_t* first;
  int32_t n_sel;
  int32_t n_items;
  int32_t tile_cols;            // columns of one work item (matrix-core kernel: a multiple of kApkBlockCols)
  int32_t xcd_remap;            // 0: workgroup b takes items b, b + grid, ...; 1: each XCD takes a contiguous eighth of every
                                // grid-wide round of items; 2 (k_switch_mfma): each XCD walks its own eighth of the list
  int32_t from_base;            // 1: the switch kernels read Wbase instead of W (and still write W): lsw_rebase
  int32_t exact_one_pass;       // 1: bf16-stored factors of a rank that is a multiple of 16 run one matrix-core pass (chunked kernel)
  // Adapter-path mode of the matrix-core kernels (Z != null): up to kAdMaxLin matrices described by `ad` (W = the
  // [T, out] activations to add to, Apk = the packed B^T of the linear, B = that linear's Z, out = T, in = ld = out
  // features), ad_first[i] = number of the first work item of ad[i]; n_sel = how many; lin/sel/first are unused.
  // The row operand is not coeff * B but row t of Z (fp32 [T, z_stride]: the gated down-projection of token t, all
  // experts side by side), and the fused rank runs over all E * r columns of Z.
  const float* Z;               // non-null = adapter mode (the Z of ad[0])
  int32_t z_stride;
  LinDesc ad[kAdMaxLin];
  int32_t ad_first[kAdMaxLin + 1];
  int32_t flat;                 // 1 (adapter mode of k_switch_mfma and k_switch_mfma_bigk): the items are numbered in units of one column step
                                // (tile_cols = kApkBlockCols) and every workgroup takes ONE contiguous range of the numbering,
                                // all ranges equal to within a step; a range is worked off as items that each run to the end of
                                // their row of units or of the range (walk_init_flat, mfma_load_item)
  // Per-XCD order of k_switch_mfma / k_switch_mfma_res: two zeroed counters in device memory ([0] items claimed from the shared pool, [1] workgroups
  // finished; the kernel leaves both at zero), or null for a purely static split of the items.
  int32_t* pool;
  int32_t pool_div;             // every XCD range gives its last 1/pool_div to the pool
  int32_t panel_group;          // column panels per group in the item order of a linear (see decode_item); 0 = row-major
  int32_t probe;                // 1 (k_switch_mfma, k_switch_mfma_res): the kernel's walk and W traffic only, no operand loads, no
                                // matrix work; every value is rewritten as it is (lsw_probe_inplace with waves_per_cu = 0)
};

// Kernel launchers (one .hip file per kernel family).  All return the hipError of the launch.
// t.n sizes the launch; with t_dev != null the kernels read the list (possibly shorter, or empty) from device memory
// qp: 2 = fp32-stored factors (split into two bf16 parts on the matrix cores), 1 = bf16-stored factors
hipError_t launch_switch_valu(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int qp, int grid, hipStream_t s);
hipError_t launch_switch_mfma(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int qp, int grid, hipStream_t s);
hipError_t launch_switch_mfma_res(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int qp, int grid, hipStream_t s);
hipError_t launch_switch_mfma_bigk(const LaunchPlan& p, const Terms& t, const Terms* t_dev, int r, int qp, int grid, hipStream_t s);
hipError_t launch_route(const float* logits, int n_tokens, int E, int k, int32_t* ids, float* gates, int32_t* err, hipStream_t s);
hipError_t launch_build_terms(const int32_t* old_ids, const float* old_gates, int k_old, const int32_t* new_ids,
                              const float* new_gates, int k_new, int E, float scale, Terms* out, int32_t* err, hipStream_t s);
hipError_t launch_probe_inplace(const LaunchPlan& p, int grid, hipStream_t s);
hipError_t launch_probe_matrix_loop(void* out, const void* pin, const void* qsrc, int grid, int iters, int copies, int zero_operands, hipStream_t s);
// transposed = 0: source A [E][r][in] (columns = in);  1: source B [E][out][r] read as B^T [E][r][out] (columns = out)
hipError_t launch_pack_A(const void* A, uint16_t* Apk, int E, int r, int in, int qp, int transposed, hipStream_t s);
// adapter path (Eq. 2 for many tokens)
constexpr size_t kStaticScratchBytes = size_t(32) << 20;          // workspace limit of lsw_adapter_forward_static (a device array of this size per GPU)
hipError_t adapter_static_scratch(int device, void** ptr);        // its address on `device`, which must be the current device
int64_t adapter_atk_elems(int E, int r, int in, int qp);          // bf16 elements of the down-projection layout of one linear
int adapter_slices(int T, int in, int N);                         // partial sums the down-projection of N = E * r rows is cut into
hipError_t launch_pack_Atk(const void* A, uint16_t* Atk, int E, int r, int in, int qp, hipStream_t s);
// the linears one call of the adapter path covers (all with the same T tokens, the same per-token lists)
struct AdJobs {
  int32_t n;                       // linears, 1..kAdMaxLin
  int32_t T;
  const uint16_t* X[kAdMaxLin];    // bf16 [T, in]
  const uint16_t* Atk[kAdMaxLin];  // down-projection layout of the linear's A
  float* Upart[kAdMaxLin];         // partial sums [n_slices][T][N]
  float* Z[kAdMaxLin];             // gate table [T][z_stride]
  int32_t in[kAdMaxLin];
  int32_t cps[kAdMaxLin];          // 64-column chunks per slice
  int32_t n_slices[kAdMaxLin];
  int32_t first[kAdMaxLin + 1];    // first workgroup of each linear in the down-projection launch
};
hipError_t launch_adapter_down(const AdJobs& jobs, int N, int qp, hipStream_t s);      // fills first[] itself
hipError_t launch_adapter_gate(const AdJobs& jobs, const int32_t* ids, const float* gates, int k, int E, int r,
                               float scale, int z_stride, int32_t* err, hipStream_t s);
int adapter_chunks_per_slice(int T, int in, int N);
hipError_t launch_gemv(const uint16_t* W, const uint16_t* x, float* y, int out, int in, int ld, int grid_cap, hipStream_t s);
hipError_t launch_gemv_all(const LaunchPlan& p, const uint16_t* x_all, float* y_all, int grid, hipStream_t s);

}  // namespace lsw
#endif
