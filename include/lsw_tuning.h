/*
 * lsw_tuning.h -- tuning knobs, diagnostics and host-side test hooks of liblsw.
 *
 * Nothing here is needed to run the adapter switch (lsw.h is the interface of the method).  Declared here: the
 * launch-shape options of lsw_set_option, a bandwidth probe that gives a switch latency its yardstick, and the work
 * decomposition of a launch (the tiles Sec. 3.4 hands to thread blocks) as pure host functions, so that tests can
 * check on the CPU that every weight element is covered exactly once.  All of it is stable only as far as the
 * kernels it describes are.
 */
#ifndef LSW_TUNING_H
#define LSW_TUNING_H

#include "lsw.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Launch-shape options for lsw_set_option (options 1 and 2 are in lsw.h).  None of them changes a result bit. */
enum {
  LSW_OPT_GRID = 3,          /* workgroups per launch; 0 = automatic (one matrix-core workgroup per CU) */
  LSW_OPT_TILE_COLS = 4,     /* matrix-core kernel: columns per work item, a multiple of 256 */
  LSW_OPT_XCD_REMAP = 5,     /* order of the work items over the 8 XCDs: 0 = workgroup b takes items b, b + grid, ...; 1 = each
                                XCD takes a contiguous share of every round of items; 2 = matrix-core kernel for fused ranks
                                up to 64: each XCD walks its own eighth of the whole item list (the resident-A kernel
                                always does); 3 (default) = 2 where most weights lie in matrices of 4, 8, 16 or 32 column
                                panels, else 1 */
  LSW_OPT_GEMV_GRID = 6,     /* workgroups of the merged-decode launches; 0 = automatic (2 per CU) */
  LSW_OPT_ONE_PASS = 7,      /* 1 (default): bf16-stored factors of a rank that is a multiple of 16 run ONE matrix-core pass
                                when the fused rank exceeds 64 (bare B A products, gates applied in fp32 between the terms);
                                0: two passes with the gate folded into B (what every other rank gets) */
  LSW_OPT_RESIDENT_Q = 8,    /* matrix-core kernel for fused ranks up to 64 and fp32-stored factors: 1 (default) = where the A
                                operand of one work item fits LDS and most weights lie in matrices of 4, 8, 16 or 32 column
                                panels, A is kept in LDS across the items of a panel and each XCD walks its own eighth of
                                the items; 0 = always the kernel that streams A per step */
  LSW_OPT_XCD_POOL = 9,      /* per-XCD launches: 1 (default) = the last sixteenth of every XCD's items forms a pool that workgroups
                                draw from once their own share is done (XCDs differ in speed by 2-3 %); 0 = all items dealt
                                statically; n >= 2 = the last 1/n instead */
  LSW_OPT_PANEL_GROUP = 10   /* matrix-core kernels for fused ranks up to 64: order of the items inside a matrix with many
                                column panels (lsw_worklist_item_grouped); -1 (default) = chosen per launch so that the
                                packed A operand of one group stays within 2 MB, 0 = rows outermost, n = groups of n */
};

/*
 * Bandwidth probe for callers that cannot judge a switch latency without a yardstick (benchmarks): one in-place pass
 * over every registered W with no factor traffic and no matrix work: each bf16 is widened, has +0.0f added, is rounded
 * back and stored, so every finite value is unchanged (only a negative zero becomes +0).
 *   waves_per_cu = 1..16  that many single-wave workgroups per CU walk 32-row items in the switch's 32 x 256 steps.
 *   waves_per_cu = 0      the switch's own launch: the matrix-core switch kernel (4-wave workgroups, one per CU, its item
 *                         order, item pool and per-step schedule of stores and loads) with the operand loads and the
 *                         matrix instructions taken out.  What this sustains (4 bytes per weight / elapsed time) is the
 *                         ceiling of the switch's access pattern on the same tensors.
 * Asynchronous on hip_stream.  Errors: LSW_ERR_ARG, LSW_ERR_DEVICE.
 */
lsw_status lsw_probe_inplace(lsw_ctx* ctx, int32_t waves_per_cu, void* hip_stream);

/*
 * What the matrix cores sustain on the inner loop of the three-pass kernel for fused ranks above 64, with nothing around
 * it: per group 4 LDS reads + 6 v_mfma_f32_32x32x16_bf16 (192 matrix-pipe cycles), 4 waves per workgroup, one workgroup
 * per CU, no weight traffic, no barriers; `copies_per_group` (0..2) LDS-DMA copies of 1 KB ride along as in the kernel;
 * zero_operands != 0 multiplies zeros (the chip then holds a higher clock).  Runs 2 + `launches` launches of `iters`
 * chunk quadruples (64 groups each) on the current device, synchronously, and stores the mean nanoseconds per group of
 * the timed ones in *ns_per_group.  A switch of fused rank K over n weights needs n / 8192 x K / 4 groups per CU-wave,
 * i.e. at least n x K / (8192 x 4 x 1024 waves) x ns_per_group: the ceiling the power limit of the part sets for
 * that kernel, below the datasheet rate.  Allocates about 5 MB of device memory for the duration of the call.
 * Errors: LSW_ERR_ARG, LSW_ERR_NOMEM, LSW_ERR_DEVICE.
 */
lsw_status lsw_probe_matrix_loop(int32_t iters, int32_t launches, int32_t copies_per_group, int32_t zero_operands, double* ns_per_group);

/*
 * The work decomposition of one launch, as a pure function of the shapes: linear p is cut into
 * ceil(out/tile_rows) x ceil(in/tile_cols) items, numbered linear by linear, rows outermost.  Host helpers, no
 * device.  The kernels decode an item number with the same routine.
 */
int64_t    lsw_worklist_size(const int32_t* out, const int32_t* in, int32_t n_lin,
                             int32_t tile_rows, int32_t tile_cols);            /* -1 on a bad argument */
lsw_status lsw_worklist_item(const int32_t* out, const int32_t* in, int32_t n_lin,
                             int32_t tile_rows, int32_t tile_cols, int64_t item,
                             int32_t* lin, int32_t* row0, int32_t* n_rows, int32_t* col0, int32_t* n_cols);
/* The same with the column panels of a linear taken in groups of panel_group (LSW_OPT_PANEL_GROUP): inside a linear
 * that has more panels than that, all row blocks of the first panel_group panels come first (rows outermost), then
 * those of the next group, and so on; the last group may be narrower.  panel_group = 0 is lsw_worklist_item. */
lsw_status lsw_worklist_item_grouped(const int32_t* out, const int32_t* in, int32_t n_lin,
                                     int32_t tile_rows, int32_t tile_cols, int32_t panel_group, int64_t item,
                                     int32_t* lin, int32_t* row0, int32_t* n_rows, int32_t* col0, int32_t* n_cols);

/*
 * Which work items a workgroup of a per-XCD launch (LSW_OPT_XCD_REMAP) takes, as a pure function of the counts; host
 * helpers, no device; the kernels use the same routines.  XCD x = workgroups x, x + 8, ... owns items
 * [x * per, (x + 1) * per), per = ceil(n_items / 8); workgroup `block` takes first, first + step, ... below static_end;
 * the last pool_len items of every range go to the pool, where claim number g (an atomic counter at run time) stands
 * for lsw_walk_pool_item(g), or for nothing (-1) once the pool is empty.  pool_div <= 0 = no pool.
 * share = {first, step, static_end, per, pool_len}.  LSW_ERR_ARG unless n_items >= 0, grid a positive multiple of 8
 * and 0 <= block < grid.
 */
lsw_status lsw_walk_share(int32_t n_items, int32_t grid, int32_t block, int32_t pool_div, int32_t share[5]);
int32_t    lsw_walk_pool_item(int32_t n_items, int32_t grid, int32_t pool_div, int32_t claim);

/*
 * The work decomposition of the up-projection of the prompt path (lsw_adapter_forward*), as a pure host function; the
 * kernels use the same routines.  The matrices are the outputs Y of the call's linears, rows[i] = tokens, cols[i] = out
 * features; the work is numbered in units of 128 rows x 256 columns, matrix by matrix, rows outermost.  Workgroup `block`
 * of `grid` takes ONE contiguous range of the numbering (all ranges equal to within a unit; XCD x = workgroups x, x + 8,
 * ... the x-th eighth) and works it off as items that each run to the end of their row of units or of the range.
 * unit < 0 asks for the workgroup's first item, otherwise `unit` must be a next_unit this function returned for the
 * same arguments.  Outputs: the item's matrix, first row, first column and width in columns, and the unit its successor
 * starts at (-1 = the range ends here; an empty range answers mat = -1 at once).
 * LSW_ERR_ARG: a bad shape, grid not a positive multiple of 8, block outside 0..grid-1, a null pointer.
 */
lsw_status lsw_flat_item(const int32_t* rows, const int32_t* cols, int32_t n_mat, int32_t grid, int32_t block,
                         int64_t unit, int32_t* mat, int32_t* row0, int32_t* col0, int32_t* n_cols, int64_t* next_unit);

#ifdef __cplusplus
}
#endif
#endif /* LSW_TUNING_H */
