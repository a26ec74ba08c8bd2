/*
 * lsw.h -- C ABI of the per-token LoRA expert switch for AMD MI355X (gfx950).
 *
 * The operation is the fused adapter switch of LoRA-Switch (arXiv 2405.17741,
 * Sec. 3.3): every adapted backbone weight holds, merged in place, the top-k
 * LoRA experts the router chose for the previous token; for the next token the
 * previous experts are removed (Eq. 7) and the newly routed ones are added
 * (Eq. 4) in ONE pass over the weight (Eq. 8, rewritten as Eq. 10), for every
 * adapted linear of every layer in ONE kernel launch (Sec. 3.4, Eq. 11):
 *
 *     W[i,j] <- rne_bf16( W[i,j] + sum_{c in new} s*g_c * (B_{e_c} A_{e_c})[i,j]
 *                                - sum_{c in old} s*g_c * (B_{e_c} A_{e_c})[i,j] )
 *
 * Conventions
 *   - W is bf16 [out, in] row-major.  A = LoRA_DOWN is fp32 [E, r, in],
 *     B = LoRA_UP is fp32 [E, out, r]; one expert's update is B_e @ A_e.
 *   - One (ids, gates) pair per token drives all layers (Sec. 3.2, Eq. 2: the
 *     single router G^1 gates every layer's adapters).
 *   - Accumulation is at least fp32 and there is one round-to-nearest-even to
 *     bf16 per element per switch.
 *   - Every call returns a status and never throws or aborts.  Arguments are
 *     validated before anything is launched: on an error no weight is touched.
 *   - Pointers marked DEVICE must be device memory of the current HIP device;
 *     pointers marked HOST are ordinary host memory.  Nothing here takes
 *     ownership of caller memory.
 *   - Calls on one context are not thread-safe; work is ordered by the stream.
 *     Two switches in flight on different streams over the same weights race.  Switches over
 *     DISJOINT layer subsets may overlap on different streams: every launch of lsw_switch,
 *     lsw_switch_dev and lsw_rebase takes its own small block of library-owned device memory (the
 *     device-built term list and two work counters), 16 blocks per context used in turn, so at most
 *     16 such launches of one context may be in flight at once.  A recorded HIP graph keeps the
 *     blocks its launches took: do not replay it concurrently with itself.
 *
 * Limits
 *   - One W must stay below 2 GiB counting its rows rounded up to a multiple of 128 (the kernels
 *     address a matrix with 32-bit byte offsets): a 4096 x 262144 or a 128256 x 8192 matrix is
 *     refused with LSW_ERR_SHAPE.  The whole stack may be of any size (the 70B-shaped one is 137 GB).
 *   - At most 2^31 - 1 work items per launch, LSW_MAX_K experts per list, 256 distinct layer subsets
 *     per context (see lsw_switch).
 *
 * Tuning knobs, diagnostics and the host hooks the tests use are declared in lsw_tuning.h.
 */
#ifndef LSW_H
#define LSW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lsw_ctx lsw_ctx;          /* opaque, owned by the library */

typedef enum lsw_status {
  LSW_OK = 0,
  LSW_ERR_ARG = 1,      /* null pointer, id out of range, duplicate id, k too large, non-finite gate ... */
  LSW_ERR_SHAPE = 2,    /* unsupported shape or misaligned pointer */
  LSW_ERR_STATE = 3,    /* `old` does not match what the context knows to be merged (strict mode only); a call that needs
                           lsw_set_base or lsw_enable_adapter_path first; a call made while another device than the
                           context's (the one current at lsw_create_adapters) is the calling thread's current device */
  LSW_ERR_NOMEM = 4,    /* host or device allocation failed */
  LSW_ERR_DEVICE = 5    /* no usable HIP device, or a HIP call failed */
} lsw_status;

enum { LSW_MAX_K = 8 };  /* largest top-k per list (old or new) */

/* One adapted linear.  All three tensors are BORROWED and must outlive the context. */
typedef struct lsw_linear {
  void*        W;      /* DEVICE bf16 [out, in] row-major, 16-byte aligned; updated in place by lsw_switch */
  const void*  A;      /* DEVICE fp32 (or bf16, see lsw_create_adapters_ex) [E, r, in]  (LoRA_DOWN), 16-byte aligned;
                          read at create time when r is a multiple of 8 (see below) */
  const void*  B;      /* DEVICE fp32 (or bf16) [E, out, r] (LoRA_UP), 16-byte aligned; read by every switch */
  int32_t      out;    /* rows of W, >= 1 */
  int32_t      in;     /* columns of W, a positive multiple of 8 (rows stay 16-byte aligned) */
  int32_t      layer;  /* layer number >= 0; several linears share one layer */
  int32_t      kind;   /* informational: 0..6 = q,k,v,o,gate,up,down */
  int32_t      ld;     /* leading dimension of W: elements between the starts of consecutive rows; 0 = dense (= in), else a
                          multiple of 8 that is >= in.  The columns in .. ld-1 of a row are padding: never read, never
                          written.  An in-place pass over a matrix runs fastest when its rows are 4, 8, 16 or 32 KB apart
                          (measured on MI355X: 6.4-6.7 against 5.3-5.8 TB/s at any other pitch), so a caller who can
                          afford the padding may store e.g. a 4096 x 11008 matrix at ld = 16384.  A base copy given to
                          lsw_set_base has the same leading dimension as its W. */
} lsw_linear;

/*
 * Register a stack of adapted linears (the pointer-and-shape arrays that Sec. 3.4
 * gives the fused kernel) and build the static launch metadata: a descriptor per
 * linear and the work decomposition over (layer, linear, tile).
 *
 *   lin, n_lin  HOST array of descriptors, n_lin >= 1.
 *   E, r        experts per linear (1..4096) and LoRA rank (1..512), the same for every linear.
 *   scale       multiplied into every gate (alpha/r of the LoRA recipe; 1.0 if gates are used as is).
 *   out         receives the context; destroy with lsw_destroy.
 *
 * When r is a multiple of 8 the library also keeps its OWN re-laid-out copy of every A
 * (k-contiguous, split into bf16 high and low parts for the matrix cores, E*r*in*4 bytes
 * per linear): A is read once here and must be re-registered if it changes; B is read
 * from the caller's tensor at every switch.  Nothing is merged by this call: the context
 * starts in the state "no expert merged".
 *
 * Errors: LSW_ERR_ARG (null, n_lin < 1, E/r out of range, non-finite scale, layer < 0),
 * LSW_ERR_SHAPE (out < 1, in not a positive multiple of 8, pointer not 16-byte aligned, one W of
 * 2 GiB or more counting rows rounded up to a multiple of 128, E * r * in * 4 bytes of 2 GiB or more
 * for one linear when r is a multiple of 8),
 * LSW_ERR_NOMEM, LSW_ERR_DEVICE (also when no GPU is present; validation comes first).
 */
lsw_status lsw_create_adapters(const lsw_linear* lin, int32_t n_lin, int32_t E, int32_t r,
                               float scale, lsw_ctx** out);

/*
 * The same with the storage type of the LoRA factors chosen (the paper states none; adapter
 * checkpoints are commonly kept in bf16).  LSW_FACTOR_F32 is lsw_create_adapters.  With
 * LSW_FACTOR_BF16 every A and B is a bf16 tensor of the same shape, r must be a multiple of 8,
 * and the update is computed from the stored bf16 values exactly as from fp32 ones: same formula,
 * fp32-grade accumulation, one rounding.  What changes is cost: the stored values need no low part on
 * the matrix cores (two passes instead of three), and the factor traffic halves.
 * Additional error: LSW_ERR_ARG (unknown dtype), LSW_ERR_SHAPE (bf16 with r not a multiple of 8).
 */
enum { LSW_FACTOR_F32 = 0, LSW_FACTOR_BF16 = 1 };
lsw_status lsw_create_adapters_ex(const lsw_linear* lin, int32_t n_lin, int32_t E, int32_t r,
                                  float scale, int32_t factor_dtype, lsw_ctx** out);

/*
 * The fused switch (Alg. 1 steps 2-4; Eq. 8 == Eq. 10; one launch as in Eq. 11).
 *
 *   layers, n_layers   HOST list of distinct layer numbers to switch; NULL, 0 = every layer.  The first call with a
 *                      new subset (in any order) allocates and uploads a small table for it (a blocking copy; not
 *                      inside a stream capture).  A table is never moved or freed while the context lives, so launches
 *                      in flight and recorded graphs stay valid; a context holds at most 256 of them, and a call that
 *                      would need one more fails with LSW_ERR_STATE until lsw_drop_subset_tables has been called.
 *   old_ids/old_gates  HOST, k_old entries: the experts merged now (Eq. 7 removes them).  k_old = 0: none.
 *   new_ids/new_gates  HOST, k_new entries: the experts to merge (Eq. 4).  k_new = 0: restore the base weights.
 *   hip_stream         hipStream_t (NULL = default stream).  The call is asynchronous on it.
 *
 * An expert listed in both sets is applied once with the coefficient s*g_new - s*g_old and
 * skipped when that is zero; if nothing remains nothing is launched and W is untouched.
 * Errors (nothing launched): LSW_ERR_ARG for a null list with k > 0, k outside 0..LSW_MAX_K or
 * above E, id outside [0,E), duplicate id inside one list, non-finite gate, unknown or
 * duplicate layer; LSW_ERR_STATE in strict mode (see lsw_set_option); LSW_ERR_DEVICE.
 */
lsw_status lsw_switch(lsw_ctx* ctx, const int32_t* layers, int32_t n_layers,
                      const int32_t* old_ids, const float* old_gates, int32_t k_old,
                      const int32_t* new_ids, const float* new_gates, int32_t k_new,
                      void* hip_stream);

/*
 * Frees the per-subset tables of the context (they are rebuilt on demand).  Synchronises the device first.  A HIP
 * graph recorded before this call that contains a launch over a layer subset (or any launch of this context other
 * than over all layers) must not be replayed afterwards.  Errors: LSW_ERR_ARG, LSW_ERR_STATE (another device is
 * current), LSW_ERR_DEVICE.
 */
lsw_status lsw_drop_subset_tables(lsw_ctx* ctx);

/*
 * Drift control.  Eq. 7 treats the unmerge as exact; in bf16 it is not: every switch rounds once, so after T
 * switches W differs from rne(W_base + delta_current) by a random walk of about 0.3 * sqrt(T) ulp.  A caller
 * that keeps a copy of the base weights (the second copy Sec. 3.3 avoids for memory's sake; at 288 GB per GPU
 * it is affordable) can remove the accumulated error at any token:
 *
 * lsw_set_base   registers the copies.  W_base is a HOST array of n_lin DEVICE pointers, entry p a bf16
 *                [out_p, in_p] row-major tensor, 16-byte aligned, BORROWED and never written, that holds
 *                linear p with NOTHING merged.  n_lin must equal the number of registered linears.  The call
 *                synchronises the device (it rewrites the descriptor table the kernels read).
 * lsw_rebase     W_p <- rne_bf16(W_base_p + sum_c s*g_c*(B_c A_c)) for every linear of the selected layers
 *                (Eq. 4 applied to the base copy): the same kernels as lsw_switch, one launch, reading the base
 *                copy and writing W.  ids/gates/k: HOST, the set that is to be merged afterwards (what
 *                lsw_switch would have been given as `new`); k = 0 copies the base weights back (one launch of a
 *                copy kernel over the selected linears).
 *                Asynchronous on hip_stream.  The tracked state of the touched layers becomes (ids, gates).
 * Errors: LSW_ERR_ARG (null, n_lin mismatch, base copy == W, bad list or layer), LSW_ERR_SHAPE (misaligned),
 * LSW_ERR_STATE (lsw_rebase before lsw_set_base), LSW_ERR_DEVICE.
 */
lsw_status lsw_set_base(lsw_ctx* ctx, const void* const* W_base, int32_t n_lin);
lsw_status lsw_rebase(lsw_ctx* ctx, const int32_t* layers, int32_t n_layers,
                      const int32_t* ids, const float* gates, int32_t k, void* hip_stream);

/*
 * Decode through one merged linear (Eq. 3: the backbone runs as if it had no adapters):
 * y[i] = sum_j W[i,j] * x[j], fp32 accumulation.
 *
 *   lin_index  index into the array given to lsw_create_adapters.
 *   x_bf16     DEVICE bf16 [in], 16-byte aligned.      y_fp32  DEVICE fp32 [out].
 * Asynchronous on hip_stream.  Errors: LSW_ERR_ARG, LSW_ERR_SHAPE (misaligned x), LSW_ERR_DEVICE.
 */
lsw_status lsw_merged_gemv(lsw_ctx* ctx, int32_t lin_index, const void* x_bf16, float* y_fp32,
                           void* hip_stream);

/*
 * The same decode through EVERY registered linear in one launch (the backbone pass that follows
 * the switch in Alg. 1, step 5, as far as the weights are concerned: no activations are chained
 * here, each linear gets the input the caller supplies).
 *
 *   x_all_bf16  DEVICE bf16, 16-byte aligned: the inputs of the linears back to back in registration
 *               order, linear p at element offset sum_{q<p} in_q (lsw_query LSW_Q_GEMV_X_ELEMS = total;
 *               every in is a multiple of 8, so each part stays 16-byte aligned).
 *   y_all_fp32  DEVICE fp32: the outputs back to back, linear p at offset sum_{q<p} out_q
 *               (LSW_Q_GEMV_Y_ELEMS = total).
 * Asynchronous on hip_stream.  Errors: LSW_ERR_ARG, LSW_ERR_SHAPE (misaligned x), LSW_ERR_DEVICE.
 */
lsw_status lsw_merged_gemv_all(lsw_ctx* ctx, const void* x_all_bf16, float* y_all_fp32, void* hip_stream);

/*
 * Router on given logits: G = Softmax(TopK(logits)) (definition of G under Eq. 1, used by the
 * single token-wise router of Eq. 2).  Host helper, touches no device.
 *
 *   logits HOST fp32 [E];  ids HOST int32 [k] and gates HOST fp32 [k] receive the selection in
 *   descending logit order (equal logits: lower index first; +0 equals -0); the softmax runs over
 *   the k selected logits only, in double precision, rounded once to fp32.
 * Errors: LSW_ERR_ARG (null, E < 1, k outside 0..E, NaN logit).
 */
lsw_status lsw_route(const float* logits, int32_t E, int32_t k, int32_t* ids, float* gates);

/*
 * Device-resident routing: the same three steps (router, term list, switch) with the token's
 * (ids, gates) living in DEVICE memory from start to end, so that a token step needs no trip to the
 * host between the router's output and the fused launch of Alg. 1 and can be recorded in a HIP graph
 * (none of these calls allocates, synchronises or clears memory with a memset).
 *
 * lsw_route_dev     G = Softmax(TopK(logits)) as lsw_route computes it (same order, same tie rule,
 *                   softmax in double precision rounded once), E = the context's expert count.
 *                   logits_dev DEVICE fp32 [E]; ids_dev DEVICE int32 [k]; gates_dev DEVICE fp32 [k];
 *                   0 <= k <= min(LSW_MAX_K, E).
 * lsw_switch_dev    lsw_switch with DEVICE lists.  k_old and k_new are host values (the lists' lengths
 *                   are fixed by the model's top-k); the launch is sized for k_old + k_new terms and
 *                   the device drops the cancelled ones, exactly as lsw_build_terms does.  The
 *                   context cannot know what was merged: lsw_get_state answers LSW_ERR_STATE for the
 *                   touched layers until a host-side lsw_switch sets them again, and the call is
 *                   refused (LSW_ERR_STATE) while LSW_OPT_STRICT_STATE is on.
 * lsw_dev_status    What the host cannot check before the launch is checked on the device: a NaN logit
 *                   (flag 1) or a bad list, id outside [0,E), duplicate id, non-finite gate (flag 2),
 *                   makes that switch leave every weight untouched and sets a sticky flag in the
 *                   context.  This call copies the flags to the host (it synchronises with the null
 *                   stream; synchronise the work's own stream first).
 * lsw_gemv_bf16     y = W x for any bf16 matrix [out, in] (in a multiple of 8, 16-byte aligned), e.g.
 *                   the router's logits W_g x of Eq. 2 from the first layer's input.  DEVICE pointers.
 * Errors known on the host are reported as for the host-side calls, before anything is launched.
 */
lsw_status lsw_route_dev(lsw_ctx* ctx, const float* logits_dev, int32_t k, int32_t* ids_dev, float* gates_dev,
                         void* hip_stream);
lsw_status lsw_switch_dev(lsw_ctx* ctx, const int32_t* layers, int32_t n_layers,
                          const int32_t* old_ids_dev, const float* old_gates_dev, int32_t k_old,
                          const int32_t* new_ids_dev, const float* new_gates_dev, int32_t k_new,
                          void* hip_stream);
lsw_status lsw_dev_status(lsw_ctx* ctx, int32_t* flags);
lsw_status lsw_gemv_bf16(const void* W_bf16, const void* x_bf16, float* y_fp32, int32_t out, int32_t in,
                         void* hip_stream);

/*
 * The un-merged adapter path for many tokens (Eq. 2: y = f(x) + sum_i G(x1)_i E_i(x) with E_i(x) = W_up (W_down x)),
 * what a prompt runs through before decoding starts: every token has its own (ids, gates), so nothing can be merged.
 * The backbone's own product f(x) = W x is the caller's (a plain GEMM on the base weights: switch with k_new = 0
 * first); the library adds the dynamic-adapter sum of one linear to it:
 *
 *   Y[t, i] <- rne_bf16( Y[t, i] + sum_{c<k} s*g[t,c] * sum_rho B[e][i,rho] * (sum_j A[e][rho,j] * X[t,j]) ),  e = ids[t,c]
 *
 * lsw_enable_adapter_path  builds, once, the two re-laid-out operand copies the path needs for every linear (A for
 *                          the down-projection, B^T for the up-projection, E*r*(in+out)*4 bytes per linear for fp32
 *                          factors, half for bf16).  Needs r % 8 == 0, E*r <= 256 and every out % 8 == 0
 *                          (LSW_ERR_SHAPE otherwise); synchronises the device.  The path computes the down-projection
 *                          of ALL E*r rows for every token and selects with a gate table, so its matrix work grows with
 *                          E*r, not k*r: it moves a prompt at about half of the HBM rate for E*r = 64 and becomes bound by
 *                          the matrix cores beyond (measured: a quarter of the HBM rate at E*r = 256).
 * lsw_route_batch_dev      G = Softmax(TopK(.)) for n_tokens rows of logits at once (the router of Eq. 2 over a prompt):
 *                          logits_dev DEVICE fp32 [n_tokens, E]; ids_dev DEVICE int32 [n_tokens, k]; gates_dev DEVICE
 *                          fp32 [n_tokens, k]; per row exactly what lsw_route_dev computes.
 * lsw_adapter_forward      the update above for linear lin_index and T tokens.  X_bf16 DEVICE bf16 [T, in]; ids_dev
 *                          DEVICE int32 [T, k]; gates_dev DEVICE fp32 [T, k]; Y_bf16 DEVICE bf16 [T, out], read and
 *                          written; workspace DEVICE, lsw_adapter_workspace_bytes(ctx, lin_index, T) bytes, contents
 *                          irrelevant before and after; all 16-byte aligned.  Three launches, asynchronous on
 *                          hip_stream, nothing allocated.  A token whose list is bad (id outside [0,E), duplicate id,
 *                          non-finite gate) keeps its row of Y unchanged and raises flag 2 of lsw_dev_status.
 * lsw_adapter_forward_layer the same for EVERY linear of one layer in three launches in all (all down-projections, all
 *                          gate tables, all up-projections), which is what a prompt of a few thousand tokens needs: one
 *                          linear alone does not fill the chip.  X_bf16 and Y_bf16 are HOST arrays of DEVICE pointers, one
 *                          entry per linear of `layer` in registration order (linears that read the same activations, q/k/v
 *                          or gate/up, simply get the same X pointer; every Y is distinct); all linears see the same T tokens
 *                          and the same per-token lists (the single router of Eq. 2).  workspace: DEVICE,
 *                          lsw_adapter_layer_workspace_bytes(ctx, layer, T) bytes.  A layer may have at most 8 linears
 *                          (LSW_ERR_SHAPE).  Per linear the result is bit for bit what lsw_adapter_forward gives.
 * Errors: LSW_ERR_ARG, LSW_ERR_SHAPE (misaligned, X or Y of 2 GiB or more), LSW_ERR_STATE (path not enabled),
 * LSW_ERR_NOMEM, LSW_ERR_DEVICE.
 */
lsw_status lsw_enable_adapter_path(lsw_ctx* ctx);
int64_t    lsw_adapter_workspace_bytes(const lsw_ctx* ctx, int32_t lin_index, int32_t T);   /* -1 on a bad argument */
lsw_status lsw_route_batch_dev(lsw_ctx* ctx, const float* logits_dev, int32_t n_tokens, int32_t k, int32_t* ids_dev,
                               float* gates_dev, void* hip_stream);
lsw_status lsw_adapter_forward(lsw_ctx* ctx, int32_t lin_index, const void* X_bf16, int32_t T,
                               const int32_t* ids_dev, const float* gates_dev, int32_t k,
                               void* Y_bf16, void* workspace, void* hip_stream);
int64_t    lsw_adapter_layer_workspace_bytes(const lsw_ctx* ctx, int32_t layer, int32_t T);   /* -1 on a bad argument */
lsw_status lsw_adapter_forward_layer(lsw_ctx* ctx, int32_t layer, const void* const* X_bf16, int32_t T,
                                     const int32_t* ids_dev, const float* gates_dev, int32_t k,
                                     void* const* Y_bf16, void* workspace, void* hip_stream);

/*
 * lsw_adapter_forward for callers that can neither allocate device memory nor bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace, same three
 * launches, same result bit for bit; the partial sums and the gate table live in a device array of 32 MiB that is part
 * of the library's code object (every GPU the library runs on holds its own copy until the process ends; its address on
 * the context's device is looked up once, at lsw_enable_adapter_path).  The call allocates and frees nothing and
 * synchronises nothing.  T is limited by lsw_adapter_workspace_bytes(ctx, lin_index, T) <= 32 MiB (33,554,432 bytes; about
 * 13,000 to 100,000 tokens of a 4096-wide linear, depending on E * r): beyond it LSW_ERR_SHAPE, nothing launched.  Every call on
 * one GPU, from any context, uses the same array: calls that overlap on one GPU (two streams, two threads) race on it;
 * order them.  Nothing in it has to be cleared between calls (the kernels write every word they later read).
 * Other errors: as lsw_adapter_forward.
 */
lsw_status lsw_adapter_forward_static(lsw_ctx* ctx, int32_t lin_index, const void* X_bf16, int32_t T,
                                      const int32_t* ids_dev, const float* gates_dev, int32_t k,
                                      void* Y_bf16, void* hip_stream);

/*
 * The signed coefficient list one switch applies (Alg. 1 steps 2-3 without moving any tensor:
 * Eq. 5 puts the gate on one factor, Eq. 9 negates the previous set): new experts with
 * +scale*g, old experts with -scale*g, an expert in both with scale*g_new - scale*g_old,
 * zero coefficients dropped.  Host helper; lsw_switch uses exactly this.
 *
 *   terms_ids / terms_coeff  HOST arrays with room for k_old + k_new entries; n_terms receives the count.
 * Errors: as the list checks of lsw_switch (LSW_ERR_ARG).
 */
lsw_status lsw_build_terms(const int32_t* old_ids, const float* old_gates, int32_t k_old,
                           const int32_t* new_ids, const float* new_gates, int32_t k_new,
                           int32_t E, float scale,
                           int32_t* terms_ids, float* terms_coeff, int32_t* n_terms);

/*
 * What the context believes is merged in `layer` now (the pair Eq. 7 needs for the next
 * switch).  ids/gates HOST arrays with room for LSW_MAX_K entries; k receives the count.
 */
lsw_status lsw_get_state(const lsw_ctx* ctx, int32_t layer, int32_t* ids, float* gates, int32_t* k);

/* Options (lsw_set_option) and queries (lsw_query).  The tuning knobs (options 3..10) are declared in lsw_tuning.h. */
enum {
  LSW_OPT_KERNEL = 1,        /* 0 = automatic, 1 = fp32 vector-ALU kernel (any rank), 2 = matrix-core kernels
                                (need r % 8 == 0 and at most 256 fused ranks = terms * r per switch) */
  LSW_OPT_STRICT_STATE = 2   /* 1: lsw_switch rejects an `old` that differs from the tracked state of a layer */
};
enum {
  LSW_Q_N_LINEARS = 1, LSW_Q_N_LAYERS = 2,
  LSW_Q_LAST_KERNEL = 3,     /* kernel the last lsw_switch launched: 0 none, 1 vector-ALU, 2 matrix-core */
  LSW_Q_LAST_ITEMS = 4,      /* work items of the last launch */
  LSW_Q_LAST_GRID = 5,       /* workgroups of the last launch */
  LSW_Q_PACKED_BYTES = 6,    /* bytes of device memory the context owns */
  LSW_Q_GEMV_X_ELEMS = 7,    /* elements of lsw_merged_gemv_all's x_all (sum of in over the linears) */
  LSW_Q_GEMV_Y_ELEMS = 8,    /* elements of its y_all (sum of out) */
  LSW_Q_LAST_VARIANT = 9     /* which matrix-core kernel the last launch was: 0 none / vector-ALU, 1 A streamed per step,
                                2 A resident in LDS, 3 chunked (fused rank above 64) */
};
lsw_status lsw_set_option(lsw_ctx* ctx, int32_t option, int64_t value);
int64_t    lsw_query(const lsw_ctx* ctx, int32_t what);   /* -1 on a bad argument */

void        lsw_destroy(lsw_ctx* ctx);       /* frees what the library owns; NULL is allowed */
const char* lsw_last_error(void);            /* message of the last failing call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* LSW_H */
