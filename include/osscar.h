/*
 * osscar.h -- C interface of the MI355X (gfx950) per-layer structured-pruning solver of OSSCAR
 * (arxiv 2403.12983).
 *
 * Problem (Section 3, eq. (MIQP); Section 4.1, eq. (struc)): the rows of the dense weight matrix
 * W (d1 x m) are split into p contiguous groups of q rows (d1 = p*q: FFN neurons q = 1, conv input
 * channels q = k_H*k_W, attention heads q = D_head).  Keep k groups K, zero the other rows and refit
 * the kept rows so that
 *        obj(What) = || X W - X What ||_F^2 + lambda || W - What ||_F^2
 * is as small as the local search of Section 4.2 can make it.  With H = X^T X + lambda I, G = H W this
 * is c0 + 2 L(What), L the quadratic of eq. (MIQP), c0 = Tr(W^T H W).
 *
 * Naming: this interface uses K for the KEPT groups (the paper's S is the pruned set, K its
 * complement), W for the given dense weights (the paper's W-hat) and What for the solved weights.
 *
 * Conventions for every call
 *   - "dev" pointers are device (HBM) addresses on the current HIP device, "host" pointers are host
 *     addresses.  All matrices are row-major; leading dimensions are in elements.
 *   - The library allocates no device memory.  The caller hands one workspace of at least
 *     osscar_workspace_bytes() bytes (256-byte aligned) to osscar_create and owns it, X, W and What.
 *     The context keeps pointers into the workspace only; W is read only during osscar_gram.
 *   - All work is ordered on the stream given to osscar_create.  Calls that return host values
 *     synchronise that stream; osscar_gram without finalize does not (bf16 chunks on the matrix-core path; other chunks
 *     may).  The context owns one more stream (default
 *     priority) for a product of the search that overlaps with others; it forks from and joins the caller's stream
 *     through events inside a call, so the caller sees the ordering of a single stream.
 *   - Every call returns an osscar_status.  No exception crosses this boundary and nothing aborts.
 *     After a failure other than OSSCAR_EINVAL the context refuses further compute calls
 *     (OSSCAR_ESTATE) until it is destroyed and re-created.  osscar_last_error() describes the failure.
 *   - Groups are equal-sized and contiguous (the three cases of Section 3; Prop. 4.2 assumes equal size).  There is no
 *     group map argument: a caller whose groups are scattered permutes the rows of W (and the columns of X) first.
 *   - Precision.  H, G and the search state are stored in float32 (products accumulated in float64 where it matters).
 *     Choices, kept sets, final weights and final objective follow a float64 evaluation of the same method for any H the
 *     inverse converges on.  Quantities tracked through many updates (the objective trace of a search) follow it to about
 *     1e-5 relative while the diagonally scaled H restricted to the kept rows has a condition number below about 1e4; above
 *     that the float32 rounding of H alone moves them by up to 6e-8 * cond, and refresh_every (a rebuild from H and G every so
 *     many swaps) bounds the drift.
 *   - Calls on one context must not overlap; contexts sharing a workspace must not be used concurrently.
 */
#ifndef OSSCAR_H
#define OSSCAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct osscar_ctx osscar_ctx; /* opaque; host memory owned by the library */

typedef enum {
  OSSCAR_OK = 0,
  OSSCAR_EINVAL = 1, /* bad argument (shape, k > p, NULL pointer, misaligned buffer, ...) */
  OSSCAR_ENOMEM = 2, /* workspace too small */
  OSSCAR_ENOTPD = 3, /* H_KK (or a q x q pivot block) is not positive definite to working precision */
  OSSCAR_EHIP = 4,   /* a HIP runtime call failed */
  OSSCAR_ESTATE = 5  /* call order violated, or the context is poisoned by an earlier failure */
} osscar_status;

typedef enum { OSSCAR_F32 = 0, OSSCAR_BF16 = 1 } osscar_dtype;

/* Problem description (Section 3: d1 x m weights, p groups of q rows; Section 4.1: keep k = p - p'). */
typedef struct {
  int64_t d1;        /* rows of W = columns of X; must equal p*q */
  int64_t m;         /* columns of W */
  int32_t p;         /* number of groups */
  int32_t q;         /* rows per group, 1 <= q <= 64 */
  int32_t k;         /* groups to keep, 1 <= k <= p */
  int32_t max_swaps; /* upper bound on the swap budget of any osscar_local_search call (sizes the trace) */
  int32_t x_dtype;   /* osscar_dtype of X */
  int32_t w_dtype;   /* osscar_dtype of W */
  int32_t from_dense; /* nonzero: size the workspace for osscar_init_greedy too (it inverts all of H) */
  int32_t target_output; /* nonzero: size the workspace for osscar_gram_target too */
} osscar_desc;

/* Bytes of device workspace osscar_create needs for this description (0 if the description is invalid). */
size_t osscar_workspace_bytes(const osscar_desc* desc);

/* Creates a context.  workspace_dev: device, >= osscar_workspace_bytes(desc) bytes, 256-byte aligned.
 * hip_stream: a hipStream_t (NULL = the default stream).  *out receives the context. */
osscar_status osscar_create(osscar_ctx** out, const osscar_desc* desc, void* workspace_dev, size_t workspace_bytes,
                            void* hip_stream);
osscar_status osscar_destroy(osscar_ctx* ctx);

/* Quadratic-form construction (Section 3, dense-layer paragraph: H = X^T X, G = X^T X W; the ridge is
 * this build's addition).  Each call adds one chunk of calibration rows: H += Xc^T Xc with
 * Xc dev, row-major n_c x d1 (leading dimension ldx >= d1), dtype desc.x_dtype.  Any number of chunks,
 * any n_c >= 0; products are accumulated in float64 across chunks.
 * finalize != 0 (after adding Xc, which may be NULL with n_c = 0): lambda = lambda_abs + lambda_rel *
 * mean(diag(X^T X)); H += lambda I (stored float32); G = H W (float32); c0 = Tr(W^T G); the group norms
 * ||W_{Q^j}||_F are recorded for osscar_init_support.  W_dev: dev, row-major d1 x m, leading dimension
 * ldw, dtype desc.w_dtype (ignored unless finalize).  A new first chunk after finalize starts a new layer. */
osscar_status osscar_gram(osscar_ctx* ctx, const void* Xc_dev, int64_t n_c, int64_t ldx, int finalize,
                          const void* W_dev, int64_t ldw, double lambda_abs, double lambda_rel);

/* Convolutional layers (Section 3, "Structured pruning in convolutional layers": W is (C_in * k_H * k_W) x C_out and
 * the rows of X are the k_H x k_W patches of the layer's input).  Same as osscar_gram, but takes the input feature map
 * itself and forms the patches on the fly, so that the caller never holds the k_H * k_W times larger patch matrix.
 * F_dev: dev, contiguous (batch, channels, h_in, w_in), dtype desc.x_dtype, zero padding `pad` on every side.  The
 * patch at output position (b, oy, ox) is the row (b * h_out + oy) * w_out + ox, and input channel c, kernel offset
 * (dy, dx) is the column (c * kh + dy) * kw + dx: the rows of W acting on channel c form the group of kh * kw rows c.
 * channels * kh * kw must equal desc.d1.  Chunks (batches of feature maps) may be mixed with osscar_gram chunks. */
osscar_status osscar_gram_conv(osscar_ctx* ctx, const void* F_dev, int32_t batch, int32_t channels, int32_t h_in, int32_t w_in,
                               int32_t kh, int32_t kw, int32_t stride, int32_t pad, int finalize, const void* W_dev,
                               int64_t ldw, double lambda_abs, double lambda_rel);

/* Sequential-pipeline variant of osscar_gram (Appendix B.1, "Pruning strategies": the layer is asked to reproduce
 * the DENSE model's output from the PRUNED model's input).  Yc_dev: dev, row-major n_c x m, leading dimension
 * ldy >= m, dtype desc.x_dtype: the dense model's output of this layer for the same calibration rows as Xc.
 * Accumulates H += Xc^T Xc and X^T Y += Xc^T Yc (float64 across chunks) and ||Y||_F^2.  finalize: lambda as in
 * osscar_gram; H += lambda I; G = X^T Y + lambda W; c0 = ||Y||_F^2 + lambda ||W||_F^2, so that
 * obj(What) = ||Y - X What||_F^2 + lambda ||W - What||_F^2 = c0 - 2 Tr(G^T What) + Tr(What^T H What) and every later
 * call works unchanged.  Needs desc.target_output != 0.  A layer takes all its chunks through this call or all
 * through osscar_gram (OSSCAR_ESTATE otherwise). */
osscar_status osscar_gram_target(osscar_ctx* ctx, const void* Xc_dev, const void* Yc_dev, int64_t n_c, int64_t ldx,
                                 int64_t ldy, int finalize, const void* W_dev, int64_t ldw, double lambda_abs,
                                 double lambda_rel);

/* Alternative to osscar_gram for callers that already hold the quadratic form: copies H (d1 x d1,
 * symmetric positive definite, ridge included) and G (d1 x m), both dev float32 row-major and dense
 * (ld = d1, m), and takes c0 and the p group norms (host float64) used by the magnitude mode. */
osscar_status osscar_set_quadratic(osscar_ctx* ctx, const float* H_dev, const float* G_dev, double c0,
                                   const double* group_norms_host);

/* Support initialisation.  OSSCAR_INIT_MAGNITUDE: keep the k groups of largest Frobenius norm
 * (Appendix B.1, "MP"; equal norms: the lower group index stays).  OSSCAR_INIT_GIVEN: keep
 * groups_host[0..k) (distinct, any order).  Then builds the state Proposition 4.1 assumes -- the
 * inverse P of H on the kept rows, the optimal kept weights B = P G_K (eq. (optf)) -- plus the
 * candidate-side quantities V = P H_{K,Kc} and R = G_Kc - V^T G_K used by the impact scores
 * (eq. (impact)), and returns obj(K) = c0 - Tr(G_K^T B) in *obj_host (may be NULL). */
enum { OSSCAR_INIT_MAGNITUDE = 0, OSSCAR_INIT_GIVEN = 1 };
osscar_status osscar_init_support(osscar_ctx* ctx, int mode, const int32_t* groups_host, double* obj_host);

/* Nested schedule of Algorithm 1 from the dense layer (S_0 empty and t_i = p_i = t_hat for every iteration:
 * Section 4.2; Appendix B.1 takes t_hat = 2 for channels and attention heads and 10 for the intermediate
 * dimension of feed-forward layers).  Starts with every group kept (P = H^-1, B = H^-1 G; obj = 0 after
 * osscar_gram, c0 - Tr(G^T B) otherwise); each
 * iteration scores every kept group by the cost of removing it (eq. (impact), closed form of
 * Proposition 4.1 Case 1) at the state the iteration starts from, removes the t_hat cheapest (lowest group
 * index on ties; the last iteration takes what is left to reach k) and updates inverse, weights and objective
 * by Case 1.  Leaves the context as osscar_init_support does, so osscar_local_search and osscar_backsolve
 * can follow.  Needs desc.from_dense != 0.  1 <= t_hat <= 64.
 * refresh_every > 0 rebuilds the state from H and G after that many removals (at iteration boundaries).
 * flags: 0, or OSSCAR_SEARCH_EAGER to update the state in place after every removal also for q = 1, or
 * OSSCAR_SEARCH_NO_LOOKAHEAD (see osscar_local_search).
 * removed_host (host, optional): p - k group ids in the order removed (within an iteration: cheapest first).
 * gaps_host (host, optional): one float per iteration, ceil((p - k) / t_hat) of them: relative gap between the
 * costliest removal chosen and the cheapest kept group left out (inf if none was left out).
 * obj_host (host, optional): the tracked objective of the resulting kept set. */
osscar_status osscar_init_greedy(osscar_ctx* ctx, int32_t t_hat, int32_t refresh_every, uint32_t flags,
                                 int32_t* removed_host, float* gaps_host, double* obj_host);

/* Local search (Section 4.2 and Algorithm 1 with t-hat = 2, p-hat = 0: one group leaves, one enters).
 * Each iteration scores every kept group by the cost of removing it and every outside group by the
 * gain of adding it (eq. (impact), via the closed forms of Proposition 4.1, Cases 1 and 2), picks the
 * cheapest removal and the largest gain (ties: lowest group index), evaluates the pair's exact effect
 * (Case 3) and applies it by low-rank up/downdates if obj drops by more than rel_tol*obj; otherwise
 * the search stops.  At most max_swaps (<= desc.max_swaps) iterations.
 * flags: OSSCAR_SEARCH_ALWAYS_ACCEPT applies every selected pair (Algorithm 1 as printed).
 * OSSCAR_SEARCH_EAGER applies every swap to the whole state at once (one pass over HBM per swap); by
 * default, layers with q = 1 keep up to 64 swaps pending as a small low-rank correction and apply them
 * together on the matrix cores -- the same swaps, with less traffic.  In that mode the products of Z with the
 * rows most likely to be swapped next are computed ahead by one matrix product per flush;
 * OSSCAR_SEARCH_NO_LOOKAHEAD turns that off (every swap then reads Z once).
 * OSSCAR_SEARCH_EXACT_IN (a stronger rule than the separable scores of eq. (impact), not in the paper): with the
 * leaving group fixed as above, the entering group is the one with the largest exact gain of the pair, i.e. every
 * candidate is scored at the state without the leaving group (Case 1 applied to the blocks its score needs); costs one
 * more pass over Z per iteration and runs on the in-place path; trace_gap[2i+1] then refers to these scores.
 * refresh_every > 0 recomputes V, R and B from P, H, G by GEMM after that many accepted swaps.
 * Optional host outputs of length max_swaps (entry i describes iteration i, including a final rejected
 * one): trace_out / trace_in = group leaving / entering; trace_gap[2i], trace_gap[2i+1] = relative gap
 * between best and second-best removal cost / addition gain; trace_obj[i] = obj after the iteration. */
enum { OSSCAR_SEARCH_ALWAYS_ACCEPT = 1u, OSSCAR_SEARCH_EAGER = 2u, OSSCAR_SEARCH_NO_LOOKAHEAD = 4u, OSSCAR_SEARCH_EXACT_IN = 8u };
typedef struct {
  int32_t iters;     /* iterations run (accepted swaps + at most one rejected) */
  int32_t accepted;  /* swaps applied */
  double obj_initial;
  double obj_final;  /* tracked through the updates */
} osscar_search_result;
osscar_status osscar_local_search(osscar_ctx* ctx, int32_t max_swaps, double rel_tol, uint32_t flags,
                                  int32_t refresh_every, osscar_search_result* res_host, int32_t* trace_out_host,
                                  int32_t* trace_in_host, float* trace_gap_host, double* trace_obj_host);

/* Block moves (Section 4.2 with t-hat = 2 * block, p-hat = 0: s1 = s2 = block).  Each iteration scores every group
 * at the current state (eq. (impact)), takes the `block` kept groups that are cheapest to remove and the `block`
 * outside groups with the largest gain (lowest index on ties; cut to min(block, k, p - k)), applies the whole move
 * by the low-rank updates of Proposition 4.1 and keeps it if obj dropped by more than rel_tol*obj; otherwise the
 * move is taken back and the search stops.  block = 1 is osscar_local_search's move.  1 <= block <= 64.
 * flags as for osscar_local_search.  Optional host outputs: trace_out / trace_in, max_iters * block entries each
 * (iteration i at [i*block, (i+1)*block), cheapest removal / largest gain first, -1 padding); trace_gap[2i],
 * trace_gap[2i+1] = relative gap between the last group chosen and the first left out on either side;
 * trace_obj[i] = obj after iteration i.  res->iters counts iterations, res->accepted the moves kept. */
osscar_status osscar_block_search(osscar_ctx* ctx, int32_t max_iters, int32_t block, double rel_tol, uint32_t flags,
                                  osscar_search_result* res_host, int32_t* trace_out_host, int32_t* trace_in_host,
                                  float* trace_gap_host, double* trace_obj_host);

/* Test hook: applies the swap (group g_out leaves, g_in enters) unconditionally (Case 3). */
osscar_status osscar_apply_swap(osscar_ctx* ctx, int32_t g_out, int32_t g_in);

/* Final weights (closed-form optimum for the final kept set, Appendix A.1): What_K = (H_KK)^-1 G_K, other
 * rows zero.  The maintained weights are refined by float64-residual correction steps B += P (G_K - H_KK B)
 * until the correction is below float32 resolution; if the maintained inverse P has drifted too far for
 * that, H_KK is inverted afresh.
 * What_dev: dev, row-major d1 x m, leading dimension ldw_hat, dtype out_dtype.  support_host (may be
 * NULL): the k kept groups, ascending.  *obj_host (may be NULL): c0 - Tr(G_K^T What_K). */
osscar_status osscar_backsolve(osscar_ctx* ctx, void* What_dev, int64_t ldw_hat, int32_t out_dtype,
                               int32_t* support_host, double* obj_host);

/* Inspection hook: copies an internal array to dst_dev (dev, dense row-major).  float32: H d1 x d1;
 * G d1 x m; P kr x kr; B kr x m; V kr x cr; R cr x m (kr = k*q, cr = d1 - kr; rows / columns follow the
 * kept groups, resp. the other groups, in ascending group order).  float64: REM, ADD: length p, indexed
 * by group id (+inf / -inf where not applicable).  int32: KEPT_SLOTS / CAND_SLOTS: the kept / other
 * group ids, ascending. */
enum { OSSCAR_T_H = 0, OSSCAR_T_G = 1, OSSCAR_T_P = 2, OSSCAR_T_B = 3, OSSCAR_T_V = 4, OSSCAR_T_R = 5,
       OSSCAR_T_REM = 6, OSSCAR_T_ADD = 7, OSSCAR_T_KEPT_SLOTS = 8, OSSCAR_T_CAND_SLOTS = 9 };
osscar_status osscar_get_tensor(osscar_ctx* ctx, int which, void* dst_dev, size_t dst_bytes);

/* Scalars of the last finalize: lambda, c0 (host float64). */
osscar_status osscar_get_scalars(osscar_ctx* ctx, double* lambda_host, double* c0_host);

/* Device times of the last call of each kind, in milliseconds (HIP events on the context's stream):
 * [0] the Gram accumulation of the chunk passed together with finalize, [1] finalize, [2] init_support,
 * [3] local_search, [4] backsolve, [6] total time of the search's refreshes and flushes.  Sampled once
 * per batch of iterations: eager search [5] mean duration of one bulk update of N, [7] of one update of Z;
 * delayed-update search [5] mean duration of the kernel with the acceptance test and u = ZT [y1 y2] (it also makes a pass
 * over Z for a pivot whose products were not computed ahead), [7] of all kernels of that iteration from there on.
 * [8] the product G = H W inside finalize (one GEMM launch, or the three bf16 products and their repacking when W is
 * bf16).  [9] the inverse of H on the kept rows in the last state build: the blocked sweep on a float64 copy of H_KK
 * (about 2 kr^3 flops on the float64 matrix cores).  [10] zero.  [11] not a time: the largest P_ii H_ii over the kept rows
 * (the variance inflation factor 1 / (1 - R_i^2): how much of a kept row the other kept rows explain), a
 * measure of the conditioning of H_KK.  [12] the candidate-side products V, S, R of the last state build together.
 * [13] mean duration of one launch of the bf16 Gram kernel (one launch per 16384 calibration rows) in the last
 * osscar_gram call that added rows on that path before the last finalize, [14] the number of launches averaged, [15] the rows
 * that call added.  out_host: 16 doubles. */
osscar_status osscar_get_timers(osscar_ctx* ctx, double* out_host);

/* Diagnostics of the last osscar_local_search call on the delayed-update path (all zero otherwise), 8 values:
 * [0] flushes (the pending low-rank correction applied to the stored state by matrix products), [1] how many of them the
 * kernels asked for by stopping early (a selected group was still pending, or the spare slots for products not computed
 * ahead ran out), [2] pivots whose products with Z had not been computed ahead (each costs one pass over Z), [3] iterations
 * run; [4..7] reserved (zero).  out_host: 8 int64. */
osscar_status osscar_get_counters(osscar_ctx* ctx, int64_t* out_host);

/* Diagnostic log of the library's general matrix-product launches (all contexts of the process; not thread-safe).
 * osscar_debug_gemm_log(1) clears the log and starts recording: every launch is bracketed by two events on its stream.
 * osscar_debug_gemm_log(0) stops and clears.  osscar_debug_gemm_log_read waits for the recorded launches and writes up to
 * `capacity` rows of five float64 {M, N, K, kind, milliseconds} (kind: 1 = float32 accumulation, + 2 = float64 output,
 * + 4 = lower-triangle tiles only, + 8 = second operand transposed, 16 = int8-digit product, packing included) to out_host; returns the number of rows, -1 on a bad
 * argument.  At most 16384 launches are kept. */
osscar_status osscar_debug_gemm_log(int32_t enable);
int32_t osscar_debug_gemm_log_read(double* out_host, int32_t capacity);

/* The large products that define the state of a support (every dimension >= 1024: B = P G_K, V = P H_{K,Kc}, the Schur
 * complement S and R of Proposition 4.1's closed forms) run on the int8 matrix cores from five 7-bit digits per float32
 * operand, with exact integer sums (kind 16 in the log above), and so does the residual of the back-solve; smaller ones, and
 * the residuals that involve the inverse, on the float64-accumulating kernel.  osscar_debug_int_products(0) sends all of them to the
 * float64-accumulating kernel, osscar_debug_int_products(1) restores the default.  Process-wide, for tests that hold the two
 * against each other. */
osscar_status osscar_debug_int_products(int32_t enable);

/* The inverse of H on the kept rows (P of Proposition 4.1) is computed by a blocked sweep on a float64 copy of H_KK and
 * rounded to float32 once.  osscar_debug_refined_inverse(1) switches to the other route - the sweep in float32 storage,
 * then Newton-Schulz steps P <- P + P (I - H_KK P) with a float64-accumulated residual - and (0) back.  Process-wide, for
 * tests that hold the two against each other.  Timer slot 9 is the duration of the float64 sweep (of the residual product
 * on the other route), slot 11 the largest P_ii H_ii (the residual |I - H_KK P| before the last step on the other route). */
osscar_status osscar_debug_refined_inverse(int32_t enable);

/* The library overlaps independent parts of two phases on a second stream of its own: in the inverse of H_KK the bulk of
 * each panel's update beside the next panel's small kernels, in the flush of the delayed-update search (Proposition 4.1
 * applied to 64 pending swaps at once) the update of N beside that of Z and the products computed ahead.
 * osscar_debug_side_stream(0) runs everything in order on the context's stream, (1) (the default) restores the overlap.
 * Process-wide.  The inverse is bit-identical either way (every tile sees the same operations in the same order); the
 * search may differ in the last digits of the row norms, because the candidates for the products computed ahead are then
 * picked after the score refresh instead of before it. */
osscar_status osscar_debug_side_stream(int32_t enable);

/* Host-only inspection of the Gram kernel's tile schedule (no device is touched): writes up to `capacity` (row, column)
 * pairs of 128 x 128 tiles, in workgroup order, to out_host (2 ints each; (-1, -1) = padding) and returns the length of
 * the schedule, or -1 for a bad d1.  Workgroup i runs on XCD i % 8. */
int32_t osscar_debug_tile_schedule(int64_t d1, int32_t* out_host, int32_t capacity);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the quadratic form of one small layer in one call, with no context and no workspace.  Same result
 * as osscar_gram(ctx, X, n, ldx, finalize = 1, W, ...) followed by reading H, G, lambda and c0 back:
 *   H = X^T X + lambda I (float32, d1 x d1, both triangles), lambda = lambda_abs + lambda_rel * mean(diag(X^T X)),
 *   G = H W (float32, d1 x m), c0 = Tr(W^T G); products accumulated in float64.
 * X_dev: dev, row-major n x d1 (leading dimension ldx), dtype x_dtype; W_dev: dev, d1 x m (ldw), dtype w_dtype;
 * H_dev, G_dev: dev outputs, dense (leading dimensions d1 and m); scalars_dev: dev, 2 float64 = {lambda, c0}.
 * Everything is enqueued on hip_stream (a hipStream_t, NULL = default stream); the call does not wait for it and
 * calls no hipMalloc, hipFree or other allocating routine.  What osscar_gram keeps in the caller's workspace meanwhile
 * (float64 accumulator, float32 W, transposed staging of X) lives in a device array of OSSCAR_STATIC_SCRATCH_BYTES that
 * every GPU the library runs on holds until the process ends.  Limits: d1, m <= OSSCAR_STATIC_MAX_DIM, any n >= 0;
 * larger sizes return OSSCAR_ENOMEM.  All calls on one GPU share that array: calls that overlap in time on one GPU
 * (different streams or host threads) race and must be serialised by the caller.  After a failure
 * osscar_last_error(NULL) describes it (per host thread). */
#define OSSCAR_STATIC_MAX_DIM 1024
#define OSSCAR_STATIC_SCRATCH_BYTES 21037056
osscar_status osscar_gram_static(const void* X_dev, int64_t n, int64_t ldx, int32_t x_dtype, const void* W_dev, int64_t ldw,
                                 int32_t w_dtype, int64_t d1, int64_t m, double lambda_abs, double lambda_rel, float* H_dev,
                                 float* G_dev, double* scalars_dev, void* hip_stream);

/* Description of the last failure: of a context, or (ctx == NULL) of the last failed call on this host thread that takes
 * no context. */
const char* osscar_last_error(const osscar_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* OSSCAR_H */
