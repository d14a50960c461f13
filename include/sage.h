/*
 * sage.h -- C ABI of the MI355X (gfx950) SAGE hot-path library.
 *
 * SAGE (arxiv 2510.02470) selects a training subset in two streaming passes over per-example gradient rows
 * g_i in R^D:  pass 1 keeps a Frequent Directions (FD) sketch of the rows (Method, FD paragraph; Algorithm 1,
 * Phase I); pass 2 projects each row on the frozen sketch, normalises, forms the consensus direction and scores
 * each row by its cosine to it, then keeps the top fraction (Method, "Two-pass scoring"; Algorithm 1, Phase II
 * and the "Select top-k" line).
 *
 * Conventions
 *   - Every pointer argument says whether it is HOST or DEVICE memory. DEVICE means memory of the GPU that was
 *     current when the context was created. The library owns the sketch, the basis, the score store and all
 *     work space; the caller owns every G_batch, every output array and keeps them valid until the call's work
 *     has completed on the context's stream (sage_sync, sage_select, sage_stats and the export calls wait).
 *   - Work is enqueued on one HIP stream per context, given at creation (NULL = the default stream). Calls on
 *     one context must not overlap in time.
 *   - Rows are row-major with leading dimension D (no padding): element (i, d) of a batch is at i*D + d.
 *   - ell is the sketch size; the buffer holds n = 2*ell rows; k is the rank of the scoring basis; the example
 *     index of a scored row is its 0-based arrival order within the scoring pass.
 *   - Every call returns 0 on success or a negative sage_status; nothing throws. Non-finite input is not
 *     detected and gives unspecified (but memory-safe) results, unless sage_set_debug_checks is on.
 *   - A call that fails with SAGE_ERR_ARG, SAGE_ERR_STATE, SAGE_ERR_CAPACITY or SAGE_ERR_ALLOC leaves the context
 *     as it was. A call that fails with SAGE_ERR_HIP (a runtime call or a kernel launch failed after part of the
 *     call's work was enqueued) leaves it poisoned: every later call on it returns SAGE_ERR_STATE; only
 *     sage_destroy is still allowed.
 */
#ifndef SAGE_H
#define SAGE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sage_ctx sage_ctx;

typedef enum {
    SAGE_F32 = 0, /* rows are IEEE binary32 */
    SAGE_BF16 = 1 /* rows are bfloat16 (upper half of a binary32); widened exactly, all arithmetic in fp32 */
} sage_dtype;

typedef enum {
    SAGE_OK = 0,
    SAGE_ERR_ARG = -1,      /* bad argument (null pointer, size out of range) */
    SAGE_ERR_STATE = -2,    /* call not allowed in the context's current state */
    SAGE_ERR_ALLOC = -3,    /* device or host allocation failed */
    SAGE_ERR_HIP = -4,      /* a HIP runtime call or kernel launch failed */
    SAGE_ERR_CAPACITY = -5  /* fixed-capacity store or output array too small */
} sage_status;

typedef struct {
    int64_t rows_seen;   /* rows given to sage_fd_update so far */
    int64_t n_shrinks;   /* shrink steps performed */
    int64_t n_scored;    /* rows given to sage_score since the last sage_fd_basis / sage_set_basis */
    double sum_delta;    /* sum of the delta of every shrink: upper bound on ||A^T A - B^T B||_2 */
    double frob2;        /* ||A||_F^2 of the rows seen, fp32 products accumulated in fp32/fp64 */
    double last_delta;   /* delta of the most recent shrink */
    int last_sweeps;     /* Jacobi sweeps used by the most recent eigensolve (100 + the sweeps launched if they did
                            not reach the tolerance; the next solves then launch the full number) */
    int fill;            /* buffer rows in use, 0..2*ell-1 */
    int64_t n_unconverged; /* eigensolves so far (shrinks and bases) that ended above their tolerance: sticky. Such a
                            shrink is still a valid FD step (the rows are rotated by an exactly orthogonal matrix and
                            damped; the Gram block the next cycle takes as known includes what was left off the
                            diagonal), but its delta is not exactly sigma_ell^2 */
    double last_offdiag; /* largest |off-diagonal| / trace the most recent eigensolve left */
} sage_stats_t;

/* ---- the five calls of the path --------------------------------------------------------------------------- */

/*
 * Create a context for an FD sketch of fp32 rows on the default stream: a zeroed buffer of 2*ell rows by D
 * columns, fill pointer 0 (Algorithm 1, "Initialize S <- 0, row counter r <- 0"; the buffer has 2*ell rows so
 * that new rows only ever land in zero rows, Liberty's form of FD).
 * out: HOST pointer receiving the handle. 2 <= ell <= 256, D >= 1. Device memory: about 2*ell*D*4 bytes for the
 * sketch plus work space; SAGE_ERR_ALLOC if it does not fit.
 */
int sage_fd_create(sage_ctx** out, int ell, int64_t D);

/*
 * As above with the row type, a score-store capacity and a stream. max_rows > 0 fixes the number of rows one
 * scoring pass may hold (sage_score returns SAGE_ERR_CAPACITY beyond it); 0 lets the store grow by doubling.
 * hip_stream: a hipStream_t passed as void* (NULL = default stream); it must outlive the context.
 */
int sage_fd_create_ex(sage_ctx** out, int ell, int64_t D, sage_dtype in_dtype, int64_t max_rows,
                      void* hip_stream);

/*
 * Pass 1 (Algorithm 1, Phase I): append `rows` rows to the sketch. Each row is copied into the next free buffer
 * row; whenever the buffer becomes full the shrink step runs: with sigma_j, v_j the singular values / right
 * singular vectors of the buffer, delta = sigma_ell^2 and row j becomes sqrt(max(sigma_j^2 - delta, 0)) v_j^T
 * (Method, FD paragraph). It is computed as: Gram C = B B^T (fp32 matrix cores, split over D, partial sums added
 * in fp64) -> Jacobi eigensolve C = Y Lambda Y^T (fp64) -> B[0:ell] <- diag(w) Y^T B with
 * w_j = sqrt(max(lambda_j - delta, 0) / lambda_j) (fp32 matrix cores), rows ell.. zeroed.
 * G_batch: DEVICE, rows x D of the context's dtype. rows >= 0 (0 is a no-op). Asynchronous on the context's
 * stream. Invalidates a basis made earlier. The host never reads device data in this call.
 * When a call ends exactly on a full buffer, that shrink is left for the next sage_fd_update (which can then overlap
 * part of it with the storing of its own first rows) or for the first call that looks at the sketch (sage_fd_basis,
 * sage_stats, the exports and probes); results are the same either way. Part of the work runs on a second stream
 * owned by the context; the batch is free for reuse once the call's work is complete on the context's stream.
 */
int sage_fd_update(sage_ctx* ctx, const void* G_batch, int64_t rows);

/*
 * Freeze the sketch (Algorithm 1, "Freeze S for scoring") and form the scoring basis: the top-k right singular
 * vectors of the buffer as it stands (filled rows and zero rows; no shrink; the sketch is left unchanged).
 * A direction whose sigma_j^2 <= 2*ell * 2^-23 * sigma_1^2 is returned as the zero vector.
 * 1 <= k <= min(ell-1, 128) (SAGE_ERR_ARG otherwise; 128 is this library's limit: the score kernels keep two
 * coordinates per lane).
 * Resets the scoring pass (row count, consensus sum, score store). Asynchronous.
 */
int sage_fd_basis(sage_ctx* ctx, int k);

/*
 * As sage_fd_basis, but row j of the basis is sqrt(max(sigma_j^2 - delta, 0)) v_j^T with delta = sigma_ell^2 of the
 * buffer as it stands: the first k rows of the sketch S = Sigma' V^T that a shrink would write, so that sage_score
 * computes the paper's own projection z = S g (Method, "Two-pass scoring"; Algorithm 1, Phase II) on its k leading
 * rows. Right after a shrink these are the sketch rows themselves. The sketch is left unchanged.
 */
int sage_fd_basis_weighted(sage_ctx* ctx, int k);

/*
 * Pass 2 (Algorithm 1, Phase II, first line): for each row g of the batch z = V_k^T g, zhat = z/||z||_2 (0 if
 * z = 0); zhat is stored at the row's example index and added to the consensus sum.
 * G_batch: DEVICE, rows x D of the context's dtype. Needs a basis (else SAGE_ERR_STATE). Asynchronous.
 */
int sage_score(sage_ctx* ctx, const void* G_batch, int64_t rows);

/*
 * Finish pass 2 (Algorithm 1, Phase II: "zbar", "u", "alpha_i", "Select top-k by alpha_i"): u = sum(zhat) /
 * ||sum(zhat)||_2 (0 if the sum is 0; the 1/N factor cancels), alpha_i = <zhat_i, u> clamped to [-1, 1] with -0
 * stored as +0, m = floor(keep_rate*N + 0.5) clipped to [0, N], and the m indices that are greatest under
 * (alpha descending, index ascending) are written in ascending index order.
 * keep_rate in [0, 1]. out_idx: DEVICE, room for `cap` int64 (SAGE_ERR_CAPACITY if m > cap; may be NULL when
 * cap = 0 and m = 0). out_m: HOST, receives m. Waits for the stream. May be called again (e.g. another rate).
 */
int sage_select(sage_ctx* ctx, double keep_rate, int64_t* out_idx, int64_t cap, int64_t* out_m);

/*
 * Class-balanced variant, CB-SAGE (Algorithm 1, "if class balance required"; "Agreement Scoring and Selection").
 * sage_score_labeled is sage_score with the class label of every row: labels: DEVICE, `rows` int32, each in
 * [0, n_classes) of the later sage_select_cb call (checked there). A pass must be scored entirely with labels to be
 * selected class by class (SAGE_ERR_STATE otherwise); sage_select may still be called on it.
 *
 * sage_select_cb: for every class c, zbar_c = mean of zhat over its rows, u_c = zbar_c / ||zbar_c||_2 (0 if the sum is 0),
 * alpha_i = <zhat_i, u_c(i)> clamped to [-1, 1] (-0 stored as +0), and the k_c rows of the class that are greatest under
 * (alpha descending, index ascending) are kept. The paper asks for sum_c k_c = k and leaves the k_c open; here the
 * subset size is the plain selection's m = floor(keep_rate * N + 0.5), class c gets floor(keep_rate * N_c), and the rows
 * still missing from m go one each to the classes with the largest fractional part of keep_rate * N_c (equal parts:
 * the lower class first) that are not yet full -- proportional budgets that sum to m exactly (SAGE_CB_PROPORTIONAL,
 * what sage_select_cb uses). sage_select_cb_ex takes the rule: SAGE_CB_EQUAL deals the m rows one at a time to the classes
 * in turn, lowest class first, passing over a class that is full -- every class ends with the same budget up to one
 * row and up to its size. All kept indices are
 * written in ascending order. out_idx: DEVICE, room for `cap` int64 (SAGE_ERR_CAPACITY if sum(k_c) > cap); out_m: HOST, receives
 * sum(k_c). 1 <= n_classes <= 65536. A label outside [0, n_classes) gives SAGE_ERR_ARG. Waits for the stream.
 * sage_scores / sage_scores_export then give these class-wise scores. Class sums are accumulated in 64-bit fixed
 * point (2^-40 resolution), so the result does not depend on the order in which the device adds.
 */
int sage_score_labeled(sage_ctx* ctx, const void* G_batch, const int32_t* labels, int64_t rows);
typedef enum { SAGE_CB_PROPORTIONAL = 0, SAGE_CB_EQUAL = 1 } sage_cb_rule;
int sage_select_cb(sage_ctx* ctx, double keep_rate, int n_classes, int64_t* out_idx, int64_t cap, int64_t* out_m);
int sage_select_cb_ex(sage_ctx* ctx, double keep_rate, int n_classes, int rule, int64_t* out_idx, int64_t cap,
                      int64_t* out_m);

/*
 * Scoring without the N x k store of zhat (Abstract: O(l D) memory, no explicit N x l store). With
 * store_zhat = 0, sage_score only accumulates the consensus sum (rows are counted, nothing per row is kept), and a
 * further pass over the same rows in the same order, sage_rescore, recomputes zhat_i and writes alpha_i =
 * clamp(<zhat_i, u>, -1, 1) (4 bytes per row); sage_select then selects from those. The scores are bit-equal to the
 * stored run's. store_zhat = 1 (the default) is the two-pass run. Either call resets the scoring pass.
 * In the store-free run: sage_score after the first sage_rescore, sage_rescore of more rows than were scored,
 * sage_select before every row has been rescored, sage_score_labeled / sage_select_cb and sage_zhat_export return
 * SAGE_ERR_STATE. G_batch: DEVICE, as for sage_score. Asynchronous on the context stream.
 */
int sage_set_score_store(sage_ctx* ctx, int store_zhat);
int sage_rescore(sage_ctx* ctx, const void* G_batch, int64_t rows);

/* Release the context and everything it owns (waits for its stream). NULL is allowed. */
void sage_destroy(sage_ctx* ctx);

/* ---- auxiliaries for tests, harnesses and callers that need the intermediate results ---------------------- */

/* Wait until all work enqueued by this context has completed. */
int sage_sync(sage_ctx* ctx);

/*
 * Merge another sketch into this one (Method, FD paragraph: the sketch is the Frequent Directions sketch, which is
 * mergeable -- feeding the rows of one sketch to another as if they were data gives a sketch of the two streams
 * together whose covariance error is at most the sum of the two sum_delta plus what this context's later shrinks add).
 * B_other: DEVICE, rows x D fp32 row-major (e.g. the first `fill` rows of sage_fd_sketch_export's output of the other
 * context: all the rows its buffer holds), whatever this context's row type is; rows >= 0. The rows go through the
 * same insert / shrink cycle as sage_fd_update's; sage_stats counts them like data rows (rows_seen, frob2 = their
 * squared norms). Asynchronous on
 * the context stream like sage_fd_update; invalidates the basis. The building block for sharding a stream by rows.
 */
int sage_fd_merge(sage_ctx* ctx, const float* B_other, int64_t rows);

/*
 * Rows given by their two factors (Method, definition of g_i as the per-example gradient, taken for a linear last
 * layer with n_classes x n_features weights followed by n_classes biases and a loss on its logits: the gradient is the
 * outer product of the logit error e_i = dL/dlogits with [h_i; 1], h_i the layer's input). Row i of the batch is
 *     g_i[c * n_features + t] = e_i[c] * h_i[t],     g_i[n_classes * n_features + c] = e_i[c],
 * with every product rounded as a stored row of the context's type would hold it (fp32: the fp32 product; bf16: the
 * exact product rounded to nearest even), so that each call below computes exactly what its row-major counterpart
 * (sage_fd_update, sage_score / sage_score_labeled, sage_rescore) computes on those rows -- the sketch bit for bit,
 * projections up to the order of fp32 summation -- while the D-long rows are never stored or read: the update writes
 * them straight into the sketch buffer, the scoring pass forms them in registers.
 * E: DEVICE, rows x n_classes row-major; H: DEVICE, rows x n_features row-major (16-byte aligned); both of the
 * context's row type; n_classes * (n_features + 1) must equal D (SAGE_ERR_ARG otherwise). labels: DEVICE, rows int32,
 * or NULL. The in-register projection needs n_features to be a multiple of 128 bytes of the row type (64 bf16, 32
 * fp32 values); for other shapes the rows are written to a staging buffer of rows x D values, at most 2048 rows at a
 * time, and projected from there (in the store-free run the scores of such shapes equal the stored run's bit for bit
 * only when both passes cut the stream into the same batches: the order of summation follows a row's place in the
 * staging buffer). Asynchronous on the context stream; state rules and errors as for the row-major calls.
 */
int sage_fd_update_outer(sage_ctx* ctx, const void* E, const void* H, int64_t rows, int64_t n_classes,
                         int64_t n_features);
int sage_score_outer(sage_ctx* ctx, const void* E, const void* H, const int32_t* labels, int64_t rows,
                     int64_t n_classes, int64_t n_features);
int sage_rescore_outer(sage_ctx* ctx, const void* E, const void* H, int64_t rows, int64_t n_classes,
                       int64_t n_features);

/*
 * Copy the sketch buffer to B_out as a plain row-major (2*ell) x D fp32 matrix (the library keeps it in a
 * column-slab layout internally). B_out: DEVICE, 2*ell*D floats. Rows >= fill are zero. Waits for the stream.
 */
int sage_fd_sketch_export(sage_ctx* ctx, float* B_out);

/* Copy the scoring basis to Vt_out, row-major k x D fp32, row j = v_j^T. Vt_out: DEVICE. Needs a basis. Waits. */
int sage_basis_export(sage_ctx* ctx, float* Vt_out);

/*
 * Install a basis given by the caller instead of the sketch's (stage-isolated tests; also lets a caller score
 * against a basis saved earlier). Vt: DEVICE, row-major k x D fp32, 1 <= k <= 128. Resets the scoring pass.
 */
int sage_set_basis(sage_ctx* ctx, const float* Vt, int k);

/*
 * Arithmetic of the projection z = V_k^T g (Algorithm 1, Phase II, first line). SAGE_PROJ_AUTO (default): when
 * every row of a batch starts on a 16-byte boundary (D * element size a multiple of 16, batch pointer 16-byte
 * aligned, D >= 64 for bf16 / 32 for fp32 rows, D * element size < 16 MiB) the products run on the bf16 matrix cores
 * with every fp32 basis entry split as hi + lo (two bf16, relative error <= 2^-17) and fp32 rows split the same
 * way, accumulated in fp32; otherwise, and always under SAGE_PROJ_F32, on the fp32 matrix cores. Drops the current
 * basis: call before sage_fd_basis / sage_set_basis.
 */
typedef enum { SAGE_PROJ_AUTO = 0, SAGE_PROJ_F32 = 1 } sage_proj_mode;
int sage_set_projection_mode(sage_ctx* ctx, int mode);

/*
 * Arithmetic of the shrink's dense products: the Gram blocks C = B B^T and the rebuild S <- Sigma' V^T = diag(w) Y^T B
 * (Method, FD paragraph; Algorithm 1, Phase I). SAGE_MM_SPLIT (default): every fp32 value is written as three bf16
 * parts (24 significant bits) and the six partial products that matter run on the bf16 matrix cores, accumulated in
 * fp32 -- the fp32 result to within a few 2^-24 per term, at a multiple of the fp32 matrix-core rate. It is used where
 * a kernel exists: the rebuild for ell >= 97 (padded sketch size 128 or 256), the Gram blocks of the steady state
 * (new rows x top rows, new rows x new rows) for ell >= 193 (padded size 256); everything else, and everything under
 * SAGE_MM_F32, runs on the fp32 matrix cores. Rows that arrive through sage_fd_update or sage_fd_update_outer in a bf16 context
 * are bf16 values kept as fp32: they have one part, not three, and the split kernels leave out the products with their (zero) second
 * and third parts -- three products instead of six wherever a buffered row of the stream is a factor, with the same
 * bits as the result. SAGE_MM_SPLIT_ALL_PARTS is SAGE_MM_SPLIT without that shortcut (a check that the bits are indeed
 * the same, and the rate fp32 rows would see). May be changed at any time between calls.
 */
typedef enum { SAGE_MM_F32 = 0, SAGE_MM_SPLIT = 1, SAGE_MM_SPLIT_ALL_PARTS = 2 } sage_mm_mode;
int sage_set_update_arithmetic(sage_ctx* ctx, int mode);

/* View of the scores of the last sage_select: *alpha receives a DEVICE pointer to N fp32 owned by the library,
 * valid until the next scoring call; *n receives N. HOST pointers. */
int sage_scores(sage_ctx* ctx, const float** alpha, int64_t* n);

/* Copy the scores of the last sage_select (N fp32) to alpha_out (DEVICE, N floats). Waits. */
int sage_scores_export(sage_ctx* ctx, float* alpha_out);

/* Copy the stored normalised projections of the current scoring pass (N x k fp32 row-major) to zhat_out
 * (DEVICE, N*k floats). Waits. */
int sage_zhat_export(sage_ctx* ctx, float* zhat_out);

/* Counters of the context (HOST struct). Waits for the stream. */
int sage_stats(sage_ctx* ctx, sage_stats_t* out);

/*
 * Stand-alone top-m (Algorithm 1, "Select top-k by alpha_i") of any fp32 score vector: the m indices greatest
 * under (alpha descending, index ascending), written ascending. alpha: DEVICE, N floats (NaN not allowed);
 * out_idx: DEVICE, m int64; 0 <= m <= N; hip_stream as in sage_fd_create_ex. Allocates and frees its own work
 * space; returns after the result is complete.
 */
int sage_topm(const float* alpha, int64_t N, int64_t m, int64_t* out_idx, void* hip_stream);

/*
 * sage_topm for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc. Same arguments and result as sage_topm, but the work space (a histogram, the
 * select state and two counters per block of 2048 keys, 67 KB in all) is a fixed array inside the library, one copy
 * per GPU, held until the process ends; the call allocates and frees nothing and does not wait: the work is enqueued
 * on hip_stream and out_idx is complete when that stream reaches the end of it. N > SAGE_TOPM_STATIC_MAX_N gives
 * SAGE_ERR_CAPACITY. All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race; calls on one stream, or otherwise ordered, are safe -- every call clears what it needs
 * cleared with its own first kernel.
 */
#define SAGE_TOPM_STATIC_MAX_N 16777216
int sage_topm_static(const float* alpha, int64_t N, int64_t m, int64_t* out_idx, void* hip_stream);

/*
 * Stage probes for tests: run the Gram of the current buffer (C_out: DEVICE, n_pad*n_pad doubles, row-major,
 * n_pad returned in *n_pad) and, if eig != 0, the Jacobi eigensolve of it (Y_out: DEVICE n_pad*n_pad doubles
 * with eigenvectors in columns, lam_out: DEVICE n_pad doubles, unsorted). Any output pointer may be NULL.
 * The sketch is not modified. Waits.
 */
int sage_probe_gram_eig(sage_ctx* ctx, double* C_out, int eig, double* Y_out, double* lam_out, int* n_pad);

/*
 * Stage probe: the two Gram blocks of the steady-state cycle, (new rows) x (top rows) and (new rows) x (new rows),
 * formed by the split-arithmetic kernels (see sage_set_update_arithmetic) from the current buffer. C_out as above
 * (buffer-row order, both triangles); its top x top block is zero. SAGE_ERR_STATE when this sketch size has no such
 * kernels (ell < 193). The sketch is not modified. Waits.
 */
int sage_probe_gram_split(sage_ctx* ctx, double* C_out, int* n_pad);

/*
 * Stage probe: run the context's Jacobi eigensolve on a symmetric matrix given by the caller. C_in: DEVICE,
 * n_pad*n_pad doubles (n_pad as reported by sage_probe_gram_eig), left untouched. Y_out, lam_out as above.
 * sweep_stat_out: DEVICE, 18 doubles: [0] trace, [1+s] largest |off-diagonal| / trace met in sweep s (0 for
 * sweeps that were skipped), [17] the number of sweeps launched. Outputs may be NULL. The sketch is not modified. Waits.
 */
int sage_probe_eig_matrix(sage_ctx* ctx, const double* C_in, double* Y_out, double* lam_out, double* sweep_stat_out);

/*
 * A plain device-to-device copy kernel of `bytes` bytes (16 bytes per work-item; bytes and both DEVICE pointers
 * multiples of 16), asynchronous on hip_stream. Harnesses run it under a profiler to learn what the memory-traffic
 * counters report for a known amount of traffic (bytes read, bytes written), and scale the readings of the path's
 * kernels by that.
 */
int sage_copy_probe(void* dst, const void* src, int64_t bytes, void* hip_stream);

/*
 * Per-kernel timing for harnesses: when enabled, every kernel launch is bracketed by HIP events on the
 * context's stream (this serialises host and device, so whole-call timings taken while it is on are not
 * representative). sage_profile_read waits, then reports the accumulated milliseconds and launch count of
 * the kernel class `which` (0 gram, 1 gram reduce, 2 eigensolve, 3 coefficients, 4 rebuild/basis, 5 insert,
 * 6 project, 7 score finalise, 8 select) and clears that class.
 */
int sage_profile_enable(sage_ctx* ctx, int on);
int sage_profile_read(sage_ctx* ctx, int which, double* ms, int64_t* launches);

/*
 * How many Jacobi sweeps a shrink's eigensolve may use (Method, FD paragraph: the SVD of the buffer). Sweeps are
 * enqueued ahead of time, and a sweep that finds the matrix already diagonal to tolerance returns at once, but its
 * launches still cost time (about 50 us per sweep at ell = 256). SAGE_SWEEPS_ADAPTIVE (default): as many sweeps as
 * the most demanding of the last eight solves whose count has come back needed, plus two; a solve that still ends above the tolerance is
 * counted in sage_stats_t.n_unconverged (and the next 64 solves get every sweep); such a shrink remains a valid step,
 * see there. SAGE_SWEEPS_ALL: always the full 14 sweeps, for streams whose spectrum may change abruptly from one
 * cycle to the next: no solve ends early for want of sweeps, at about 4% of the update rate at ell = 256.
 * sage_fd_basis always has every sweep. May be changed between calls.
 */
typedef enum { SAGE_SWEEPS_ADAPTIVE = 0, SAGE_SWEEPS_ALL = 1 } sage_sweep_policy;
int sage_set_sweep_policy(sage_ctx* ctx, int policy);

/*
 * Debug checks of caller data (off by default: they cost a pass over the batch and a wait). With on != 0,
 * sage_fd_update, sage_fd_merge, sage_fd_update_outer, sage_score, sage_score_labeled and sage_score_outer first
 * scan their batch (the factors, for the factored calls) and return SAGE_ERR_ARG, leaving the context as it was, if
 * any entry is an infinity or a NaN.
 */
int sage_set_debug_checks(sage_ctx* ctx, int on);

/*
 * Test hook for the error path: the nth kernel launch from now that the context issues for its main sequence (Gram,
 * reduce, eigensolve, coefficients, rebuild, insert, projection, finalise, select) is not made and is reported as a
 * failed launch instead, so that the call in progress returns SAGE_ERR_HIP and the context becomes poisoned exactly as
 * after a real launch failure. Nothing faulty runs on the GPU. nth = 0 disarms the hook.
 */
int sage_debug_fail_launch(sage_ctx* ctx, int nth);

/* Static description of a status code (HOST string, never NULL). */
const char* sage_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SAGE_H */
