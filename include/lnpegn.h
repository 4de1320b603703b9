/*
 * lnpegn -- LayerNorm backward fused with per-example gradient norms, and the
 * gradient-noise-scale estimator they feed.  C ABI of the MI355X (gfx950) library.
 *
 * Notation.  Activations x and upstream gradients dy are row-major contiguous
 * [B,T,D]: B examples, T positions per example (every dimension between the
 * first and the last is flattened into T), D features.  N = B*T rows.  For a
 * row r:  mu = mean_d x,  var = mean_d (x-mu)^2 (biased),
 * rstd = 1/sqrt(var+eps),  xhat = (x-mu)*rstd,  y = gamma*xhat + beta.
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer unless it says "host".  The caller owns
 *     every buffer, the workspace included.  The library allocates no memory,
 *     frees none and never synchronises.  The only state it keeps is named where
 *     it arises: the benchmarking overrides (lnpegn_set_tuning,
 *     lnpegn_set_profile_events) and the side stream of embedding_pegn.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it and the call returns before it completes; a
 *     call may therefore be captured into a HIP graph.
 *   - Outputs are overwritten, unless a flag of the call says they accumulate.
 *   - The return value is a lnpegn_status.  Arguments are validated on the host before
 *     anything is enqueued: LNPEGN_EINVAL, LNPEGN_EUNSUPPORTED and LNPEGN_EWORKSPACE mean that
 *     nothing was launched and no output was touched.  LNPEGN_EHIP means that the HIP runtime
 *     refused a launch (or an event call); a call is several launches, so those that went out
 *     before the refused one stay enqueued and the outputs are then unspecified.
 *   - Results are bitwise reproducible from call to call for a fixed shape:
 *     no floating-point atomics are used anywhere.
 *   - Index arithmetic is 64-bit; B*T*D may exceed 2^31.
 *   - Any D >= 1 is computed correctly.  The bandwidth-tuned kernels need
 *     D % 8 == 0 (bf16) or D % 4 == 0 (fp32), D <= 16384
 *     and 16-byte aligned x, dy, dx; other cases take a slower generic kernel.
 *   - Loading.  The library links against the HIP runtime (libamdhip64) by its soname.  A
 *     process must hold ONE copy of that runtime: a host program that also loads another
 *     package which ships a HIP runtime of its own (PyTorch-ROCm does) must load that package
 *     first, so that this library binds to the copy already in the process; with two copies
 *     every launch fails with hipErrorNoDevice (reported as LNPEGN_EHIP).
 */
#ifndef LNPEGN_H
#define LNPEGN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LNPEGN_OK = 0,
    LNPEGN_EINVAL = 1,       /* null required pointer, B/T/D <= 0, eps < 0, misaligned pointer ... */
    LNPEGN_EUNSUPPORTED = 2, /* unknown dtype */
    LNPEGN_EWORKSPACE = 3,   /* workspace NULL or smaller than lnpegn_workspace_bytes() */
    LNPEGN_EHIP = 4          /* a HIP launch reported an error */
} lnpegn_status;

/* Storage type of x, dy, dx (and of gamma, see gamma_dt).  Arithmetic is fp32 either way;
 * dx is rounded to the storage type with round-to-nearest-even. */
typedef enum { LNPEGN_F32 = 0, LNPEGN_BF16 = 1 } lnpegn_dtype;

/* Host function, touches no device.  Bytes of workspace that ln_bwd and ln_bwd_pegn need for
 * this shape (the same buffer serves both).  Returns 0 for invalid arguments.  The workspace
 * must be 256-byte aligned; its contents before and after a call are unspecified. */
size_t lnpegn_workspace_bytes(int B, int T, int D, lnpegn_dtype dt);

/* Short English text for a status code (host pointer to a static string). */
const char *lnpegn_status_string(int status);
/* The hipError_t (as an int) behind the calling thread's most recent LNPEGN_EHIP from a backward call's row
 * kernel launch, 0 if there was none: what to look up when a launch is refused. */
int lnpegn_last_hip_error(void);

/*
 * LayerNorm row statistics, the part of the forward pass the backward needs.
 *   x     [N,D] in dt
 *   mean  [N] fp32   mu_r
 *   rstd  [N] fp32   1/sqrt(var_r + eps), biased variance
 * (LayerNorm of Ba et al. 2016, the layer whose backward Section 5.1 of the paper fuses
 * with the per-example norms; two-pass variance in fp32.)
 */
int ln_fwd_stats(const void *x, float *mean, float *rstd, int B, int T, int D, lnpegn_dtype dt,
                 float eps, void *stream);

/*
 * LayerNorm forward: y = gamma*xhat + beta over the last dimension, and the row statistics the
 * backward reuses (the forward half of the forward+backward workload measured in Section 5.1).
 *   x, y      [B,T,D] in dt (y is rounded to dt with round-to-nearest-even; y may alias x)
 *   gamma,beta [D], both in gamma_dt
 *   mean,rstd [N] fp32; either may be NULL if not wanted
 */
int ln_fwd(const void *x, const void *gamma, const void *beta, void *y, float *mean, float *rstd, int B,
           int T, int D, lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *stream);

/*
 * Plain LayerNorm backward (no per-example outputs): the comparison kernel for the paper's
 * "zero overhead" claim of Section 5.1.
 *   x, dy     [B,T,D] in dt
 *   gamma     [D] in gamma_dt
 *   mean,rstd [N] fp32 from ln_fwd_stats, or BOTH NULL to recompute them from x with eps
 *   dx        [B,T,D] in dt:  rstd*(dyh - mean_d(dyh) - xhat*mean_d(dyh*xhat)),  dyh = dy*gamma.
 *             dx may alias dy (in place); it must not alias x.
 *   dgamma    [D] fp32:  sum_{b,t} dy*xhat
 *   dbeta     [D] fp32:  sum_{b,t} dy
 *   workspace >= lnpegn_workspace_bytes(B,T,D,dt) bytes
 */
int ln_bwd(const void *x, const void *dy, const void *gamma, const float *mean, const float *rstd,
           void *dx, float *dgamma, float *dbeta, int B, int T, int D, lnpegn_dtype dt,
           lnpegn_dtype gamma_dt, float eps, void *workspace, size_t workspace_bytes, void *stream);

/*
 * LayerNorm backward fused with per-example gradient norms: Appendix B, algorithm
 * "Layernorm Simultaneous Per-Example Gradient Norm Computation", steps 1-3 and 5-7, in the
 * same single pass over x and dy that produces dx (Section 5.1).  All of ln_bwd's arguments
 * and results, plus
 *   pe_gamma_sq [B] fp32   s_gamma[b] = || sum_t dy[b,t,:]*xhat[b,t,:] ||^2   (steps 1-2)
 *   pe_beta_sq  [B] fp32   s_beta[b]  = || sum_t dy[b,t,:] ||^2               (steps 5-6)
 *   big_sq      [2] fp32   ||dgamma||^2, ||dbeta||^2; may be NULL
 * The per-example squared norms are RAW: the mean over b and the B^2 correction of steps 4
 * and 8 are applied by gns_estimate (pe_scale).
 */
int ln_bwd_pegn(const void *x, const void *dy, const void *gamma, const float *mean,
                const float *rstd, void *dx, float *dgamma, float *dbeta, float *pe_gamma_sq,
                float *pe_beta_sq, float *big_sq, int B, int T, int D, lnpegn_dtype dt,
                lnpegn_dtype gamma_dt, float eps, void *workspace, size_t workspace_bytes,
                void *stream);

/*
 * ln_bwd_pegn for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bitwise the same results as ln_bwd_pegn, without `workspace`: the per-chunk column sums live in a
 * fixed array of LNPEGN_STATIC_SCRATCH_BYTES (64 MiB) that is part of the library's device image, one
 * copy on every GPU the library runs on, held until the process ends.  The call allocates nothing and
 * frees nothing.
 *   - Shapes whose chunk sums need more than that return LNPEGN_EWORKSPACE (nothing is launched);
 *     lnpegn_workspace_bytes(B,T,D,dt) <= LNPEGN_STATIC_SCRATCH_BYTES is sufficient, and all five benchmark
 *     shapes fit (the largest, B=8 T=4096 D=8192, takes 33 MiB).
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress, kept per device) and
 *     must therefore be made outside graph capture; a failure there is LNPEGN_EHIP.
 *   - Every call on a GPU shares that GPU's array, which keeps the last call's contents; nothing in it
 *     needs clearing (every word read was written earlier in the same call).  Two calls in flight on
 *     one GPU at the same time (different streams, or threads) race on it: serialise them.
 */
#define LNPEGN_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int ln_bwd_pegn_static(const void *x, const void *dy, const void *gamma, const float *mean, const float *rstd,
                       void *dx, float *dgamma, float *dbeta, float *pe_gamma_sq, float *pe_beta_sq,
                       float *big_sq, int B, int T, int D, lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps,
                       void *stream);

/*
 * Deferred reduction, for callers that run many LayerNorm layers of one shape (the 24 blocks x 2
 * LayerNorms of a transformer's backward pass).  ln_bwd_deferred / ln_bwd_pegn_deferred take the
 * arguments of ln_bwd / ln_bwd_pegn and run only the pass over x and dy: dx is complete in
 * stream order, while dgamma, dbeta, pe_gamma_sq, pe_beta_sq and big_sq are NOT written yet.
 * The per-chunk column sums (Appendix B steps 1 and 5 over a chunk of rows) and the output
 * pointers stay in that call's workspace, which must therefore be private to the call and left
 * untouched until lnpegn_reduce_deferred has run.  lnpegn_reduce_deferred then finishes n such
 * calls in two launches in all (steps 2, 3, 6, 7 for every layer), instead of two small launches
 * per layer.  Results are bitwise the same as those of the immediate calls.
 *   workspaces  HOST array of n device workspace pointers, each used by one deferred call with
 *               exactly these B, T, D, dt (plain and per-example calls may be mixed)
 */
int ln_bwd_deferred(const void *x, const void *dy, const void *gamma, const float *mean,
                    const float *rstd, void *dx, float *dgamma, float *dbeta, int B, int T, int D,
                    lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *workspace,
                    size_t workspace_bytes, void *stream);
int ln_bwd_pegn_deferred(const void *x, const void *dy, const void *gamma, const float *mean,
                         const float *rstd, void *dx, float *dgamma, float *dbeta,
                         float *pe_gamma_sq, float *pe_beta_sq, float *big_sq, int B, int T, int D,
                         lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *workspace,
                         size_t workspace_bytes, void *stream);
int lnpegn_reduce_deferred(void *const *workspaces, int n, int B, int T, int D, lnpegn_dtype dt,
                           void *stream);

/*
 * The general form of the backward calls above: flags select the per-example outputs
 * (LNPEGN_PER_EXAMPLE: ln_bwd_pegn; without it pe_gamma_sq, pe_beta_sq, big_sq are ignored), the
 * deferred reduction (LNPEGN_DEFER) and gradient accumulation (LNPEGN_ACCUMULATE).
 *
 * LNPEGN_ACCUMULATE is for training with several micro-batches per optimiser step (the setting
 * of the paper's timing figure in Section 5.1 and of its batch-size schedule, Section 5.2):
 * dgamma and dbeta are ADDED to (they must hold valid values, e.g. zeros before the first
 * micro-batch); big_sq receives the squared norms of the accumulated dgamma and dbeta, so after
 * the last micro-batch it is ||G_big||^2 of the whole batch; pe_gamma_sq / pe_beta_sq are those
 * of this micro-batch's B examples, to be placed by the caller at its slice of an [A*B] table.
 * With A micro-batches of B examples and a loss averaged over all of them, gns_estimate is then
 * called with B_big = A*B columns per group and pe_scale = A*B.
 */
typedef enum { LNPEGN_PER_EXAMPLE = 1, LNPEGN_DEFER = 2, LNPEGN_ACCUMULATE = 4 } lnpegn_flags;
int ln_bwd_ex(const void *x, const void *dy, const void *gamma, const float *mean, const float *rstd,
              void *dx, float *dgamma, float *dbeta, float *pe_gamma_sq, float *pe_beta_sq, float *big_sq,
              int B, int T, int D, lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *workspace,
              size_t workspace_bytes, unsigned flags, void *stream);

/*
 * RMSNorm variant (Appendix B remarks that the per-example algorithm carries over unchanged, the
 * gradient being with respect to the affine parameter):  rstd = 1/sqrt(mean_d x^2 + eps),  xhat = x*rstd,
 * y = gamma*xhat; there is no beta.
 *   rms_fwd     y [B,T,D] in dt; rstd [N] fp32 or NULL
 *   rms_bwd_ex  dx = rstd*(dyh - xhat*mean_d(dyh*xhat));  dgamma [D] = sum dy*xhat;
 *               pe_gamma_sq [B] and big_sq [1] = ||dgamma||^2 with LNPEGN_PER_EXAMPLE;
 *               rstd [N] from rms_fwd, or NULL to recompute it from x with eps;
 *               flags, workspace (lnpegn_workspace_bytes) and deferral exactly as for ln_bwd_ex.
 */
int rms_fwd(const void *x, const void *gamma, void *y, float *rstd, int B, int T, int D, lnpegn_dtype dt,
            lnpegn_dtype gamma_dt, float eps, void *stream);
int rms_bwd_ex(const void *x, const void *dy, const void *gamma, const float *rstd, void *dx, float *dgamma,
               float *pe_gamma_sq, float *big_sq, int B, int T, int D, lnpegn_dtype dt, lnpegn_dtype gamma_dt,
               float eps, void *workspace, size_t workspace_bytes, unsigned flags, void *stream);

/*
 * Gradient-noise-scale estimate from per-example norms: Section 2.1, Eq. 4 (unbiased |G|^2),
 * Eq. 5 (S ~ tr Sigma) and Eq. 3 (B_simple = S / |G|^2) with B_small = 1 and B_big = B, after
 * steps 4 and 8 of the Appendix B algorithm (mean over examples, times pe_scale^2).
 *   pe_sq    [n_groups,B] fp32  raw per-example squared norms; every parameter group (each
 *                               layer's gamma and beta) is one row.  Groups are combined by
 *                               adding squared norms, i.e. as one concatenated gradient.
 *   big_sq   [n_groups] fp32    squared norm of each group's summed gradient
 *   pe_scale                    factor that turns a stored per-example gradient into the
 *                               gradient of that example's own loss: B for a mean-reduced
 *                               loss, 1 for a sum-reduced loss
 *   out      [5] fp32           |G_small|^2, |G_big|^2, G2 (Eq. 4), S (Eq. 5), B_simple (Eq. 3)
 * Sums and the estimator are evaluated in fp64.  Nothing is clamped: a non-positive G2 yields
 * the IEEE-754 result (negative, inf or NaN).  B == 1 makes Eq. 4/5 divide by zero and is
 * rejected with LNPEGN_EINVAL.
 */
int gns_estimate(const float *pe_sq, const float *big_sq, int n_groups, int B, float pe_scale,
                 float *out, void *stream);

/*
 * Online smoothing (Section 4.2: both estimators are smoothed with an exponential moving average
 * before the ratio is taken).  A "record" is the five floats gns_estimate writes; records [n][5]
 * (device) holds this step's record for each of n tracked groups (layers, layer types, the total).
 *   state     [n][3] fp64 (device), rows {m_G2, m_S, w}; owned by the caller, updated in place;
 *             all-zero bytes = a fresh tracker.  m <- alpha*m + (1-alpha)*v from zero, and w is the
 *             same recurrence on the constant 1 (= 1 - alpha^t), the weight the average has seen.
 *   smoothed  [n][3] fp32 (device) or NULL: {m_G2/w, m_S/w, m_S/m_G2}; raw IEEE results, no clamping.
 *   alpha in [0,1), else EINVAL.  The paper gives neither the recurrence nor alpha.
 */
int gns_ema_update(double *state, const float *records, int n, double alpha, float *smoothed, void *stream);

/*
 * Offline aggregation (Appendix A, last paragraph; Figure 2 caption): over a history records [n][5]
 * (device) of one group, the plain means of G2 and S, the ratio of the means, and the delete-one
 * jackknife of that ratio.  out [5] fp32 (device) = {mean_G2, mean_S, B_simple = mean_S/mean_G2,
 * stderr, bias-corrected B_simple = n*R - (n-1)*mean_i R_(i)}, where R_(i) is the ratio with step i
 * left out and stderr^2 = (n-1)/n * sum_i (R_(i) - mean R_(.))^2.  n >= 2, else EINVAL.
 */
int gns_offline(const float *records, int64_t n, float *out, void *stream);

/*
 * Linear batch-size schedule of Section 5.1, realised through accumulation steps: host arithmetic,
 * exact in integers.  Returns ceil(accum_final * tokens_seen / ramp_tokens) kept within
 * [1, accum_final] (accum_final once tokens_seen >= ramp_tokens or ramp_tokens == 0), or
 * -LNPEGN_EINVAL for negative arguments or accum_final < 1.
 */
int gns_linear_accum_steps(int64_t tokens_seen, int64_t ramp_tokens, int accum_final);

/*
 * Linear-layer simultaneous per-example gradient norms (Section 3, Algorithm 1, steps 1-3).
 *   x [B,T,K] activations entering the layer, g [B,T,L] gradients w.r.t. its outputs (device,
 *   row-major contiguous, dt = bf16 or fp32; every middle dimension flattened into T).
 *   w [K,L] fp32 (device): sum_b w_b, w_b[k,l] = sum_t x[b,t,k] g[b,t,l]; overwritten, or added to
 *     with LNPEGN_ACCUMULATE (the only flag accepted).
 *   s [B] fp32: raw ||w_b||^2 (step 4's mean and B^2 are gns_estimate's pe_scale, as for LayerNorm).
 *   big_sq [1] fp32 or NULL: ||w||^2 of the (accumulated) weight gradient.
 * The per-example tensor [B,K,L] is never written to memory.  With 16-byte aligned x, g and K, L
 * multiples of 8 (bf16) or 4 (fp32) the contraction runs on the matrix cores (bf16 or fp32 MFMA, fp32
 * accumulation); anything else takes a slow scalar kernel.  workspace: linear_pegn_workspace_bytes(...) bytes, 256-byte aligned, caller-owned,
 * contents scratch.  K*L <= 2^31.  Enqueued on stream, never synchronises; status codes as above.
 */
size_t linear_pegn_workspace_bytes(int B, int T, int K, int L, lnpegn_dtype dt);
int linear_pegn(const void *x, const void *g, float *w, float *s, float *big_sq, int B, int T, int K, int L,
                lnpegn_dtype dt, void *workspace, size_t workspace_bytes, unsigned flags, void *stream);

/*
 * Embedding-layer simultaneous per-example gradient norms (Appendix B, embedding-layer algorithm,
 * steps 1-4; step 5's mean and B^2 are gns_estimate's pe_scale).
 *   ids [B,T] token ids (device; int32, or int64 when ids_are_int64 != 0); an id outside [0,V) is
 *     skipped: its row of g contributes to nothing.
 *   g [B,T,D] gradients w.r.t. the embedding outputs (device, row-major contiguous, bf16 or fp32).
 *   w [V,D] fp32 (device): sum_b w_b, w_b[v,:] = sum_{t: ids[b,t]=v} g[b,t,:]; every row overwritten
 *     (rows of absent ids with zeros), or added to with LNPEGN_ACCUMULATE (the only flag accepted).
 *   s [B] fp32: raw ||w_b||^2.   big_sq [1] fp32 or NULL: ||w||^2 of the (accumulated) gradient.
 * Neither the one-hot tensor nor [B,V,D] is formed; each row of g is read once; no atomics (bitwise
 * reproducible).  workspace: embedding_pegn_workspace_bytes(...) bytes (0 if the shape is invalid or
 * no device is present: the sort's scratch is sized for the current device), 256-byte aligned,
 * caller-owned, contents scratch.  B*T < 2^31, V < 2^30.  Enqueued on stream, never synchronises.
 * Without LNPEGN_ACCUMULATE the zero fill of w (of the rows that no id selects) runs on a side stream that the library creates once per
 * device (default priority, kept until the process ends), forked from and joined back to `stream` with
 * events inside this call: to the caller the call is still one piece of work on `stream`; calls issued
 * from several streams of one device share the side stream and may serialise on it.
 */
size_t embedding_pegn_workspace_bytes(int B, int T, int D, int V);
/*
 * The same computation with the sort taken off the backward pass.  The ids are known when the forward pass runs:
 * embedding_sort_ids sorts them there (stable: by id, positions b*T+t ascending inside an id; ids outside [0,V)
 * get the key V and sort last), and embedding_pegn_presorted takes the two sorted arrays in place of ids.  Results
 * are bitwise those of embedding_pegn.
 *   sorted_ids, sorted_pos [B*T] uint32 (device), the caller's: written by embedding_sort_ids, read by
 *     embedding_pegn_presorted, which requires exactly that order (it is not checked).
 *   workspace: embedding_pegn_workspace_bytes(B, T, D, V) for embedding_pegn_presorted,
 *     embedding_pegn_workspace_bytes(B, T, 1, V) suffices for embedding_sort_ids.
 * Without the sort in front of it the zero fill of the rows that no id selects runs beside the kernels that read g.
 */
int embedding_sort_ids(const void *ids, int ids_are_int64, int B, int T, int V, uint32_t *sorted_ids,
                       uint32_t *sorted_pos, void *workspace, size_t workspace_bytes, void *stream);
int embedding_pegn_presorted(const uint32_t *sorted_ids, const uint32_t *sorted_pos, const void *g, float *w, float *s,
                             float *big_sq, int B, int T, int D, int V, lnpegn_dtype dt, void *workspace,
                             size_t workspace_bytes, unsigned flags, void *stream);
int embedding_pegn(const void *ids, int ids_are_int64, const void *g, float *w, float *s, float *big_sq, int B, int T,
                   int D, int V, lnpegn_dtype dt, void *workspace, size_t workspace_bytes, unsigned flags, void *stream);

/*
 * Benchmarking aid.  Overrides launch-shape heuristics process-wide; it never changes results
 * beyond floating-point summation order.  key 0: target number of row chunks of ln_bwd_pegn
 * (0 = automatic); key 1: the same for ln_bwd; key 2: waves per workgroup of the row kernel
 * (0 = automatic, else 1..16); key 3: rows between the sweep starts of consecutive examples,
 * plus one (0 = automatic); key 4: neighbouring chunks on one XCD (0 automatic, 1 never, 2 always);
 * key 5: cap on 16-byte vectors per lane and array of the row kernel (0 = automatic, else 1..4: fewer
 * means more waves share a row); key 6: workgroups (per group of four column blocks) of
 * embedding_pegn's run kernel, 1..65535 (default 4096; with fewer than one per 16 positions each
 * workgroup loops); key 7: dx stores of the row kernel (0 automatic: write-through while dx is at most
 * 96 MiB, streaming above; 1 always streaming; 2 always write-through); key 8: rows of a chunk (0 automatic:
 * every C-th row of its example up to 32 examples, a block of consecutive rows above; 1 always the former;
 * 2 always the latter).
 * Returns LNPEGN_EINVAL for an unknown key or a value out of range.  Not thread-safe against concurrent launches.
 */
int lnpegn_set_tuning(int key, int value);

/*
 * Benchmarking and testing aid, host only (touches no device): the launch plan that ln_bwd (per_example = 0) or
 * ln_bwd_pegn (per_example = 1) would use for this shape under the tuning in force, with 16-byte aligned pointers
 * (aligned = 1: the vector kernels where the row width allows) or without (aligned = 0: the generic kernel).
 * Writes min(n_out, LNPEGN_PLAN_FIELDS) values to the HOST array out, in this order:
 *    0 vector kernel (1) or generic kernel (0)      1 waves per row                2 row groups per workgroup
 *    3 16-byte vectors per lane and array           4 chunks per example (of the whole tensor for ln_bwd)
 *    5 chunks in all = workgroups of the row kernel 6 rows of a chunk when they are consecutive, else 0 (every
 *      C-th row)                                    7 rows between the sweep starts of consecutive examples
 *    8 chunks per XCD when an example's chunks are kept on one XCD, else 0
 *    9 bytes of LDS per workgroup                  10 the row kernel finishes the per-example norms itself (1/0)
 *   11 examples whose norms the reduction finishes 12 groups of chunks in the reduction   13 chunks per group
 *   14 workspace bytes of this plan                15 rows per example (B*T for ln_bwd)
 * Returns LNPEGN_EINVAL for an invalid shape or a null out, LNPEGN_EUNSUPPORTED for an unknown dtype.
 */
#define LNPEGN_PLAN_FIELDS 16
int lnpegn_plan_query(int B, int T, int D, lnpegn_dtype dt, int per_example, int aligned, int64_t *out, int n_out);

/*
 * Benchmarking aid, one-shot.  The next ln_bwd or ln_bwd_pegn call attaches the two hipEvent_t
 * to the dispatch of its row-streaming kernel (start of execution, end of execution), so that
 * hipEventElapsedTime(start, stop) is that kernel's own duration; then it forgets both.  The
 * caller owns the events.  Passing two NULLs disarms.  Returns LNPEGN_EINVAL if exactly one of
 * them is NULL.  Not thread-safe.
 */
int lnpegn_set_profile_events(void *start_event, void *stop_event);

/*
 * Benchmarking aid: a plain streaming kernel of known traffic, the yardstick for the row
 * kernels (empirical bandwidth ceiling of the machine, and the scale of hardware byte
 * counters).  mode 0: out = a (one read, one write); mode 1: out = a XOR b (two reads, one
 * write -- the access mix of the LayerNorm backward), four vectors per lane, ordinary loads and
 * stores; mode 2: the same two reads and one write as one-shot workgroups of one vector per lane with
 * streaming loads and stores (the fastest plain form found).  `bytes` is the size of EACH array and
 * must be a multiple of 16; a, b, out are 16-byte aligned device pointers (b is ignored in
 * mode 0).  Honours lnpegn_set_profile_events like the backward calls.
 */
int lnpegn_stream_probe(const void *a, const void *b, void *out, size_t bytes, int mode,
                        void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LNPEGN_H */
