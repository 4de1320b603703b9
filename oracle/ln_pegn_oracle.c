/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * Plain, slow, fp64 CPU definition of what the fused LayerNorm-backward +
 * per-example-gradient-norm path computes.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may build, link or call this file.  It
 * shares no code, header, table or helper with the HIP library and includes
 * nothing but the C standard library.
 *
 * What is defined here, and where the definition comes from:
 *
 *   - LayerNorm over the last dimension (Ba et al. 2016, the layer the paper's
 *     Section 5.1 kernel is built for): biased variance, eps inside the square
 *     root, y = gamma * xhat + beta.
 *   - Its backward pass for ONE example, written from the chain rule
 *     (validated in the tests by finite differences of the forward).
 *   - Per-example parameter gradients and their squared norms, Appendix B,
 *     "Layernorm Simultaneous Per-Example Gradient Norm Computation":
 *       gamma'_b[k] = sum_t xhat[b,t,k] * g[b,t,k]      (step 1)
 *       s_gamma[b]  = sum_k gamma'_b[k]^2               (step 2)
 *       gamma'[k]   = sum_b gamma'_b[k]                 (step 3)
 *       beta'_b[k]  = sum_t g[b,t,k]                    (step 5)
 *       s_beta[b]   = sum_k beta'_b[k]^2                (step 6)
 *       beta'[k]    = sum_b beta'_b[k]                  (step 7)
 *     The "activation" entering step 1 is the normalised activation xhat, the
 *     input of the affine transform, because the gradient is taken with
 *     respect to the affine parameters (Appendix B, remark on RMSNorm).
 *     The method is a re-association of these sums, so the oracle is the sums
 *     themselves, by brute force: a separate backward pass per example.
 *   - Steps 4 and 8 (mean over examples times B^2) and the unbiased
 *     estimators of Section 2.1, Eq. 4 (|G|^2), Eq. 5 (S ~ tr Sigma) and
 *     Eq. 3 (B_simple = S / |G|^2).
 *
 * All inputs and outputs are double.  Callers that test a bf16 or fp32 GPU
 * path pass the already-rounded input values converted (exactly) to double.
 *
 * Every function returns 0 on success and a negative number on bad arguments.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- LayerNorm row statistics: mean, biased variance, rstd = 1/sqrt(var+eps) ---- */
static void row_stats(const double *x, long D, double eps, double *mean, double *rstd)
{
    double sum = 0.0;
    for (long d = 0; d < D; ++d) sum += x[d];
    const double mu = sum / (double)D;
    double ss = 0.0;
    for (long d = 0; d < D; ++d) {
        const double c = x[d] - mu;
        ss += c * c;
    }
    const double var = ss / (double)D; /* biased: divide by D */
    *mean = mu;
    *rstd = 1.0 / sqrt(var + eps);
}

/* mean[N], rstd[N] of x[N,D] */
int lnpegn_oracle_ln_stats(const double *x, long N, long D, double eps, double *mean, double *rstd)
{
    if (!x || !mean || !rstd || N <= 0 || D <= 0 || eps < 0.0) return -1;
    for (long r = 0; r < N; ++r) row_stats(x + r * D, D, eps, &mean[r], &rstd[r]);
    return 0;
}

/* Forward: y[N,D] = gamma * xhat + beta.  Used by the tests for finite differences. */
int lnpegn_oracle_ln_fwd(const double *x, const double *gamma, const double *beta, long N, long D,
                         double eps, double *y)
{
    if (!x || !gamma || !beta || !y || N <= 0 || D <= 0 || eps < 0.0) return -1;
    for (long r = 0; r < N; ++r) {
        double mu, rstd;
        row_stats(x + r * D, D, eps, &mu, &rstd);
        for (long d = 0; d < D; ++d) {
            const double xhat = (x[r * D + d] - mu) * rstd;
            y[r * D + d] = gamma[d] * xhat + beta[d];
        }
    }
    return 0;
}

/*
 * Backward pass of LayerNorm for ONE example (a batch of one): x[T,D], dy[T,D].
 *   g_gamma[k] = sum_t dy[t,k] * xhat[t,k]        (Appendix B, step 1, for this b)
 *   g_beta[k]  = sum_t dy[t,k]                    (step 5)
 *   dx[t,:]    = rstd * (dyh - mean_d(dyh) - xhat * mean_d(dyh * xhat)),  dyh = dy * gamma
 * dx may be NULL (then it is not produced).
 */
int lnpegn_oracle_ln_bwd_example(const double *x, const double *dy, const double *gamma, long T,
                                 long D, double eps, double *dx, double *g_gamma, double *g_beta)
{
    if (!x || !dy || !gamma || !g_gamma || !g_beta || T <= 0 || D <= 0 || eps < 0.0) return -1;
    for (long k = 0; k < D; ++k) {
        g_gamma[k] = 0.0;
        g_beta[k] = 0.0;
    }
    for (long t = 0; t < T; ++t) {
        const double *xr = x + t * D;
        const double *gr = dy + t * D;
        double mu, rstd;
        row_stats(xr, D, eps, &mu, &rstd);
        double sum_dyh = 0.0, sum_dyh_xhat = 0.0;
        for (long k = 0; k < D; ++k) {
            const double xhat = (xr[k] - mu) * rstd;
            const double dyh = gr[k] * gamma[k];
            sum_dyh += dyh;
            sum_dyh_xhat += dyh * xhat;
            g_gamma[k] += gr[k] * xhat;
            g_beta[k] += gr[k];
        }
        if (dx) {
            const double c1 = sum_dyh_xhat / (double)D;
            const double c2 = sum_dyh / (double)D;
            for (long k = 0; k < D; ++k) {
                const double xhat = (xr[k] - mu) * rstd;
                const double dyh = gr[k] * gamma[k];
                dx[t * D + k] = rstd * (dyh - c2 - xhat * c1);
            }
        }
    }
    return 0;
}

/*
 * Whole batch, by brute force: one separate backward per example, then
 * squared norms (steps 2, 6), sums over examples (steps 3, 7), and the squared
 * norms of the summed gradients.
 *
 *   x, dy        [B,T,D]
 *   gamma        [D]
 *   dx           [B,T,D] or NULL
 *   pe_gamma     [B,D] or NULL   per-example gamma gradients  gamma'_b
 *   pe_beta      [B,D] or NULL   per-example beta gradients   beta'_b
 *   dgamma,dbeta [D]
 *   s_gamma,s_beta [B]           raw squared norms, no B^2 factor
 *   big_sq       [2]             ||dgamma||^2, ||dbeta||^2
 *   nthreads     OpenMP threads over examples (<=0: library default)
 */
int lnpegn_oracle_ln_bwd_pegn(const double *x, const double *dy, const double *gamma, long B, long T,
                              long D, double eps, double *dx, double *pe_gamma, double *pe_beta,
                              double *dgamma, double *dbeta, double *s_gamma, double *s_beta,
                              double *big_sq, int nthreads)
{
    if (!x || !dy || !gamma || !dgamma || !dbeta || !s_gamma || !s_beta || !big_sq) return -1;
    if (B <= 0 || T <= 0 || D <= 0 || eps < 0.0) return -1;

    double *gg = pe_gamma ? pe_gamma : (double *)malloc(sizeof(double) * (size_t)B * (size_t)D);
    double *gb = pe_beta ? pe_beta : (double *)malloc(sizeof(double) * (size_t)B * (size_t)D);
    if (!gg || !gb) {
        if (!pe_gamma) free(gg);
        if (!pe_beta) free(gb);
        return -2;
    }
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (long b = 0; b < B; ++b) {
        const size_t off = (size_t)b * (size_t)T * (size_t)D;
        int rc = lnpegn_oracle_ln_bwd_example(x + off, dy + off, gamma, T, D, eps,
                                              dx ? dx + off : NULL, gg + b * D, gb + b * D);
        if (rc) bad |= 1;
        double sg = 0.0, sb = 0.0;
        for (long k = 0; k < D; ++k) {
            sg += gg[b * D + k] * gg[b * D + k];
            sb += gb[b * D + k] * gb[b * D + k];
        }
        s_gamma[b] = sg;
        s_beta[b] = sb;
    }

    double ng = 0.0, nb = 0.0;
    for (long k = 0; k < D; ++k) {
        double a = 0.0, c = 0.0;
        for (long b = 0; b < B; ++b) {
            a += gg[b * D + k];
            c += gb[b * D + k];
        }
        dgamma[k] = a;
        dbeta[k] = c;
        ng += a * a;
        nb += c * c;
    }
    big_sq[0] = ng;
    big_sq[1] = nb;

    if (!pe_gamma) free(gg);
    if (!pe_beta) free(gb);
    return bad ? -3 : 0;
}

/*
 * RMSNorm variant (Appendix B: "practically identical", the gradient is with respect to the
 * affine parameter):  rstd = 1/sqrt(mean_d x^2 + eps),  xhat = x*rstd,  y = gamma*xhat.
 */
static double rms_rstd(const double *x, long D, double eps)
{
    double ss = 0.0;
    for (long d = 0; d < D; ++d) ss += x[d] * x[d];
    return 1.0 / sqrt(ss / (double)D + eps);
}

int lnpegn_oracle_rms_fwd(const double *x, const double *gamma, long N, long D, double eps, double *y,
                          double *rstd)
{
    if (!x || !gamma || !y || N <= 0 || D <= 0 || eps < 0.0) return -1;
    for (long r = 0; r < N; ++r) {
        const double rs = rms_rstd(x + r * D, D, eps);
        if (rstd) rstd[r] = rs;
        for (long d = 0; d < D; ++d) y[r * D + d] = gamma[d] * (x[r * D + d] * rs);
    }
    return 0;
}

/* Backward of ONE example: g_gamma[k] = sum_t dy*xhat (step 1 of the LayerNorm algorithm with the
 * RMS-normalised activation), dx[t,:] = rstd*(dyh - xhat*mean_d(dyh*xhat)). */
int lnpegn_oracle_rms_bwd_example(const double *x, const double *dy, const double *gamma, long T,
                                  long D, double eps, double *dx, double *g_gamma)
{
    if (!x || !dy || !gamma || !g_gamma || T <= 0 || D <= 0 || eps < 0.0) return -1;
    for (long k = 0; k < D; ++k) g_gamma[k] = 0.0;
    for (long t = 0; t < T; ++t) {
        const double *xr = x + t * D;
        const double *gr = dy + t * D;
        const double rs = rms_rstd(xr, D, eps);
        double sum_dyh_xhat = 0.0;
        for (long k = 0; k < D; ++k) {
            const double xhat = xr[k] * rs;
            sum_dyh_xhat += gr[k] * gamma[k] * xhat;
            g_gamma[k] += gr[k] * xhat;
        }
        if (dx) {
            const double c1 = sum_dyh_xhat / (double)D;
            for (long k = 0; k < D; ++k) {
                const double xhat = xr[k] * rs;
                dx[t * D + k] = rs * (gr[k] * gamma[k] - xhat * c1);
            }
        }
    }
    return 0;
}

/* Whole batch by brute force, as lnpegn_oracle_ln_bwd_pegn; big_sq is one value, ||dgamma||^2. */
int lnpegn_oracle_rms_bwd_pegn(const double *x, const double *dy, const double *gamma, long B, long T,
                               long D, double eps, double *dx, double *pe_gamma, double *dgamma,
                               double *s_gamma, double *big_sq, int nthreads)
{
    if (!x || !dy || !gamma || !dgamma || !s_gamma || !big_sq) return -1;
    if (B <= 0 || T <= 0 || D <= 0 || eps < 0.0) return -1;
    double *gg = pe_gamma ? pe_gamma : (double *)malloc(sizeof(double) * (size_t)B * (size_t)D);
    if (!gg) return -2;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (long b = 0; b < B; ++b) {
        const size_t off = (size_t)b * (size_t)T * (size_t)D;
        if (lnpegn_oracle_rms_bwd_example(x + off, dy + off, gamma, T, D, eps, dx ? dx + off : NULL,
                                          gg + b * D))
            bad |= 1;
        double sg = 0.0;
        for (long k = 0; k < D; ++k) sg += gg[b * D + k] * gg[b * D + k];
        s_gamma[b] = sg;
    }
    double ng = 0.0;
    for (long k = 0; k < D; ++k) {
        double a = 0.0;
        for (long b = 0; b < B; ++b) a += gg[b * D + k];
        dgamma[k] = a;
        ng += a * a;
    }
    big_sq[0] = ng;
    if (!pe_gamma) free(gg);
    return bad ? -3 : 0;
}

/* Number of OpenMP threads a parallel region would use (1 without OpenMP). */
int lnpegn_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Section 2.1, Eq. 4 and Eq. 5, for arbitrary batch sizes:
 *   G2 = (B_big*|G_big|^2 - B_small*|G_small|^2) / (B_big - B_small)
 *   S  = (|G_small|^2 - |G_big|^2) / (1/B_small - 1/B_big)
 * and Eq. 3, B_simple = S / G2.  No clamping: a negative or zero G2 gives the
 * IEEE-754 result.  out = {G2, S, B_simple}.
 */
int lnpegn_oracle_gns_from_norms(double g_big_sq, double g_small_sq, double b_big, double b_small,
                                 double *out)
{
    if (!out || b_big <= 0.0 || b_small <= 0.0 || b_big == b_small) return -1;
    const double G2 = (b_big * g_big_sq - b_small * g_small_sq) / (b_big - b_small);
    const double S = (g_small_sq - g_big_sq) / (1.0 / b_small - 1.0 / b_big);
    out[0] = G2;
    out[1] = S;
    out[2] = S / G2;
    return 0;
}

/*
 * From raw per-example squared norms to the estimate.
 *   pe_sq   [n_groups,B]  raw s[b] of every parameter group (each layer's gamma and beta
 *                         are separate groups); the squared norm of a concatenation of
 *                         groups is the sum of the groups' squared norms
 *   big_sq  [n_groups]    squared norms of the summed gradients
 *   pe_scale              factor c multiplying every per-example gradient; c = B for a
 *                         mean-reduced loss (Appendix B steps 4 and 8: mean over b, times B^2)
 * Per-example method: B_small = 1, B_big = B.
 *   out = {|G_small|^2, |G_big|^2, G2, S, B_simple}
 */
int lnpegn_oracle_gns_estimate(const double *pe_sq, const double *big_sq, long n_groups, long B,
                               double pe_scale, double *out)
{
    if (!pe_sq || !big_sq || !out || n_groups <= 0 || B <= 1) return -1;
    double small = 0.0, big = 0.0;
    for (long g = 0; g < n_groups; ++g) {
        double mean_s = 0.0;
        for (long b = 0; b < B; ++b) mean_s += pe_sq[g * B + b];
        mean_s /= (double)B;                       /* reduce by mean ...          */
        small += mean_s * pe_scale * pe_scale;     /* ... then apply correction   */
        big += big_sq[g];
    }
    out[0] = small;
    out[1] = big;
    return lnpegn_oracle_gns_from_norms(big, small, (double)B, 1.0, out + 2);
}
