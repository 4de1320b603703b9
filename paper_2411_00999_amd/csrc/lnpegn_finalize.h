// Second level of the two-level deterministic reduction: sums of the per-chunk column sums,
// the per-example squared norms (Appendix B steps 2 and 6), the batch gradients (steps 3
// and 7) and the gradient-noise-scale estimator (Section 2.1, Eq. 3-5).  Every sum runs in a
// fixed order, in fp64, so results do not depend on scheduling.
#pragma once
#include "lnpegn_device.h"

namespace lnpegn {

constexpr int kTile = 256;  // columns per workgroup in the column-sum kernels

struct ColSumArgs {
    const float *src;   // [M][2][D]
    float *dst0;        // group g, array 0 -> dst0 + g*dst_stride ; array 1 -> dst1 + g*dst_stride
    float *dst1;
    double *part_sq;    // [n_groups][ntile][2] sums of squares of the outputs per tile, or null
    int64_t dst_stride;
    int M;              // number of source vectors
    int gs;             // vectors per group (last group may be short)
    int D;
};

// grid (n_groups, ntile), 256 threads: thread = one column, sequential sum over the group.
__global__ __launch_bounds__(kTile) void col_sum_kernel(ColSumArgs a)
{
    __shared__ double slots[2][4];
    const int k = blockIdx.y * kTile + threadIdx.x;
    const int g = blockIdx.x;
    const int m0 = g * a.gs;
    const int m1 = min(m0 + a.gs, a.M);
    double s0 = 0.0, s1 = 0.0;
    if (k < a.D) {
        const float *p = a.src + (int64_t)m0 * 2 * a.D + k;
        int m = m0;
        for (; m + 4 <= m1; m += 4) {   // four loads in flight, added in order
            const float u0 = p[0], v0 = p[a.D];
            const float u1 = p[2 * (int64_t)a.D], v1 = p[3 * (int64_t)a.D];
            const float u2 = p[4 * (int64_t)a.D], v2 = p[5 * (int64_t)a.D];
            const float u3 = p[6 * (int64_t)a.D], v3 = p[7 * (int64_t)a.D];
            s0 = (((s0 + u0) + u1) + u2) + u3;
            s1 = (((s1 + v0) + v1) + v2) + v3;
            p += 8 * (int64_t)a.D;
        }
        for (; m < m1; ++m) {
            s0 += p[0];
            s1 += p[a.D];
            p += 2 * (int64_t)a.D;
        }
        a.dst0[(int64_t)g * a.dst_stride + k] = (float)s0;
        a.dst1[(int64_t)g * a.dst_stride + k] = (float)s1;
    }
    if (a.part_sq) {
        // squares of the values as stored (fp32), summed in fp64
        const double f0 = (double)(float)s0, f1 = (double)(float)s1;
        const double q0 = block_sum_f64(f0 * f0, slots[0]);
        const double q1 = block_sum_f64(f1 * f1, slots[1]);
        if (threadIdx.x == 0) {
            double *o = a.part_sq + ((int64_t)g * gridDim.y + blockIdx.y) * 2;
            o[0] = q0;
            o[1] = q1;
        }
    }
}

struct ScalarsArgs {
    const double *part_s;    // [B][ntile][2] or null
    const double *part_big;  // [ntile][2] or null
    float *pe_gamma_sq;      // [B]
    float *pe_beta_sq;       // [B]
    float *big_sq;           // [2] or null
    int B;
    int ntile;
};

// tiny: per-example tile partials -> s_gamma[b], s_beta[b]; tile partials -> ||dgamma||^2, ||dbeta||^2
__global__ __launch_bounds__(256) void scalars_kernel(ScalarsArgs a)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (a.part_s && i < a.B) {
        double g = 0.0, b = 0.0;
        for (int t = 0; t < a.ntile; ++t) {
            g += a.part_s[((int64_t)i * a.ntile + t) * 2];
            b += a.part_s[((int64_t)i * a.ntile + t) * 2 + 1];
        }
        a.pe_gamma_sq[i] = (float)g;
        a.pe_beta_sq[i] = (float)b;
    }
    if (a.big_sq && a.part_big && i < 2) {
        double s = 0.0;
        for (int t = 0; t < a.ntile; ++t) s += a.part_big[t * 2 + i];
        a.big_sq[i] = (float)s;
    }
}

// Section 2.1 Eq. 3-5 with B_small = 1, B_big = B; one workgroup.
__global__ __launch_bounds__(256) void gns_estimate_kernel(const float *pe_sq, const float *big_sq,
                                                           int n_groups, int B, float pe_scale,
                                                           float *out)
{
    __shared__ double slots[2][4];
    const int64_t n = (int64_t)n_groups * B;
    double s = 0.0, g = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) s += (double)pe_sq[i];
    for (int i = threadIdx.x; i < n_groups; i += blockDim.x) g += (double)big_sq[i];
    s = block_sum_f64(s, slots[0]);
    g = block_sum_f64(g, slots[1]);
    if (threadIdx.x == 0) {
        const double Bd = (double)B, c = (double)pe_scale;
        const double small = c * c * (s / Bd);  // mean over examples, then the correction
        const double big = g;
        const double G2 = (Bd * big - small) / (Bd - 1.0);   // Eq. 4 with B_small = 1
        const double S = (small - big) / (1.0 - 1.0 / Bd);   // Eq. 5 with B_small = 1
        out[0] = (float)small;
        out[1] = (float)big;
        out[2] = (float)G2;
        out[3] = (float)S;
        out[4] = (float)(S / G2);                            // Eq. 3
    }
}

}  // namespace lnpegn
