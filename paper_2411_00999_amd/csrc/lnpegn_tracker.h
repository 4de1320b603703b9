// What is done with the per-step estimates of Eq. 4 (G2) and Eq. 5 (S) after they are computed:
// the online exponential moving average of both before the ratio (Section 4.2), and the offline
// mean with the delete-one jackknife of the ratio of means (Figure 2 caption, Appendix A).
// A record is the five floats gns_estimate writes: {g_small_sq, g_big_sq, G2, S, B_simple}.
#pragma once
#include "lnpegn_device.h"

namespace lnpegn {

constexpr int kRecord = 5, kRecG2 = 2, kRecS = 3;

// state rows {m_G2, m_S, w}: m <- alpha*m + (1-alpha)*v from zero; w is the same recurrence on 1,
// i.e. the weight seen so far (1 - alpha^t), by which the averages are divided when read.
__global__ __launch_bounds__(256) void gns_ema_update_kernel(double *state, const float *records, int n,
                                                             double alpha, float *smoothed)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const double g2 = (double)records[(int64_t)i * kRecord + kRecG2];
    const double s = (double)records[(int64_t)i * kRecord + kRecS];
    const double keep = alpha, take = 1.0 - alpha;
    const double mg = keep * state[i * 3 + 0] + take * g2;
    const double ms = keep * state[i * 3 + 1] + take * s;
    const double w = keep * state[i * 3 + 2] + take;
    state[i * 3 + 0] = mg;
    state[i * 3 + 1] = ms;
    state[i * 3 + 2] = w;
    if (smoothed) {
        smoothed[i * 3 + 0] = (float)(mg / w);
        smoothed[i * 3 + 1] = (float)(ms / w);
        smoothed[i * 3 + 2] = (float)(ms / mg);   // Eq. 3 on the smoothed pair; w cancels
    }
}

// One workgroup over a history of n records: R = mean(S)/mean(G2); R_(i) with step i left out is
// (sum S - S_i)/(sum G2 - G2_i); stderr^2 = (n-1)/n * sum_i (R_(i) - mean R_(.))^2.
// out = {mean_G2, mean_S, R, stderr, n*R - (n-1)*mean R_(.)}.  Every sum in fp64, fixed order.
__global__ __launch_bounds__(256) void gns_offline_kernel(const float *records, int64_t n, float *out)
{
    __shared__ double slots[3][4];
    double sg = 0.0, ss = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) {
        sg += (double)records[i * kRecord + kRecG2];
        ss += (double)records[i * kRecord + kRecS];
    }
    sg = block_sum_f64(sg, slots[0]);
    ss = block_sum_f64(ss, slots[1]);
    double sl = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x)
        sl += (ss - (double)records[i * kRecord + kRecS]) / (sg - (double)records[i * kRecord + kRecG2]);
    const double rbar = block_sum_f64(sl, slots[2]) / (double)n;
    double sq = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) {
        const double d =
            (ss - (double)records[i * kRecord + kRecS]) / (sg - (double)records[i * kRecord + kRecG2]) - rbar;
        sq += d * d;
    }
    sq = block_sum_f64(sq, slots[0]);
    if (threadIdx.x == 0) {
        const double nd = (double)n, R = ss / sg;
        out[0] = (float)(sg / nd);
        out[1] = (float)(ss / nd);
        out[2] = (float)R;
        out[3] = (float)sqrt((nd - 1.0) / nd * sq);
        out[4] = (float)(nd * R - (nd - 1.0) * rbar);
    }
}

}  // namespace lnpegn
