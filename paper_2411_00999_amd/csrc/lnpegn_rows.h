// Row-streaming kernels: the single pass over x and dy that writes dx and accumulates the
// column sums  A_gamma[k] = sum_t dy*xhat,  A_beta[k] = sum_t dy  over one chunk of rows.
//
// Work partition.  The N = B*T rows are cut into `n_slots` chunks.  For the per-example path
// chunks never straddle an example: example b owns chunks [b*C, (b+1)*C), so the per-example
// sums of Appendix B steps 1 and 5 are sums of whole chunks.  The plain backward uses the same
// kernels with the whole tensor declared as one "example" (Bp = 1, Tp = N).
//
// Lane mapping.  A lane owns the same columns for every row it touches, so the sums over t
// live in registers and never move between lanes; only the per-row scalars (mean, variance,
// mean_d(dyh), mean_d(dyh*xhat)) cross lanes, on the DPP network.
//   wave mode  (kMulti = false): one wave owns a row; the R waves of a workgroup take rows
//                                r0+w, r0+w+R, ... and merge their column sums through LDS in
//                                wave order at the end of the chunk.
//   multi mode (kMulti = true) : all S waves of a workgroup share one row (wide D); each wave
//                                owns different columns, per-row scalars cross waves through LDS.
#pragma once
#include "lnpegn_device.h"

namespace lnpegn {

struct RowArgs {
    const void *x;
    const void *dy;
    const void *gamma;
    const float *mean;  // may be null (recompute)
    const float *rstd;
    void *dx;
    float *part;        // [n_slots][2][D] fp32 column sums per chunk
    int64_t Tp;         // rows per partition example
    int C;              // chunks per partition example
    int D;
    int nvec;           // D / elements-per-vector
    int gamma_is_f32;
    float eps;
    float inv_D;
};

template <typename T, int kVpt, bool kSaved, bool kMulti, int kMaxThreads>
__global__ __launch_bounds__(kMaxThreads) void ln_bwd_rows_kernel(RowArgs a)
{
    using V = Vec<T>;
    using Raw = typename V::Raw;
    constexpr int E = V::kElems;
    extern __shared__ __align__(16) float lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int64_t chunk = blockIdx.x;
    const int64_t b = chunk / a.C, j = chunk - b * a.C;
    const int64_t r0 = b * a.Tp + (j * a.Tp) / a.C;
    const int64_t r1 = b * a.Tp + ((j + 1) * a.Tp) / a.C;

    // vector index of slot k: multi mode interleaves the waves inside each 64*S-vector span
    int vidx[kVpt];
    bool ok[kVpt];
    int n_valid = 0;  // valid elements of this wave (uniform)
#pragma unroll
    for (int k = 0; k < kVpt; ++k) {
        const int first = kMulti ? (k * nwaves + wave) * kWave : k * kWave;
        vidx[k] = first + lane;
        ok[k] = vidx[k] < a.nvec;
        const int left = a.nvec - first;
        n_valid += (left < 0 ? 0 : (left > kWave ? kWave : left)) * E;
    }
    const float inv_nw = 1.0f / (float)n_valid;

    float gm[kVpt][E];
#pragma unroll
    for (int k = 0; k < kVpt; ++k)
#pragma unroll
        for (int e = 0; e < E; ++e)
            gm[k][e] = ok[k] ? load_gamma(a.gamma, a.gamma_is_f32, (int64_t)vidx[k] * E + e) : 0.f;

    float acc_g[kVpt][E], acc_b[kVpt][E];
#pragma unroll
    for (int k = 0; k < kVpt; ++k)
#pragma unroll
        for (int e = 0; e < E; ++e) acc_g[k][e] = acc_b[k][e] = 0.f;

    const Raw *xv = static_cast<const Raw *>(a.x);
    const Raw *dyv = static_cast<const Raw *>(a.dy);
    Raw *dxv = static_cast<Raw *>(a.dx);

    auto load_row = [&](int64_t r, Raw (&xr)[kVpt], Raw (&dr)[kVpt]) {
        const Raw *xrow = xv + r * a.nvec;
        const Raw *drow = dyv + r * a.nvec;
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            xr[k] = V::zero();
            dr[k] = V::zero();
            if (ok[k]) {
                xr[k] = xrow[vidx[k]];
                dr[k] = drow[vidx[k]];
            }
        }
    };

    // Exchange buffer of multi mode: [parity][5][16] floats; one barrier per exchange, the
    // parity flip between rows keeps a fast wave from overwriting values still being read.
    int parity = 0;

    auto process = [&](int64_t r, const Raw (&xr)[kVpt], const Raw (&dr)[kVpt]) {
        float xf[kVpt][E], df[kVpt][E];
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            V::unpack(xr[k], xf[k]);
            V::unpack(dr[k], df[k]);
        }
        float *xchg = lds + parity * 5 * 16;
        float mean, rstd, s_dyh = 0.f;
#pragma unroll
        for (int k = 0; k < kVpt; ++k)
#pragma unroll
            for (int e = 0; e < E; ++e) s_dyh += df[k][e] * gm[k][e];

        if constexpr (kSaved) {
            mean = a.mean[r];
            rstd = a.rstd[r];
        } else {
            // two-pass statistics inside the wave
            float s_x = 0.f;
#pragma unroll
            for (int k = 0; k < kVpt; ++k)
#pragma unroll
                for (int e = 0; e < E; ++e) s_x += xf[k][e];
            wave_sum2(s_x, s_dyh);
            const float m_w = s_x * (kMulti ? inv_nw : a.inv_D);
            float m2 = 0.f;
#pragma unroll
            for (int k = 0; k < kVpt; ++k)
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float c = ok[k] ? xf[k][e] - m_w : 0.f;
                    m2 += c * c;
                }
            m2 = wave_sum(m2);
            if constexpr (kMulti) {
                // merge the waves' (sum, M2) pairs: M2 = sum_w M2_w + n_w*(mean_w - mean)^2
                if (lane == 0) {
                    xchg[wave] = s_x;
                    xchg[16 + wave] = m2;
                    xchg[32 + wave] = s_dyh;
                }
                __syncthreads();
                float tot = 0.f, tdy = 0.f;
                for (int w = 0; w < nwaves; ++w) {
                    tot += xchg[w];
                    tdy += xchg[32 + w];
                }
                mean = tot * a.inv_D;
                s_dyh = tdy;
                float M2 = 0.f;
                for (int w = 0; w < nwaves; ++w) {
                    int nw = 0;
#pragma unroll
                    for (int k = 0; k < kVpt; ++k) {
                        const int left = a.nvec - (k * nwaves + w) * kWave;
                        nw += (left < 0 ? 0 : (left > kWave ? kWave : left)) * E;
                    }
                    const float d = xchg[w] / (float)nw - mean;
                    M2 += xchg[16 + w] + (float)nw * d * d;
                }
                rstd = rsqrtf(M2 * a.inv_D + a.eps);
            } else {
                mean = m_w;
                rstd = rsqrtf(m2 * a.inv_D + a.eps);
            }
        }
        // xhat; padded lanes stay at zero so they do not enter any sum
        float s_dx = 0.f;
#pragma unroll
        for (int k = 0; k < kVpt; ++k)
#pragma unroll
            for (int e = 0; e < E; ++e) {
                xf[k][e] = ok[k] ? (xf[k][e] - mean) * rstd : 0.f;
                s_dx += df[k][e] * gm[k][e] * xf[k][e];
            }
        if constexpr (kSaved) {
            wave_sum2(s_dx, s_dyh);
        } else {
            s_dx = wave_sum(s_dx);
        }
        if constexpr (kMulti) {
            if (lane == 0) {
                xchg[48 + wave] = s_dx;
                if constexpr (kSaved) xchg[64 + wave] = s_dyh;
            }
            __syncthreads();
            float t0 = 0.f, t1 = 0.f;
            for (int w = 0; w < nwaves; ++w) {
                t0 += xchg[48 + w];
                if constexpr (kSaved) t1 += xchg[64 + w];
            }
            s_dx = t0;
            if constexpr (kSaved) s_dyh = t1;
        }
        // dx = rstd*(dyh - c2 - xhat*c1)
        const float k1 = -rstd * s_dx * a.inv_D, k2 = -rstd * s_dyh * a.inv_D;
        Raw *orow = dxv + r * a.nvec;
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            float o[E];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                o[e] = (df[k][e] * gm[k][e]) * rstd + (xf[k][e] * k1 + k2);
                acc_g[k][e] += df[k][e] * xf[k][e];
                acc_b[k][e] += df[k][e];
            }
            if (ok[k]) orow[vidx[k]] = V::pack(o);
        }
        parity ^= 1;
    };

    // two register buffers, loads for the next row are in flight while the current one is reduced
    const int64_t step = kMulti ? 1 : nwaves;
    int64_t r = r0 + (kMulti ? 0 : wave);
    Raw xa[kVpt], da[kVpt], xb[kVpt], db[kVpt];
    if (r < r1) load_row(r, xa, da);
    while (r < r1) {
        if (r + step < r1) load_row(r + step, xb, db);
        process(r, xa, da);
        r += step;
        if (r >= r1) break;
        if (r + step < r1) load_row(r + step, xa, da);
        process(r, xb, db);
        r += step;
    }

    // ---- hand the chunk's column sums to the workspace ----
    float *out_g = a.part + chunk * 2 * (int64_t)a.D;
    float *out_b = out_g + a.D;
    if constexpr (kMulti) {
        // each wave owns its columns: straight from registers
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            if (ok[k]) {
#pragma unroll
                for (int q = 0; q < E / 4; ++q) {
                    const int64_t col = (int64_t)vidx[k] * E + q * 4;
                    *reinterpret_cast<float4 *>(out_g + col) = make_float4(
                        acc_g[k][q * 4], acc_g[k][q * 4 + 1], acc_g[k][q * 4 + 2], acc_g[k][q * 4 + 3]);
                    *reinterpret_cast<float4 *>(out_b + col) = make_float4(
                        acc_b[k][q * 4], acc_b[k][q * 4 + 1], acc_b[k][q * 4 + 2], acc_b[k][q * 4 + 3]);
                }
            }
        }
    } else {
        // merge the waves' sums through LDS, adding in wave order (reproducible)
        constexpr int NF = 2 * kVpt * E;  // floats per lane
        float *mine = lds + (int64_t)wave * NF * kWave;
#pragma unroll
        for (int k = 0; k < kVpt; ++k)
#pragma unroll
            for (int e = 0; e < E; ++e) {
                mine[((0 * kVpt + k) * E + e) * kWave + lane] = acc_g[k][e];
                mine[((1 * kVpt + k) * E + e) * kWave + lane] = acc_b[k][e];
            }
        __syncthreads();
        constexpr int NQ = NF / 4;  // groups of four consecutive columns per lane
        for (int q = wave; q < NQ; q += nwaves) {
            const int f0 = q * 4;
            const int arr = f0 / (kVpt * E);
            const int k = (f0 / E) % kVpt;
            const int e0 = f0 % E;
            float s[4] = {0.f, 0.f, 0.f, 0.f};
            for (int w = 0; w < nwaves; ++w) {
                const float *src = lds + ((int64_t)w * NF + f0) * kWave + lane;
#pragma unroll
                for (int i = 0; i < 4; ++i) s[i] += src[i * kWave];
            }
            const int v = k * kWave + lane;
            if (v < a.nvec) {
                float *dst = (arr == 0 ? out_g : out_b) + (int64_t)v * E + e0;
                *reinterpret_cast<float4 *>(dst) = make_float4(s[0], s[1], s[2], s[3]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Generic row kernel: any D >= 1, any alignment.  One workgroup of 256 threads per chunk, one
// row at a time, scalar element accesses; thread i owns columns i, i+256, ... and keeps their
// running sums in the chunk's workspace slot.  Correct, not fast.
// ---------------------------------------------------------------------------------------
template <typename T, bool kSaved>
__global__ void ln_bwd_rows_generic_kernel(RowArgs a)
{
    __shared__ float slots[8];
    const int64_t chunk = blockIdx.x;
    const int64_t b = chunk / a.C, j = chunk - b * a.C;
    const int64_t r0 = b * a.Tp + (j * a.Tp) / a.C;
    const int64_t r1 = b * a.Tp + ((j + 1) * a.Tp) / a.C;
    float *out_g = a.part + chunk * 2 * (int64_t)a.D;
    float *out_b = out_g + a.D;
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int k = tid; k < a.D; k += nt) {
        out_g[k] = 0.f;
        out_b[k] = 0.f;
    }
    for (int64_t r = r0; r < r1; ++r) {
        const int64_t base = r * (int64_t)a.D;
        float mean, rstd;
        float s_dyh = 0.f;
        for (int k = tid; k < a.D; k += nt)
            s_dyh += load_elem<T>(a.dy, base + k) * load_gamma(a.gamma, a.gamma_is_f32, k);
        s_dyh = block_sum(s_dyh, slots);
        if constexpr (kSaved) {
            mean = a.mean[r];
            rstd = a.rstd[r];
        } else {
            float s_x = 0.f;
            for (int k = tid; k < a.D; k += nt) s_x += load_elem<T>(a.x, base + k);
            mean = block_sum(s_x, slots) * a.inv_D;
            float ss = 0.f;
            for (int k = tid; k < a.D; k += nt) {
                const float c = load_elem<T>(a.x, base + k) - mean;
                ss += c * c;
            }
            rstd = rsqrtf(block_sum(ss, slots) * a.inv_D + a.eps);
        }
        float s_dx = 0.f;
        for (int k = tid; k < a.D; k += nt) {
            const float xhat = (load_elem<T>(a.x, base + k) - mean) * rstd;
            s_dx += load_elem<T>(a.dy, base + k) * load_gamma(a.gamma, a.gamma_is_f32, k) * xhat;
        }
        s_dx = block_sum(s_dx, slots);
        const float c1 = s_dx * a.inv_D, c2 = s_dyh * a.inv_D;
        for (int k = tid; k < a.D; k += nt) {
            const float xhat = (load_elem<T>(a.x, base + k) - mean) * rstd;
            const float dyv = load_elem<T>(a.dy, base + k);
            const float dyh = dyv * load_gamma(a.gamma, a.gamma_is_f32, k);
            store_elem<T>(a.dx, base + k, rstd * (dyh - c2 - xhat * c1));
            out_g[k] += dyv * xhat;
            out_b[k] += dyv;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Row statistics (forward): mean and rstd of every row, two-pass variance in fp32.
// Wave mode only needs a grid-stride loop over rows; wide rows use the whole workgroup.
// ---------------------------------------------------------------------------------------
struct StatsArgs {
    const void *x;
    float *mean;
    float *rstd;
    int64_t N;
    int D;
    int nvec;
    float eps;
    float inv_D;
};

template <typename T, int kVpt, bool kMulti>
__global__ void ln_stats_kernel(StatsArgs a)
{
    using V = Vec<T>;
    using Raw = typename V::Raw;
    constexpr int E = V::kElems;
    __shared__ float slots[2][16];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    int vidx[kVpt];
    bool ok[kVpt];
#pragma unroll
    for (int k = 0; k < kVpt; ++k) {
        vidx[k] = kMulti ? (k * nwaves + wave) * kWave + lane : k * kWave + lane;
        ok[k] = vidx[k] < a.nvec;
    }
    const Raw *xv = static_cast<const Raw *>(a.x);
    const int64_t first = kMulti ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * nwaves + wave;
    const int64_t stride = kMulti ? (int64_t)gridDim.x : (int64_t)gridDim.x * nwaves;
    for (int64_t r = first; r < a.N; r += stride) {
        float xf[kVpt][E];
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            Raw raw = V::zero();
            if (ok[k]) raw = xv[r * a.nvec + vidx[k]];
            V::unpack(raw, xf[k]);
#pragma unroll
            for (int e = 0; e < E; ++e) s += xf[k][e];
        }
        s = wave_sum(s);
        if constexpr (kMulti) {
            if (lane == 0) slots[0][wave] = s;
            __syncthreads();
            s = 0.f;
            for (int w = 0; w < nwaves; ++w) s += slots[0][w];
        }
        const float mean = s * a.inv_D;
        float ss = 0.f;
#pragma unroll
        for (int k = 0; k < kVpt; ++k)
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float c = ok[k] ? xf[k][e] - mean : 0.f;
                ss += c * c;
            }
        ss = wave_sum(ss);
        if constexpr (kMulti) {
            if (lane == 0) slots[1][wave] = ss;
            __syncthreads();
            ss = 0.f;
            for (int w = 0; w < nwaves; ++w) ss += slots[1][w];
            __syncthreads();  // slots are rewritten by the next row
        }
        if (threadIdx.x == (kMulti ? 0 : wave * kWave) ) {
            a.mean[r] = mean;
            a.rstd[r] = rsqrtf(ss * a.inv_D + a.eps);
        }
    }
}

template <typename T>
__global__ void ln_stats_generic_kernel(StatsArgs a)
{
    __shared__ float slots[8];
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int64_t r = blockIdx.x; r < a.N; r += gridDim.x) {
        const int64_t base = r * (int64_t)a.D;
        float s = 0.f;
        for (int k = tid; k < a.D; k += nt) s += load_elem<T>(a.x, base + k);
        const float mean = block_sum(s, slots) * a.inv_D;
        float ss = 0.f;
        for (int k = tid; k < a.D; k += nt) {
            const float c = load_elem<T>(a.x, base + k) - mean;
            ss += c * c;
        }
        ss = block_sum(ss, slots);
        if (tid == 0) {
            a.mean[r] = mean;
            a.rstd[r] = rsqrtf(ss * a.inv_D + a.eps);
        }
    }
}

}  // namespace lnpegn
