// Row-streaming kernels: the single pass over x and dy that writes dx and accumulates the
// column sums  A_gamma[k] = sum_t dy*xhat,  A_beta[k] = sum_t dy  over one chunk of rows.
//
// Work partition.  The N = B*T rows are cut into `n_slots` chunks.  For the per-example path
// chunks never straddle an example: example b owns chunks [b*C, (b+1)*C) and chunk j of it
// takes rows j, j+C, j+2C, ... of that example, so the per-example sums of Appendix B steps 1
// and 5 are sums of whole chunks and the workgroups of an example sweep one moving window of
// memory together.  The plain backward uses the same kernels with the whole tensor declared
// as one "example" (Bp = 1, Tp = N).
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
    int64_t stagger;    // example b starts its sweep at row (b*stagger) mod Tp of itself
    int C;              // chunks per partition example
    int D;
    int nvec;           // D / elements-per-vector
    int gamma_is_f32;
    float eps;
    float inv_D;
};

// gamma for one 16-byte row vector, as fp32 (gamma may be stored in either type)
template <typename T>
__device__ __forceinline__ void load_gamma_vec(const void *gamma, int gamma_is_f32, int v,
                                               float (&g)[Vec<T>::kElems])
{
    constexpr int E = Vec<T>::kElems;
    if (gamma_is_f32) {
        const float4 *p = static_cast<const float4 *>(gamma) + (int64_t)v * (E / 4);
#pragma unroll
        for (int q = 0; q < E / 4; ++q) {
            const float4 t = p[q];
            g[4 * q] = t.x; g[4 * q + 1] = t.y; g[4 * q + 2] = t.z; g[4 * q + 3] = t.w;
        }
    } else if constexpr (E == 8) {
        Vec<bf16_t>::unpack(static_cast<const uint4 *>(gamma)[v], g);
    } else {
        const uint2 t = static_cast<const uint2 *>(gamma)[v];
        g[0] = __builtin_bit_cast(float, t.x << 16);
        g[1] = __builtin_bit_cast(float, t.x & 0xffff0000u);
        g[2] = __builtin_bit_cast(float, t.y << 16);
        g[3] = __builtin_bit_cast(float, t.y & 0xffff0000u);
    }
}

// Valid elements owned by wave w (multi mode interleaves the waves inside 64*S-vector spans).
template <int kVpt, int E>
__device__ __forceinline__ int wave_valid_elems(int w, int nwaves, int nvec, bool multi)
{
    int n = 0;
#pragma unroll
    for (int k = 0; k < kVpt; ++k) {
        const int left = nvec - (multi ? (k * nwaves + w) * kWave : k * kWave);
        n += (left < 0 ? 0 : (left > kWave ? kWave : left)) * E;
    }
    return n;
}

// Row statistics with ONE cross-lane/cross-wave exchange per row.  Inside a wave the mean and
// the centred second moment are taken in two passes over registers (exact, no E[x^2]-mu^2);
// the waves of a row then merge (sum, M2) pairs with the pairwise-merge identity
//   M2 = sum_w M2_w + n_w (mean_w - mean)^2,
// and sum_d dyh*(x-mean) = sum_w [ sum dyh*(x-mean_w) + (mean_w-mean) sum dyh ]
// so the wave mean is only a pivot and the result does not lose digits to a large |mean|.
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
    // chunk j of example b owns rows  b*Tp + j + i*C : the chunks of an example sweep it together.
    // Examples sit a power of two apart in memory; starting each sweep at a different row
    // (wrapping around) keeps the concurrent sweeps on different HBM channels.
    const int64_t row_base = b * a.Tp;
    const int64_t t_end = a.Tp;
    const int64_t t_rot = (b * a.stagger) % a.Tp;

    int vidx[kVpt];
    bool ok[kVpt];
#pragma unroll
    for (int k = 0; k < kVpt; ++k) {
        vidx[k] = (kMulti ? (k * nwaves + wave) * kWave : k * kWave) + lane;
        ok[k] = vidx[k] < a.nvec;
    }
    const float inv_nw = 1.0f / (float)wave_valid_elems<kVpt, E>(wave, nwaves, a.nvec, kMulti);

    const Raw *xv = static_cast<const Raw *>(a.x);
    const Raw *dyv = static_cast<const Raw *>(a.dy);
    Raw *dxv = static_cast<Raw *>(a.dx);

    // loads are unconditional (index clamped to a valid vector); padded lanes are zeroed on unpack
    auto rotated = [&](int64_t tt) {
        const int64_t u = tt + t_rot;
        return row_base + (u >= t_end ? u - t_end : u);
    };
    auto load_row = [&](int64_t tt, Raw (&xr)[kVpt], Raw (&dr)[kVpt]) {
        const int64_t rr = rotated(tt);
        const Raw *xrow = xv + rr * a.nvec;
        const Raw *drow = dyv + rr * a.nvec;
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            const int v = ok[k] ? vidx[k] : 0;
            xr[k] = xrow[v];
            dr[k] = drow[v];
        }
    };

    // first row on its way before anything else is fetched
    const int64_t step = (int64_t)a.C * (kMulti ? 1 : nwaves);
    int64_t t = j + (kMulti ? 0 : (int64_t)wave * a.C);
    Raw xa[kVpt], da[kVpt], xb[kVpt], db[kVpt];
    if (t < t_end) load_row(t, xa, da);

    float gm[kVpt][E];
#pragma unroll
    for (int k = 0; k < kVpt; ++k) {
        load_gamma_vec<T>(a.gamma, a.gamma_is_f32, ok[k] ? vidx[k] : 0, gm[k]);
        if (!ok[k]) {
#pragma unroll
            for (int e = 0; e < E; ++e) gm[k][e] = 0.f;
        }
    }

    float acc_g[kVpt][E], acc_b[kVpt][E];
#pragma unroll
    for (int k = 0; k < kVpt; ++k)
#pragma unroll
        for (int e = 0; e < E; ++e) acc_g[k][e] = acc_b[k][e] = 0.f;

    // Exchange buffer of multi mode: [parity][4][16] floats, then 16 floats of 1/n_w.  One
    // barrier per row; the parity flip keeps a fast wave from overwriting values still being read.
    float *nw_inv = lds + 2 * 4 * 16;
    if constexpr (kMulti) {
        if (lane == 0) nw_inv[wave] = inv_nw;
    }
    int parity = 0;

    auto process = [&](int64_t tt, const Raw (&xr)[kVpt], const Raw (&dr)[kVpt]) {
        const int64_t r = rotated(tt);
        float xf[kVpt][E], df[kVpt][E];
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            V::unpack(xr[k], xf[k]);
            V::unpack(dr[k], df[k]);
            if (!ok[k]) {
#pragma unroll
                for (int e = 0; e < E; ++e) xf[k][e] = df[k][e] = 0.f;
            }
        }
        // pass 1: pivot = the wave's own mean (or the saved row mean)
        float s_x = 0.f, pivot;
        if constexpr (kSaved) {
            pivot = a.mean[r];
        } else {
#pragma unroll
            for (int k = 0; k < kVpt; ++k)
#pragma unroll
                for (int e = 0; e < E; ++e) s_x += xf[k][e];
            s_x = wave_sum(s_x);
            pivot = s_x * (kMulti ? inv_nw : a.inv_D);
        }
        // pass 2: centre about the pivot; M2, sum dyh, sum dyh*xc
        float m2 = 0.f, s_dyh = 0.f, s_dyx = 0.f;
#pragma unroll
        for (int k = 0; k < kVpt; ++k)
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float xc = ok[k] ? xf[k][e] - pivot : 0.f;
                const float dyh = df[k][e] * gm[k][e];
                xf[k][e] = xc;
                s_dyh += dyh;
                s_dyx += dyh * xc;
                if constexpr (!kSaved) m2 += xc * xc;
            }
        if constexpr (kSaved) {
            wave_sum2(s_dyh, s_dyx);
        } else {
            wave_sum3(m2, s_dyh, s_dyx);
        }
        float rstd, shift = 0.f;
        if constexpr (kMulti) {
            float *xchg = lds + parity * 4 * 16;
            if (lane == 0) {
                xchg[wave] = s_dyh;
                xchg[16 + wave] = s_dyx;
                if constexpr (!kSaved) {
                    xchg[32 + wave] = s_x;
                    xchg[48 + wave] = m2;
                }
            }
            __syncthreads();
            if constexpr (kSaved) {
                float t0 = 0.f, t1 = 0.f;
                for (int w = 0; w < nwaves; ++w) {
                    t0 += xchg[w];
                    t1 += xchg[16 + w];
                }
                s_dyh = t0;
                s_dyx = t1;
                rstd = a.rstd[r];
            } else {
                float tot = 0.f;
                for (int w = 0; w < nwaves; ++w) tot += xchg[32 + w];
                const float mean = tot * a.inv_D;
                float M2 = 0.f, t0 = 0.f, t1 = 0.f;
                for (int w = 0; w < nwaves; ++w) {
                    const float inw = nw_inv[w];
                    const float d = xchg[32 + w] * inw - mean;   // mean_w - mean
                    M2 += xchg[48 + w] + d * d / inw;
                    t0 += xchg[w];
                    t1 += xchg[16 + w] + d * xchg[w];
                }
                s_dyh = t0;
                s_dyx = t1;
                shift = pivot - mean;
                rstd = rsqrtf(M2 * a.inv_D + a.eps);
            }
        } else {
            if constexpr (kSaved) rstd = a.rstd[r];
            else rstd = rsqrtf(m2 * a.inv_D + a.eps);
        }
        // pass 3: dx = rstd*(dyh - c2 - xhat*c1), c1 = rstd*mean_d(dyh*(x-mean)), c2 = mean_d(dyh)
        const float k1 = -rstd * rstd * s_dyx * a.inv_D, k2 = -rstd * s_dyh * a.inv_D;
        Raw *orow = dxv + r * a.nvec;
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            float o[E];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float xhat = kMulti && !kSaved ? (xf[k][e] + shift) * rstd : xf[k][e] * rstd;
                o[e] = (df[k][e] * gm[k][e]) * rstd + (xhat * k1 + k2);
                acc_g[k][e] += df[k][e] * xhat;
                acc_b[k][e] += df[k][e];
            }
            if (ok[k]) orow[vidx[k]] = V::pack(o);
        }
        parity ^= 1;
    };

    // two register buffers: the next row's loads are in flight while the current row is reduced
    while (t < t_end) {
        if (t + step < t_end) load_row(t + step, xb, db);
        process(t, xa, da);
        t += step;
        if (t >= t_end) break;
        if (t + step < t_end) load_row(t + step, xa, da);
        process(t, xb, db);
        t += step;
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
