// Row-streaming kernels: the single pass over x and dy that writes dx and accumulates the
// column sums  A_gamma[k] = sum_t dy*xhat,  A_beta[k] = sum_t dy  over one chunk of rows.
//
// Work partition.  The N = B*T rows are cut into `n_slots` chunks, one workgroup each.  For the
// per-example path chunks never straddle an example: example b owns chunks [b*C, (b+1)*C), so the
// per-example sums of Appendix B steps 1 and 5 are sums of whole chunks.  Chunk j takes rows
// j, j+C, j+2C, ... of its example (the workgroups of an example then sweep one moving window of
// memory together) or, when the host says so, a block of consecutive rows.  The plain backward
// uses the same kernels with the whole tensor declared as one "example" (Tp = N).
//
// Lane mapping.  A lane owns the same columns for every row it touches, so the sums over t
// live in registers and never move between lanes; only the per-row scalars cross lanes, on the
// DPP network.  A workgroup is R row groups of S waves: the S waves of a group share a row
// (each owns different columns, 16 per lane and up to 32 for the widest rows), the R groups take different rows and
// merge their column sums through LDS in group order when the chunk is done.
#pragma once
#include <type_traits>

#include "lnpegn_device.h"

namespace lnpegn {

struct RowArgs {
    const void *x;
    const void *dy;
    const void *gamma;
    const float *mean;   // may be null (recompute)
    const float *rstd;
    void *dx;
    float *part;         // [n_slots][2][D] fp32 column sums per chunk
    float *pe_gamma_sq;  // [B], written here only when emit_pe
    float *pe_beta_sq;
    DeferHeader *defer;  // not null: leave `hdr` there for the batched reduction
    DeferHeader hdr;
    int64_t Tp;          // rows per partition example
    int64_t stagger;     // example b starts its sweep at row (b*stagger) mod Tp of itself
    int C;               // chunks per partition example
    int rows_per;        // > 0: chunk j owns the rows [j*rows_per, (j+1)*rows_per) of its example; 0: the rows
                         //      j, j + C, j + 2C, ... (the chunks of an example sweep it side by side)
    int D;
    int nvec;            // D / elements-per-vector
    int S;               // waves per row
    int gamma_is_f32;
    int emit_pe;         // C == 1: a chunk is a whole example, its squared norms are final here
    int rms;             // RMSNorm variant: no mean is subtracted, no beta (uniform run-time flag)
    int xcd_chunks;      // > 0: chunks per XCD; workgroup i (dispatched to XCD i % 8) takes chunk
                         //      (i % 8) * xcd_chunks + i / 8, so neighbouring chunks share an L2
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

// Valid elements owned by wave ws of a row group (the S waves interleave inside 64*S-vector spans).
template <int kVpt, int E>
__device__ __forceinline__ int wave_valid_elems(int ws, int S, int nvec)
{
    int n = 0;
#pragma unroll
    for (int k = 0; k < kVpt; ++k) {
        const int left = nvec - (k * S + ws) * kWave;
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
//
// kS: waves per row.  1: a wave owns a row, nothing crosses waves.  2, 4, 8: that many waves share
// a row and exchange their scalars through LDS (one barrier per row; every wave of the
// workgroup takes part in every barrier, also a group that has run out of rows).  0: the same
// with S read at run time (3, 5, 6, 7 waves).
// kFull: every lane owns kVpt valid vectors (nvec == 64*S*kVpt), so no padding logic is compiled.
// Launch bounds.  Lanes that own more than 8 elements (two or more 16-byte vectors of bf16) run as one workgroup
// of up to 8 waves per CU, whatever the number of waves per row; lanes with one vector run as several small
// workgroups per CU, except that four waves per row may also pair up as two row groups.
constexpr bool rows_kernel_narrow4(int kS, int elems) { return kS == 4 && elems <= 8; }
constexpr int rows_kernel_max_threads(int kS, int elems)
{
    return (kS == 0 || kS == 8 || elems > 8 || rows_kernel_narrow4(kS, elems)) ? 512 : 256;
}
constexpr int rows_kernel_min_blocks(int kS, int elems)
{
    return elems > 8 ? 1 : rows_kernel_narrow4(kS, elems) ? 2 : 4;
}

// kPlain: the plain backward (one partition "example" spanning the whole tensor, never any
// per-example output); it is a kernel of its own name so that a kernel trace tells the two apart.
// kDxCached: dx is small enough for the memory-side cache: write-through stores instead of streaming ones.
template <typename T, int kVpt, bool kSaved, int kS, bool kFull, bool kPlain, bool kDxCached>
__device__ __forceinline__ void ln_bwd_rows_body(const RowArgs &a)
{
    using V = Vec<T>;
    using Raw = typename V::Raw;
    constexpr int E = V::kElems;
    constexpr bool kSync = kS != 1;
    // Cache policy of the row accesses (bits of the buffer instructions: 1 = sc0, 2 = nt, 16 = sc1), every one
    // of them from measurements on B*T = 32768 rows:
    //   x, dy   streaming loads at every row width (they are read once; cached loads: D=8192 291 against 276 us,
    //           D=4096 145 against 139 us)
    //   dx      streaming stores when dx is larger than what the memory-side cache takes next to the reads;
    //           system-scope write-through stores (sc0 sc1) when it is not (B=512 T=64 D=1024: streaming 41.6,
    //           plain write-back 37.3, sc0 sc1 35.6 us; at B=16 T=2048 D=2048 streaming wins, 70.6 against 77.5 us)
    constexpr int kLoadAux = 2;
    constexpr int kStoreAuxLarge = 2;
    constexpr int kStoreAuxSmall = 17;
    constexpr bool kDrainStores = kS == 2;
    constexpr int NF = 2 * kVpt * E;  // accumulator floats per lane
    constexpr int KL = kVpt - 1;      // only a lane's last vector slot can be padding
    extern __shared__ __align__(16) float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int S = kS > 0 ? kS : a.S;
    const int R = nwaves / S;
    const int g = wave / S, ws = wave - g * S;
    const int chunk = a.xcd_chunks > 0 ? (blockIdx.x & 7) * a.xcd_chunks + (blockIdx.x >> 3) : blockIdx.x;
    const int b = chunk / a.C, j = chunk - b * a.C;
    // Chunk j of example b owns rows b*Tp + j + m*C, or a block of consecutive rows.  Examples sit
    // a power of two apart in memory; starting each sweep at a different row (wrapping around)
    // keeps the concurrent sweeps on different HBM channels.
    const int Tp = (int)a.Tp;
    const int row_base = b * Tp;
    const int t_rot = (int)(((int64_t)b * a.stagger) % a.Tp);
    const bool blocked = a.rows_per > 0;
    const int row_first = blocked ? j * a.rows_per : j;
    const int row_step = blocked ? 1 : a.C;
    const int n_rows = blocked ? max(0, min(a.rows_per, Tp - row_first))
                               : (Tp - j + a.C - 1) / a.C;   // rows of this chunk
    const int n_full = n_rows / R;                 // iterations in which every row group has a row
    const bool has_tail = n_rows - n_full * R > 0;
    if (a.defer && blockIdx.x == 0 && threadIdx.x == 0) *a.defer = a.hdr;

    int vidx[kVpt];
#pragma unroll
    for (int k = 0; k < kVpt; ++k) vidx[k] = (k * S + ws) * kWave + lane;
    const bool ok_last = kFull ? true : vidx[KL] < a.nvec;
    const int v_last = ok_last ? vidx[KL] : 0;     // gamma of a padded lane: a valid vector, then zeroed
    const int n_w = wave_valid_elems<kVpt, E>(ws, S, a.nvec);

    // Rows are addressed as buffers of one row each: a padded lane (vector index >= nvec) reads
    // zeros and its store is dropped, with no branch around the access.
    const int row_bytes = a.nvec * (int)sizeof(Raw);
    const char *xbase = static_cast<const char *>(a.x);
    const char *dybase = static_cast<const char *>(a.dy);
    char *dxbase = static_cast<char *>(a.dx);

    auto row_of = [&](int m) {   // m-th row of the chunk -> global row index (wave-uniform)
        int u = row_first + m * row_step + t_rot;
        u = u >= Tp ? u - Tp : u;
        return __builtin_amdgcn_readfirstlane(row_base + u);
    };
    // saved statistics of the row in flight: fetched with the row, a whole iteration before use
    float st_mean = 0.f, st_rstd = 0.f;
    auto load_row = [&](int m, Raw (&xr)[kVpt], Raw (&dr)[kVpt]) {
        const int rr = row_of(m);
        if constexpr (kSaved) {
            st_mean = a.rms ? 0.f : a.mean[rr];
            st_rstd = a.rstd[rr];
        }
        const int64_t off = (int64_t)rr * row_bytes;
        const rsrc_t rx = make_rsrc(xbase + off, row_bytes);
        const rsrc_t rd = make_rsrc(dybase + off, row_bytes);
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            xr[k] = V::template load_buf<kLoadAux>(rx, vidx[k] * (int)sizeof(Raw));
            dr[k] = V::template load_buf<kLoadAux>(rd, vidx[k] * (int)sizeof(Raw));
        }
    };

    // first row on its way before anything else is fetched
    int m = g;
    Raw xr[kVpt], dr[kVpt];
    if (m < n_rows) load_row(m, xr, dr);

    float gm[kVpt][E];
#pragma unroll
    for (int k = 0; k < kVpt; ++k) {
        load_gamma_vec<T>(a.gamma, a.gamma_is_f32, k < KL ? vidx[k] : v_last, gm[k]);
        if (k == KL && !ok_last) {
#pragma unroll
            for (int e = 0; e < E; ++e) gm[k][e] = 0.f;
        }
    }

    float acc_g[kVpt][E], acc_b[kVpt][E];
#pragma unroll
    for (int k = 0; k < kVpt; ++k)
#pragma unroll
        for (int e = 0; e < E; ++e) acc_g[k][e] = acc_b[k][e] = 0.f;

    // LDS: [parity][R][S] exchange float4 {sum dyh, sum dyh*xc, sum x, M2}, then S floats n_w and
    // S floats 1/n_w (rows with padding only), two floats per wave for the per-example norms, then the
    // merge buffer (16-byte aligned).
    float4 *xchg_base = reinterpret_cast<float4 *>(lds);
    float *nw_tab = lds + 8 * nwaves;
    float *pe_slots = nw_tab + 2 * S;     // 2 floats per wave: the waves' parts of an example's squared norms
    float *merge = lds + ((10 * nwaves + 2 * S + 3) & ~3);
    if constexpr (kSync && !kFull) {
        if (lane == 0 && g == 0) {
            nw_tab[ws] = (float)n_w;
            nw_tab[S + ws] = 1.0f / (float)n_w;
        }
    }
    const float inv_nw = 1.0f / (float)n_w;
    int parity = 0;

    // kTail: the last, partial iteration -- only row groups that still have a row do the work,
    // but every wave meets the barrier.
    // One register buffer: a row is unpacked to fp32, then the same registers receive the next
    // row's loads, which stay in flight while the current row is reduced.
    auto process = [&](auto tail_tag, int mm) {
        constexpr bool kTail = decltype(tail_tag)::value;
        const bool act = kTail ? mm < n_rows : true;
        float xf[kVpt][E], df[kVpt][E];
        float s_x = 0.f, pivot = 0.f, m2 = 0.f, s_dyh = 0.f, s_dyx = 0.f, rstd_saved = 0.f;
        int r = 0;
        float4 *xchg = xchg_base + (parity * R + g) * S;
        if (act) {
            r = row_of(mm);
            // Rows shared by two waves run faster when a row group lets its previous dx stores land before
            // it asks for the next row (measured, B=16 T=2048 D=2048: 69.6 -> 67.0 us per-example,
            // 66.0 -> 65.4 plain); every other row width is faster with the stores left in flight.
            if constexpr (kDrainStores) __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0) only
#pragma unroll
            for (int k = 0; k < kVpt; ++k) {
                V::unpack(xr[k], xf[k]);   // padded lanes hold zeros: the buffer load returned them
                V::unpack(dr[k], df[k]);
            }
            const float saved_mean = st_mean, saved_rstd = st_rstd;   // this row's, before the prefetch
            if (mm + R < n_rows) load_row(mm + R, xr, dr);
            // pass 1: pivot = the wave's own mean (or the saved row mean)
            if constexpr (kSaved) {
                pivot = saved_mean;
                rstd_saved = saved_rstd;
            } else {
                if (!a.rms) {   // RMSNorm: the pivot is zero, M2 is the plain sum of squares
#pragma unroll
                    for (int k = 0; k < kVpt; ++k)
#pragma unroll
                        for (int e = 0; e < E; ++e) s_x += xf[k][e];
                    s_x = wave_sum(s_x);
                    pivot = s_x * (kSync ? inv_nw : a.inv_D);
                }
            }
            // pass 2: centre about the pivot; M2, sum dyh, sum dyh*xc
#pragma unroll
            for (int k = 0; k < kVpt; ++k)
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    float xc = xf[k][e] - pivot;
                    if (!kFull && k == KL) xc = ok_last ? xc : 0.f;
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
            if constexpr (kSync) {
                if (lane == 0) xchg[ws] = make_float4(s_dyh, s_dyx, s_x, m2);
            }
        }
        if constexpr (kSync) __syncthreads();
        if (act) {
            float rstd, shift_r = 0.f;   // shift_r = (pivot - mean) * rstd
            if constexpr (kSync) {
                const int nS = kS > 0 ? kS : S;    // compile-time trip count when kS > 0
                float4 part[kS > 0 ? kS : 8];
#pragma unroll
                for (int w = 0; w < (kS > 0 ? kS : 8); ++w)
                    part[w] = w < nS ? xchg[w] : make_float4(0.f, 0.f, 0.f, 0.f);
                if constexpr (kSaved) {
                    float t0 = 0.f, t1 = 0.f;
#pragma unroll
                    for (int w = 0; w < (kS > 0 ? kS : 8); ++w) {
                        t0 += part[w].x;
                        t1 += part[w].y;
                    }
                    s_dyh = t0;
                    s_dyx = t1;
                    rstd = rstd_saved;
                } else {
                    float tot = 0.f;
#pragma unroll
                    for (int w = 0; w < (kS > 0 ? kS : 8); ++w) tot += part[w].z;
                    const float mean = tot * a.inv_D;
                    float M2 = 0.f, t0 = 0.f, t1 = 0.f;
#pragma unroll
                    for (int w = 0; w < (kS > 0 ? kS : 8); ++w) {
                        if (kS > 0 || w < nS) {
                            const float nw = kFull ? (float)(kVpt * E * kWave) : nw_tab[w];
                            const float inw = kFull ? 1.0f / (float)(kVpt * E * kWave) : nw_tab[S + w];
                            const float d = part[w].z * inw - mean;   // mean_w - mean
                            M2 += part[w].w + d * d * nw;
                            t0 += part[w].x;
                            t1 += part[w].y + d * part[w].x;
                        }
                    }
                    s_dyh = t0;
                    s_dyx = t1;
                    rstd = rsqrtf(M2 * a.inv_D + a.eps);
                    shift_r = (pivot - mean) * rstd;
                }
            } else {
                if constexpr (kSaved) rstd = rstd_saved;
                else rstd = rsqrtf(m2 * a.inv_D + a.eps);
            }
            // pass 3: dx = rstd*(dyh - c2 - xhat*c1), c1 = rstd*mean_d(dyh*(x-mean)), c2 = mean_d(dyh)
            const float k1 = -rstd * rstd * s_dyx * a.inv_D;
            const float k2 = a.rms ? 0.f : -rstd * s_dyh * a.inv_D;   // RMSNorm has no mean(dyh) term
            const rsrc_t ro = make_rsrc(dxbase + (int64_t)r * row_bytes, row_bytes);
            Raw packed[kVpt];
#pragma unroll
            for (int k = 0; k < kVpt; ++k) {
                float o[E];
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float xhat = kSync && !kSaved ? xf[k][e] * rstd + shift_r : xf[k][e] * rstd;
                    o[e] = (df[k][e] * gm[k][e]) * rstd + (xhat * k1 + k2);
                    acc_g[k][e] += df[k][e] * xhat;
                    acc_b[k][e] += df[k][e];
                }
                packed[k] = V::pack(o);
            }
            // dx is written once and not read back here.  Streaming stores for tensors that no cache
            // holds, write-back stores where the memory-side cache can take them: a compile-time choice,
            // because a branch around a store makes the compiler wait for every store at the loop head
#pragma unroll
            for (int k = 0; k < kVpt; ++k)
                V::template store_buf<kDxCached ? kStoreAuxSmall : kStoreAuxLarge>(
                    ro, vidx[k] * (int)sizeof(Raw), packed[k]);
        }
        parity ^= 1;
    };

    using Full = std::integral_constant<bool, false>;
    using Tail = std::integral_constant<bool, true>;
    // The first row is taken outside the loop so that the loop is entered in the state it
    // repeats: next row's loads issued, then this row's stores.  The wait for a row's data can
    // then leave the younger stores outstanding (vmcnt counts loads and stores in issue order);
    // entered straight from the prologue, the compiler has to wait for everything at the loop
    // head, i.e. for the previous row's stores to be acknowledged by memory, once per row.
    if (n_full > 0) {
        process(Full{}, m);
        m += R;
    }
    for (int it = 1; it < n_full; ++it) {
        process(Full{}, m);
        m += R;
    }
    if (has_tail) process(Tail{}, m);

    // ---- hand the chunk's column sums to the workspace ----
    float *out_g = a.part + (int64_t)chunk * 2 * a.D;
    float *out_b = out_g + a.D;
    double sq_g = 0.0, sq_b = 0.0;   // squares of the final sums this lane writes (emit_pe)
    if (R == 1) {
        // one row group: every wave owns its columns, straight from registers
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            if (k < KL || ok_last) {
#pragma unroll
                for (int q = 0; q < E / 4; ++q) {
                    const int64_t col = (int64_t)vidx[k] * E + q * 4;
                    *reinterpret_cast<float4 *>(out_g + col) = make_float4(
                        acc_g[k][q * 4], acc_g[k][q * 4 + 1], acc_g[k][q * 4 + 2], acc_g[k][q * 4 + 3]);
                    *reinterpret_cast<float4 *>(out_b + col) = make_float4(
                        acc_b[k][q * 4], acc_b[k][q * 4 + 1], acc_b[k][q * 4 + 2], acc_b[k][q * 4 + 3]);
                }
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    sq_g += (double)acc_g[k][e] * (double)acc_g[k][e];
                    sq_b += (double)acc_b[k][e] * (double)acc_b[k][e];
                }
            }
        }
    } else {
        // merge the row groups' sums through LDS, adding in group order (reproducible); a lane's 2*kVpt*E
        // sums travel as NQ quads of four consecutive columns, one 16-byte LDS access each
        constexpr int NQ = NF / 4;
        float4 *merge4 = reinterpret_cast<float4 *>(merge);
        float4 *mine = merge4 + (int64_t)wave * NQ * kWave + lane;
#pragma unroll
        for (int k = 0; k < kVpt; ++k)
#pragma unroll
            for (int h = 0; h < E / 4; ++h) {
                mine[((0 * kVpt + k) * (E / 4) + h) * kWave] =
                    make_float4(acc_g[k][4 * h], acc_g[k][4 * h + 1], acc_g[k][4 * h + 2], acc_g[k][4 * h + 3]);
                mine[((1 * kVpt + k) * (E / 4) + h) * kWave] =
                    make_float4(acc_b[k][4 * h], acc_b[k][4 * h + 1], acc_b[k][4 * h + 2], acc_b[k][4 * h + 3]);
            }
        __syncthreads();
        for (int q = g; q < NQ; q += R) {
            const int f0 = q * 4;
            const int arr = f0 / (kVpt * E);
            const int k = (f0 / E) % kVpt;
            const int e0 = f0 % E;
            float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int gg = 0; gg < R; ++gg) {
                const float4 t = merge4[((int64_t)(gg * S + ws) * NQ + q) * kWave + lane];
                s4.x += t.x; s4.y += t.y; s4.z += t.z; s4.w += t.w;
            }
            const int v = (k * S + ws) * kWave + lane;
            if (v < a.nvec) {
                float *dst = (arr == 0 ? out_g : out_b) + (int64_t)v * E + e0;
                *reinterpret_cast<float4 *>(dst) = s4;
                const double q2 = (double)s4.x * s4.x + (double)s4.y * s4.y + (double)s4.z * s4.z +
                                  (double)s4.w * s4.w;
                if (arr == 0) sq_g += q2;
                else sq_b += q2;
            }
        }
    }
    if (!kPlain && a.emit_pe) {
        // Appendix B steps 2 and 6 for the example this workgroup owns entirely.  A lane's squares are
        // summed in fp64; the 64 lanes' sums then cross the wave as fp32 on the DPP network (positive
        // terms, a tree of depth 6: relative error below 1e-6) and the waves' sums are added in wave
        // order in fp64: one barrier in all.
        float wg = (float)sq_g, wb = (float)sq_b;
        wave_sum2(wg, wb);
        if (lane == 0) {
            pe_slots[2 * wave] = wg;
            pe_slots[2 * wave + 1] = wb;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            double tg = 0.0, tb = 0.0;
            for (int w = 0; w < nwaves; ++w) {
                tg += (double)pe_slots[2 * w];
                tb += (double)pe_slots[2 * w + 1];
            }
            a.pe_gamma_sq[b] = (float)tg;
            if (a.pe_beta_sq) a.pe_beta_sq[b] = (float)tb;
        }
    }
}

template <typename T, int kVpt, bool kSaved, int kS, bool kFull, bool kDxCached>
__global__ __launch_bounds__(rows_kernel_max_threads(kS, kVpt * Vec<T>::kElems),
                             rows_kernel_min_blocks(kS, kVpt * Vec<T>::kElems))
void ln_bwd_rows_kernel(RowArgs a)
{
    ln_bwd_rows_body<T, kVpt, kSaved, kS, kFull, false, kDxCached>(a);
}

template <typename T, int kVpt, bool kSaved, int kS, bool kFull, bool kDxCached>
__global__ __launch_bounds__(rows_kernel_max_threads(kS, kVpt * Vec<T>::kElems),
                             rows_kernel_min_blocks(kS, kVpt * Vec<T>::kElems))
void ln_bwd_plain_rows_kernel(RowArgs a)
{
    ln_bwd_rows_body<T, kVpt, kSaved, kS, kFull, true, kDxCached>(a);
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
    if (a.defer && blockIdx.x == 0 && tid == 0) *a.defer = a.hdr;
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
            mean = a.rms ? 0.f : a.mean[r];
            rstd = a.rstd[r];
        } else {
            float s_x = 0.f;
            if (!a.rms)
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
        const float c1 = s_dx * a.inv_D, c2 = a.rms ? 0.f : s_dyh * a.inv_D;
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
// Forward: mean and rstd of every row (two-pass variance in fp32) and, with kWriteY, the
// LayerNorm output y = gamma*xhat + beta.  Rows are taken in a grid-stride sweep (one moving
// window of memory); wide rows use the whole workgroup.
// ---------------------------------------------------------------------------------------
struct FwdArgs {
    const void *x;
    const void *gamma;  // kWriteY only
    const void *beta;   // kWriteY only
    void *y;            // kWriteY only
    float *mean;        // may be null
    float *rstd;        // may be null
    int64_t N;
    int D;
    int nvec;
    int gamma_is_f32;
    int rms;            // RMSNorm: mean taken as zero, beta absent
    float eps;
    float inv_D;
};

template <typename T, int kVpt, bool kMulti, bool kWriteY>
__global__ void ln_fwd_kernel(FwdArgs a)
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
    float gm[kWriteY ? kVpt : 1][E], bt[kWriteY ? kVpt : 1][E];
    if constexpr (kWriteY) {
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            load_gamma_vec<T>(a.gamma, a.gamma_is_f32, ok[k] ? vidx[k] : 0, gm[k]);
            if (a.beta) {
                load_gamma_vec<T>(a.beta, a.gamma_is_f32, ok[k] ? vidx[k] : 0, bt[k]);
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) bt[k][e] = 0.f;
            }
        }
    }
    const Raw *xv = static_cast<const Raw *>(a.x);
    Raw *yv = static_cast<Raw *>(a.y);
    const int64_t first = kMulti ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * nwaves + wave;
    const int64_t stride = kMulti ? (int64_t)gridDim.x : (int64_t)gridDim.x * nwaves;
    for (int64_t r = first; r < a.N; r += stride) {
        float xf[kVpt][E];
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < kVpt; ++k) {
            Raw raw = V::zero();
            if (ok[k]) raw = V::load_stream(xv + r * a.nvec + vidx[k]);   // x is not read again by this kernel
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
        const float mean = a.rms ? 0.f : s * a.inv_D;
        float ss = 0.f;
#pragma unroll
        for (int k = 0; k < kVpt; ++k)
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float c = ok[k] ? xf[k][e] - mean : 0.f;
                xf[k][e] = c;
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
        const float rstd = rsqrtf(ss * a.inv_D + a.eps);
        if (threadIdx.x == (kMulti ? 0 : wave * kWave)) {
            if (a.mean) a.mean[r] = mean;
            if (a.rstd) a.rstd[r] = rstd;
        }
        if constexpr (kWriteY) {
#pragma unroll
            for (int k = 0; k < kVpt; ++k) {
                float o[E];
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = xf[k][e] * rstd * gm[k][e] + bt[k][e];
                if (ok[k]) V::store_stream(yv + r * a.nvec + vidx[k], V::pack(o));
            }
        }
    }
}

template <typename T, bool kWriteY>
__global__ void ln_fwd_generic_kernel(FwdArgs a)
{
    __shared__ float slots[8];
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int64_t r = blockIdx.x; r < a.N; r += gridDim.x) {
        const int64_t base = r * (int64_t)a.D;
        float s = 0.f;
        for (int k = tid; k < a.D; k += nt) s += load_elem<T>(a.x, base + k);
        const float mean = a.rms ? 0.f : block_sum(s, slots) * a.inv_D;
        float ss = 0.f;
        for (int k = tid; k < a.D; k += nt) {
            const float c = load_elem<T>(a.x, base + k) - mean;
            ss += c * c;
        }
        ss = block_sum(ss, slots);
        const float rstd = rsqrtf(ss * a.inv_D + a.eps);
        if (tid == 0) {
            if (a.mean) a.mean[r] = mean;
            if (a.rstd) a.rstd[r] = rstd;
        }
        if constexpr (kWriteY) {
            for (int k = tid; k < a.D; k += nt) {
                const float xhat = (load_elem<T>(a.x, base + k) - mean) * rstd;
                store_elem<T>(a.y, base + k,
                              xhat * load_gamma(a.gamma, a.gamma_is_f32, k) +
                                  (a.beta ? load_gamma(a.beta, a.gamma_is_f32, k) : 0.f));
            }
        }
    }
}

}  // namespace lnpegn
