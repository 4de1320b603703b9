// Linear-layer simultaneous per-example gradient norms (Section 3, Algorithm 1) for gfx950:
//   w_b[k,l] = sum_t x[b,t,k] g[b,t,l]   (step 1; never leaves the chip)
//   s[b]     = sum_{k,l} w_b[k,l]^2      (step 2)
//   w'[k,l]  = sum_b w_b[k,l]            (step 3)
// One MFMA contraction per example with two accumulator sets per wave: the example's own tile, squared
// and folded into the running total at every example boundary.  The paper materialises [B,K,L] and
// pays its I/O (Section 3.1, Appendix E); here the only extra HBM traffic is B floats per tile.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lnpegn.h"
#include "lnpegn_device.h"

namespace lnpegn {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// Workgroup tile: 256 (k) x 128 (l) outputs, 64 positions t per LDS stage, 8 waves as 4 (k) x 2 (l),
// each wave 64 x 64 = 2 x 2 MFMA tiles of 32 x 32.  Operands sit in LDS transposed, [column][t], so an
// MFMA operand (8 consecutive t of one column) is one 16-byte read; rows are padded to 144 bytes,
// which spreads 16 consecutive columns over all 64 banks.
constexpr int kTileK = 256, kTileL = 128, kStageT = 64, kThreads = 512, kWaves = 8;
constexpr int kPitch = 144;                                   // bytes per LDS row (64 t x 2 B + 16)
constexpr int kStageBytes = (kTileK + kTileL) * kPitch;       // 55,296
constexpr int kMaxSplit = 64;

struct LinArgs {
    const uint16_t *x;      // [B,T,K] bf16
    const uint16_t *g;      // [B,T,L] bf16
    float *out;             // nsplit == 1: w [K,L]; else partial totals [nsplit][K][L]
    float *tile_s;          // [B][ntiles*kWaves] per-wave parts of s[b]
    double *tile_big;       // [ntiles*kWaves] per-wave parts of ||w'||^2 (nsplit == 1 only)
    int B, T, K, L;
    int tiles_k, tiles_l, nsplit, b_per_split;
    int accumulate;         // nsplit == 1: add the total to what out holds
};

__device__ __forceinline__ int xcd_spread(int bid, int n)
{
    // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of logical
    // tiles (k fastest), so that workgroups sharing an operand share an L2.
    const int q = n >> 3, r = n & 7, xcd = bid & 7, loc = bid >> 3;
    return xcd * q + (xcd < r ? xcd : r) + loc;
}

__global__ __launch_bounds__(kThreads) void linear_pegn_kernel(LinArgs a)
{
    // two named buffers rather than an indexed pair: the compiler then knows that writing one and
    // reading the other never alias, and may interleave the two
    __shared__ __align__(16) unsigned char lds0[kStageBytes], lds1[kStageBytes];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: branches on it are scalar
    const int ntiles = a.tiles_k * a.tiles_l;
    const int tile = xcd_spread(blockIdx.x, ntiles);
    const int split = blockIdx.y;
    const int k0 = (tile % a.tiles_k) * kTileK, l0 = (tile / a.tiles_k) * kTileL;
    const int b_begin = split * a.b_per_split;
    const int b_end = b_begin + a.b_per_split < a.B ? b_begin + a.b_per_split : a.B;
    const int nst = (a.T + kStageT - 1) / kStageT;
    const int nstages = (b_end - b_begin) * nst;

    // ---- loader role: waves 0-3 bring 64 columns of x each, waves 4-5 bring 64 columns of g each.
    // A lane owns an 8 (t) x 8 (column) block: eight 16-byte row loads, transposed in registers.
    const bool loads = wave < 6;
    const bool from_x = wave < 4;
    const int sub = from_x ? wave : wave - 4;
    const int cg = lane & 7, tb = lane >> 3;                  // 8 adjacent lanes read one 128-byte line
    const int ncols = from_x ? a.K : a.L;
    const int col = (from_x ? k0 : l0) + sub * 64 + cg * 8;
    const bool col_ok = loads && col < ncols;                 // K, L are multiples of 8: all or nothing
    const uint16_t *src = from_x ? a.x : a.g;
    // Column cg*8 + i of a wave's 64 goes to LDS row i*8 + cg: the eight lanes of a line then write
    // eight consecutive rows (bank-conflict free), and the compute side undoes the permutation when
    // it names its outputs (an MFMA row can be any column as long as the result is filed under it).
    const int lds_row = (from_x ? 0 : kTileK) + sub * 64 + cg;
    u32x4_t raw[8];

    unsigned raw_ok = 0;                                       // bit j: row j of the block exists
    int fb = b_begin, fs = 0;                                  // the next stage to fetch: example, stage in it
    const int colx = col_ok ? col : 0;
    auto fetch = [&]() {
        // nothing here waits for the data; a row past the end of the example is read from the
        // example's last row instead and replaced by zeros when the block is transposed
        const int rows_left = a.T - fs * kStageT;
        const uint16_t *base = src + ((int64_t)fb * a.T + fs * kStageT) * ncols + colx;
        raw_ok = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = tb * 8 + j;
            const bool ok = col_ok && r < rows_left;
            raw_ok |= (ok ? 1u : 0u) << j;
            const int rc = r < rows_left ? r : rows_left - 1;
            raw[j] = *reinterpret_cast<const u32x4_t *>(base + (int64_t)rc * ncols);
        }
        if (++fs == nst) {
            fs = 0;
            ++fb;
        }
    };
    auto stash = [&](unsigned char *dst) {
        unsigned char *base = dst + lds_row * kPitch + tb * 16;
        if (raw_ok != 0xffu) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (!((raw_ok >> j) & 1u)) raw[j] = u32x4_t{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {                          // column i of the block
            u32x4_t o;
#pragma unroll
            for (int tp = 0; tp < 4; ++tp) {                   // positions 2tp, 2tp+1
                const uint32_t u = raw[2 * tp][i >> 1], v = raw[2 * tp + 1][i >> 1];
                o[tp] = (i & 1) ? ((u >> 16) | (v & 0xffff0000u)) : ((u & 0xffffu) | (v << 16));
            }
            *reinterpret_cast<u32x4_t *>(base + i * 8 * kPitch) = o;
        }
    };

    // ---- compute role: wave (wm, wn) owns outputs k0 + wm*64 .. +64, l0 + wn*64 .. +64
    const int wm = wave & 3, wn = wave >> 2;
    const int frag_off = (lane & 31) * kPitch + (lane >> 5) * 16;
    const int a_off = (wm * 64) * kPitch + frag_off;
    const int b_off = (kTileK + wn * 64) * kPitch + frag_off;
    f32x16_t acc[2][2], tot[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                acc[mi][ni][i] = 0.f;
                tot[mi][ni][i] = 0.f;
            }

    // Pipeline: stage st is multiplied out of LDS buffer st&1 while stage st+1 is transposed into the
    // other buffer and stage st+2 is in flight from memory, so a load has a whole iteration to land.
    // Loading and non-loading waves run separate copies of the loop (the branch is scalar), so that in
    // a loading wave the transpose of one block and the MFMAs of another sit in one basic block and the
    // scheduler can put the former into the shadow of the latter.
    int cb = b_begin, cs = 0;                                  // the stage being multiplied
    auto multiply = [&](const unsigned char *cur) {
        const unsigned char *sa = cur + a_off, *sb = cur + b_off;
#pragma unroll
        for (int kk = 0; kk < kStageT / 16; ++kk) {
            bf16x8_t fa[2], fb[2];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
                fa[mi] = *reinterpret_cast<const bf16x8_t *>(sa + mi * 32 * kPitch + kk * 32);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                fb[ni] = *reinterpret_cast<const bf16x8_t *>(sb + ni * 32 * kPitch + kk * 32);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
        }
    };
    auto example_done = [&]() {
        // example boundary: step 2 on this wave's 64 x 64 part, then fold it into the total (step 3)
        float ssq = 0.f;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float v = acc[mi][ni][i];
                    ssq = fmaf(v, v, ssq);
                    tot[mi][ni][i] += v;
                    acc[mi][ni][i] = 0.f;
                }
        ssq = wave_sum(ssq);
        if (lane == 0) a.tile_s[(int64_t)cb * (ntiles * kWaves) + tile * kWaves + wave] = ssq;
        ++cb;
    };
    auto interleave = [&]() {
        // Ask the scheduler for one MFMA, then a handful of the transpose's VALU operations in its
        // shadow, an LDS write and an LDS read, sixteen times over; the loads for stage st+2 last.
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x020, 8, 0);
    };
    auto boundary = [&]() {
        if (++cs == nst) {
            cs = 0;
            example_done();
        }
    };
    if (loads) {
        if (nstages > 0) {
            fetch();
            stash(lds0);
            if (nstages > 1) fetch();
        }
        __syncthreads();
        int st = 0;
        for (; st + 3 < nstages; st += 2) {                    // steady state: no conditions in the bodies
            stash(lds1);
            fetch();
            multiply(lds0);
            interleave();
            boundary();
            __syncthreads();
            stash(lds0);
            fetch();
            multiply(lds1);
            interleave();
            boundary();
            __syncthreads();
        }
        for (; st < nstages; ++st) {
            unsigned char *cur = (st & 1) ? lds1 : lds0, *nxt = (st & 1) ? lds0 : lds1;
            if (st + 1 < nstages) stash(nxt);
            if (st + 2 < nstages) fetch();
            multiply(cur);
            boundary();
            __syncthreads();
        }
    } else {
        __syncthreads();
        for (int st = 0; st < nstages; ++st) {
            multiply((st & 1) ? lds1 : lds0);
            boundary();
            __syncthreads();
        }
    }

    // ---- write the total: lane holds rows (i/4)*8 + (lane/32)*4 + i%4, column lane%32 of each 32x32 tile,
    // both in LDS row numbering; unperm() gives the column of x (of g) that sits in an LDS row
    auto unperm = [](int p) { return (p & 7) * 8 + (p >> 3); };
    float *out = a.out + (a.nsplit > 1 ? (int64_t)split * a.K * a.L : 0);
    double bsq = 0.0;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int l = l0 + wn * 64 + unperm(ni * 32 + (lane & 31));
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int k = k0 + wm * 64 + unperm(mi * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3));
                if (k < a.K && l < a.L) {
                    float *p = out + (int64_t)k * a.L + l;
                    float v = tot[mi][ni][i];
                    if (a.accumulate && a.nsplit == 1) v += *p;
                    *p = v;
                    bsq += (double)v * (double)v;
                }
            }
        }
    if (a.nsplit == 1) {
        bsq = wave_sum_f64(bsq);
        if (lane == 0) a.tile_big[tile * kWaves + wave] = bsq;
    }
}

// Any shape, any alignment, fp32 or bf16: one thread per output (k,l), fp32 FMA over t, no MFMA.
// Correct, not fast; covers what the MFMA kernel does not take.
template <typename T>
__global__ __launch_bounds__(256) void linear_pegn_generic_kernel(const T *x, const T *g, float *w, float *blk_s,
                                                                  double *blk_big, int B, int Tn, int K, int L,
                                                                  int accumulate)
{
    __shared__ float slots[4];
    __shared__ double dslots[4];
    const int l = blockIdx.x * 16 + (threadIdx.x & 15), k = blockIdx.y * 16 + (threadIdx.x >> 4);
    const bool ok = k < K && l < L;
    const int blk = blockIdx.y * gridDim.x + blockIdx.x;
    float total = 0.f;
    for (int b = 0; b < B; ++b) {
        float acc = 0.f;
        if (ok) {
            const T *px = x + (int64_t)b * Tn * K + k, *pg = g + (int64_t)b * Tn * L + l;
            for (int t = 0; t < Tn; ++t)
                acc = fmaf(load_elem<T>(px, (int64_t)t * K), load_elem<T>(pg, (int64_t)t * L), acc);
        }
        total += acc;
        const float ssq = block_sum(acc * acc, slots);
        if (threadIdx.x == 0) blk_s[(int64_t)b * (gridDim.x * gridDim.y) + blk] = ssq;
    }
    double bsq = 0.0;
    if (ok) {
        float *p = w + (int64_t)k * L + l;
        if (accumulate) total += *p;
        *p = total;
        bsq = (double)total * (double)total;
    }
    bsq = block_sum_f64(bsq, dslots);
    if (threadIdx.x == 0) blk_big[blk] = bsq;
}

// w = (accumulate ? w : 0) + sum over splits, in split order; per-block parts of ||w||^2.
__global__ __launch_bounds__(256) void linear_sum_splits_kernel(const float *part, float *w, double *blk_big,
                                                                int64_t n, int nsplit, int accumulate)
{
    __shared__ double dslots[4];
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double bsq = 0.0;
    if (i < n) {
        float v = accumulate ? w[i] : 0.f;
        for (int s = 0; s < nsplit; ++s) v += part[(int64_t)s * n + i];
        w[i] = v;
        bsq = (double)v * (double)v;
    }
    bsq = block_sum_f64(bsq, dslots);
    if (threadIdx.x == 0) blk_big[blockIdx.x] = bsq;
}

// s[b] = sum of its parts, big_sq = sum of the parts of ||w'||^2; fp64, in an order fixed by the launch
// shape alone (thread p % 1024 takes parts p, p + 1024, ...; then the fixed-order block sum).
// Workgroup b serves example b; workgroup B serves big_sq.
__global__ __launch_bounds__(1024) void linear_final_kernel(const float *part_s, int nparts, const double *part_big,
                                                            int64_t nbig, float *s, float *big_sq, int B)
{
    __shared__ double slots[16];
    const int b = blockIdx.x;
    double t = 0.0;
    if (b < B) {
        for (int p = threadIdx.x; p < nparts; p += 1024) t += (double)part_s[(int64_t)b * nparts + p];
        t = block_sum_f64(t, slots);
        if (threadIdx.x == 0) s[b] = (float)t;
    } else if (big_sq) {
        for (int64_t i = threadIdx.x; i < nbig; i += 1024) t += part_big[i];
        t = block_sum_f64(t, slots);
        if (threadIdx.x == 0) big_sq[0] = (float)t;
    }
}

struct LinPlan {
    bool mfma;
    int tiles_k, tiles_l, nsplit, b_per_split;
    int nparts;            // rows of the s parts
    int64_t nbig;          // entries of the ||w'||^2 parts
    size_t off_s, off_big, off_part, bytes;
};

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

LinPlan make_lin_plan(int B, int T, int K, int L, int dt, bool aligned)
{
    LinPlan p{};
    p.mfma = dt == LNPEGN_BF16 && K % 8 == 0 && L % 8 == 0 && aligned;
    if (p.mfma) {
        p.tiles_k = (K + kTileK - 1) / kTileK;
        p.tiles_l = (L + kTileL - 1) / kTileL;
        const int ntiles = p.tiles_k * p.tiles_l;
        // enough workgroups for 256 CUs: split the examples when the output has few tiles
        int want = (256 + ntiles - 1) / ntiles;
        if (want > B) want = B;
        if (want > kMaxSplit) want = kMaxSplit;
        p.b_per_split = (B + want - 1) / want;
        p.nsplit = (B + p.b_per_split - 1) / p.b_per_split;
        p.nparts = ntiles * kWaves;
        p.nbig = p.nsplit == 1 ? (int64_t)ntiles * kWaves : ((int64_t)K * L + 255) / 256;
    } else {
        p.tiles_k = (K + 15) / 16;
        p.tiles_l = (L + 15) / 16;
        p.nsplit = 1;
        p.b_per_split = B;
        p.nparts = p.tiles_k * p.tiles_l;
        p.nbig = p.nparts;
    }
    p.off_s = 0;
    p.off_big = align256(p.off_s + (size_t)p.nparts * B * sizeof(float));
    p.off_part = align256(p.off_big + (size_t)p.nbig * sizeof(double));
    p.bytes = p.off_part + (p.nsplit > 1 ? (size_t)p.nsplit * K * L * sizeof(float) : 0);
    return p;
}

bool lin_shape_ok(int B, int T, int K, int L)
{
    return B > 0 && T > 0 && K > 0 && L > 0 && (int64_t)K * L <= ((int64_t)1 << 31);
}

}  // namespace
}  // namespace lnpegn

using namespace lnpegn;

extern "C" {

size_t linear_pegn_workspace_bytes(int B, int T, int K, int L, lnpegn_dtype dt)
{
    if (!lin_shape_ok(B, T, K, L) || (dt != LNPEGN_F32 && dt != LNPEGN_BF16)) return 0;
    // sized for either kernel, whatever the alignment of the pointers turns out to be
    const size_t m = make_lin_plan(B, T, K, L, dt, true).bytes, g = make_lin_plan(B, T, K, L, dt, false).bytes;
    return m > g ? m : g;
}

int linear_pegn(const void *x, const void *g, float *w, float *s, float *big_sq, int B, int T, int K, int L,
                lnpegn_dtype dt, void *workspace, size_t workspace_bytes, unsigned flags, void *stream)
{
    if (!lin_shape_ok(B, T, K, L) || !x || !g || !w || !s || !workspace) return LNPEGN_EINVAL;
    if (flags & ~(unsigned)LNPEGN_ACCUMULATE) return LNPEGN_EINVAL;
    if (dt != LNPEGN_F32 && dt != LNPEGN_BF16) return LNPEGN_EUNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return LNPEGN_EINVAL;
    const bool aligned = ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(g)) & 15u) == 0;
    const LinPlan p = make_lin_plan(B, T, K, L, dt, aligned);
    if (workspace_bytes < p.bytes) return LNPEGN_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int accumulate = (flags & LNPEGN_ACCUMULATE) ? 1 : 0;
    char *ws = static_cast<char *>(workspace);
    float *part_s = reinterpret_cast<float *>(ws + p.off_s);
    double *part_big = reinterpret_cast<double *>(ws + p.off_big);
    float *part_w = reinterpret_cast<float *>(ws + p.off_part);
    if (p.mfma) {
        LinArgs a{};
        a.x = static_cast<const uint16_t *>(x);
        a.g = static_cast<const uint16_t *>(g);
        a.out = p.nsplit > 1 ? part_w : w;
        a.tile_s = part_s;
        a.tile_big = part_big;
        a.B = B; a.T = T; a.K = K; a.L = L;
        a.tiles_k = p.tiles_k; a.tiles_l = p.tiles_l; a.nsplit = p.nsplit; a.b_per_split = p.b_per_split;
        a.accumulate = accumulate;
        linear_pegn_kernel<<<dim3(p.tiles_k * p.tiles_l, p.nsplit), dim3(kThreads), 0, st>>>(a);
        if (hipGetLastError() != hipSuccess) return LNPEGN_EHIP;
        if (p.nsplit > 1) {
            const int64_t n = (int64_t)K * L;
            linear_sum_splits_kernel<<<dim3((unsigned)p.nbig), dim3(256), 0, st>>>(part_w, w, part_big, n, p.nsplit,
                                                                                  accumulate);
            if (hipGetLastError() != hipSuccess) return LNPEGN_EHIP;
        }
    } else {
        const dim3 grid(p.tiles_l, p.tiles_k);
        if (dt == LNPEGN_BF16)
            linear_pegn_generic_kernel<bf16_t><<<grid, dim3(256), 0, st>>>(
                static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(g), w, part_s, part_big, B, T, K, L,
                accumulate);
        else
            linear_pegn_generic_kernel<float><<<grid, dim3(256), 0, st>>>(
                static_cast<const float *>(x), static_cast<const float *>(g), w, part_s, part_big, B, T, K, L,
                accumulate);
        if (hipGetLastError() != hipSuccess) return LNPEGN_EHIP;
    }
    linear_final_kernel<<<dim3(B + 1), dim3(1024), 0, st>>>(part_s, p.nparts, part_big, p.nbig, s, big_sq, B);
    return hipGetLastError() == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

}  // extern "C"
