// Second level of the two-level deterministic reduction: sums of the per-chunk column sums,
// the per-example squared norms (Appendix B steps 2 and 6), the batch gradients (steps 3
// and 7) and the gradient-noise-scale estimator (Section 2.1, Eq. 3-5).  Every sum runs in a
// fixed order, in fp64, so results do not depend on scheduling.  The levels are separate
// launches on purpose: a device-scope fence inside a kernel writes back and invalidates the
// whole L2 of an XCD on this part, which costs more than a launch.
#pragma once
#include "lnpegn_device.h"

namespace lnpegn {

constexpr int kTile = 256;  // columns per workgroup

struct ReduceArgs {
    const float *part;     // [n_slots][2][D] column sums per chunk
    float *grp;            // [G1][2][D] sums per group of chunks
    double *part_s;        // [n_ex][ntile][2] per-example squared norms per tile
    double *part_big;      // [ntile][2] squared norms of the batch gradients per tile
    float *dgamma;         // [D]
    float *dbeta;          // [D]
    float *pe_gamma_sq;    // [n_ex]
    float *pe_beta_sq;
    float *big_sq;         // [2] or null
    int n_slots;
    int gs;                // chunks per group (the last group may be short)
    int G1;                // number of groups
    int n_ex;              // examples whose squared norms are taken from their chunks' sums here (Appendix B
                           // steps 2, 6); 0 when there are none or the row kernel wrote them itself
    int ex_gs;             // chunks per example: example b owns chunks [b*ex_gs, (b+1)*ex_gs)
    int D;
    int ntile;
    int accumulate;        // dgamma, dbeta: add to what is there (gradient accumulation) instead of overwrite
};

// An example's chunks are also one of the groups (as many groups as examples, of as many chunks): one workgroup
// then serves as both, and level 1 takes n_ex workgroups per tile instead of n_ex + G1.
__host__ __device__ inline bool examples_are_groups(const ReduceArgs &a) { return a.n_ex == a.G1 && a.ex_gs == a.gs; }
__host__ __device__ inline int reduce_groups_count(const ReduceArgs &a)
{
    return examples_are_groups(a) ? a.n_ex : a.n_ex + a.G1;
}

// These kernels are a handful of dependent memory round trips long, so every level issues its
// loads in batches of eight before it adds them (in index order: the sums are reproducible).

// Level 1.  grid (ntile, reduce_groups_count), 256 threads: the column tiles of a run of chunks are neighbours in
// launch order, so that the 1 KiB pieces they read of the same chunk vectors are fetched together (with the tiles
// as the slow grid index the batched launch of the 48-layer step took 57 us instead of 35).  A workgroup adds
// the column sums of a run of consecutive chunks: the four waves split the run, add in chunk order, then the
// waves' partial sums are added in wave order.
// The first n_ex workgroups of a tile take one example each and leave the squares of its sums (their sums are
// not kept); the other G1 take one group of chunks each, for the batch gradients.  With a single group the group
// sums ARE the batch gradients and go straight to dgamma / dbeta.
__device__ __forceinline__ void reduce_groups_body(const ReduceArgs &a, int gx, int tile)
{
    __shared__ double wsum[4][8][kWave];   // [wave][array*4 + component][lane]
    __shared__ double slots[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col0 = tile * kTile;

    const bool example = gx < a.n_ex;
    const int g = example ? gx : gx - a.n_ex;
    const int run = example ? a.ex_gs : a.gs;
    const int m0 = g * run, m1 = min(m0 + run, a.n_slots);
    const int per = (m1 - m0 + 3) / 4;
    const int w0 = min(m0 + wave * per, m1), w1 = min(w0 + per, m1);
    const int c4 = col0 + lane * 4;            // this lane's four columns
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (c4 < a.D) {
        const int64_t stride = 2 * (int64_t)a.D;
        if ((a.D & 3) == 0) {                  // rows of the workspace are 16-byte aligned
            for (int m = w0; m < w1; m += 8) {
                float4 u[8], v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int mm = min(m + i, w1 - 1);
                    const float *p = a.part + mm * stride + c4;
                    u[i] = *reinterpret_cast<const float4 *>(p);
                    v[i] = *reinterpret_cast<const float4 *>(p + a.D);
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (m + i < w1) {
                        acc[0] += u[i].x; acc[1] += u[i].y; acc[2] += u[i].z; acc[3] += u[i].w;
                        acc[4] += v[i].x; acc[5] += v[i].y; acc[6] += v[i].z; acc[7] += v[i].w;
                    }
                }
            }
        } else {                               // any D: element by element
            const int nc = min(4, a.D - c4);
            for (int m = w0; m < w1; ++m) {
                const float *p = a.part + m * stride + c4;
                for (int i = 0; i < nc; ++i) {
                    acc[i] += p[i];
                    acc[4 + i] += p[a.D + i];
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) wsum[wave][i][lane] = acc[i];
    __syncthreads();
    // thread -> one column of the tile
    const int col = col0 + tid;
    const int src_lane = tid >> 2, comp = tid & 3;
    double v0 = 0.0, v1 = 0.0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        v0 += wsum[w][comp][src_lane];
        v1 += wsum[w][4 + comp][src_lane];
    }
    if (example) {
        // an example's gradient as fp32 values, their squares summed in fp64
        const float f0 = (float)v0, f1 = (float)v1;
        const double e0 = block_sum_f64(col < a.D ? (double)f0 * f0 : 0.0, slots[0]);
        const double e1 = block_sum_f64(col < a.D ? (double)f1 * f1 : 0.0, slots[1]);
        if (tid == 0) {
            a.part_s[((int64_t)g * a.ntile + tile) * 2] = e0;
            a.part_s[((int64_t)g * a.ntile + tile) * 2 + 1] = e1;
        }
        if (!examples_are_groups(a)) return;
    }
    const bool single = a.G1 == 1;
    if (single && a.accumulate && col < a.D) {   // on top of what dgamma / dbeta hold
        v0 += (double)a.dgamma[col];
        if (a.dbeta) v1 += (double)a.dbeta[col];
    }
    const float f0 = (float)v0, f1 = (float)v1;
    if (col < a.D) {
        if (single) {
            a.dgamma[col] = f0;
            if (a.dbeta) a.dbeta[col] = f1;
        } else {
            a.grp[((int64_t)g * 2) * a.D + col] = f0;
            a.grp[((int64_t)g * 2 + 1) * a.D + col] = f1;
        }
    }
    if (single) {
        // squares of the values as stored (fp32), summed in fp64
        const double q0 = block_sum_f64(col < a.D ? (double)f0 * f0 : 0.0, slots[0]);
        const double q1 = block_sum_f64(col < a.D ? (double)f1 * f1 : 0.0, slots[1]);
        if (tid == 0) {
            a.part_big[tile * 2] = q0;
            a.part_big[tile * 2 + 1] = q1;
        }
    }
}

__global__ __launch_bounds__(kTile) void reduce_groups_kernel(ReduceArgs a)
{
    reduce_groups_body(a, blockIdx.y, blockIdx.x);
}

// Sum over the groups for one column (Appendix B steps 3, 7), groups added in order.
__device__ __forceinline__ void sum_groups(const float *grp, int G1, int D, int col, double &s0,
                                           double &s1)
{
    const int64_t stride = 2 * (int64_t)D;
    s0 = s1 = 0.0;
    for (int g = 0; g < G1; g += 8) {
        float u[8], v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float *p = grp + min(g + i, G1 - 1) * stride + col;
            u[i] = p[0];
            v[i] = p[D];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (g + i < G1) {
                s0 += u[i];
                s1 += v[i];
            }
        }
    }
}

// Per-example and batch squared norms from their per-tile parts, tiles added in order.
__device__ __forceinline__ void finish_scalars(const ReduceArgs &a, int tid, int nthreads)
{
    for (int b = tid; b < a.n_ex; b += nthreads) {
        double sg = 0.0, sb = 0.0;
        for (int t = 0; t < a.ntile; ++t) {
            sg += a.part_s[((int64_t)b * a.ntile + t) * 2];
            sb += a.part_s[((int64_t)b * a.ntile + t) * 2 + 1];
        }
        a.pe_gamma_sq[b] = (float)sg;
        if (a.pe_beta_sq) a.pe_beta_sq[b] = (float)sb;
    }
}

// Levels 2 and 3 in ONE workgroup of 1024 threads: dgamma, dbeta, their squared norms, and the
// per-example squared norms.  Used alone when the group sums are small, and one workgroup per
// layer when many layers are finished at once.
__device__ __forceinline__ void reduce_final_body(const ReduceArgs &a)
{
    __shared__ double slots[2][16];
    const int tid = threadIdx.x;
    double q0 = 0.0, q1 = 0.0;
    if (a.G1 > 1) {
        for (int col = tid; col < a.D; col += 1024) {
            double s0, s1;
            sum_groups(a.grp, a.G1, a.D, col, s0, s1);
            if (a.accumulate) {
                s0 += (double)a.dgamma[col];
                if (a.dbeta) s1 += (double)a.dbeta[col];
            }
            const float f0 = (float)s0, f1 = (float)s1;
            a.dgamma[col] = f0;
            if (a.dbeta) a.dbeta[col] = f1;
            q0 += (double)f0 * f0;
            q1 += (double)f1 * f1;
        }
    }
    finish_scalars(a, tid, 1024);
    if (a.big_sq) {
        if (a.G1 > 1) {
            q0 = block_sum_f64(q0, slots[0]);
            q1 = block_sum_f64(q1, slots[1]);
        } else if (tid < 2) {   // level 1 already left the per-tile parts
            double t2 = 0.0;
            for (int t = 0; t < a.ntile; ++t) t2 += a.part_big[t * 2 + tid];
            if (tid == 0) q0 = t2;
            else q1 = t2;
        }
        if (tid == 0) a.big_sq[0] = (float)q0;
        if (tid == (a.G1 > 1 ? 0 : 1) && a.dbeta) a.big_sq[1] = (float)q1;   // one norm without beta
    }
}

__global__ __launch_bounds__(1024) void reduce_final_small_kernel(ReduceArgs a)
{
    reduce_final_body(a);
}

// Many layers at once (deferred reduction).  Every layer's workspace starts with a DeferHeader
// and has the same layout, because the layers have the same shape.
constexpr int kBatchMax = 64;
struct BatchArgs {
    char *ws[kBatchMax];
    int n;
    int D;
    int ntile;
    size_t off_grp, off_part_s, off_part_big, off_part;
};

__device__ __forceinline__ ReduceArgs batch_layer_args(const BatchArgs &b, int layer)
{
    char *ws = b.ws[layer];
    const DeferHeader h = *reinterpret_cast<const DeferHeader *>(ws);
    ReduceArgs a;
    a.part = reinterpret_cast<const float *>(ws + b.off_part);
    a.grp = reinterpret_cast<float *>(ws + b.off_grp);
    a.part_s = reinterpret_cast<double *>(ws + b.off_part_s);
    a.part_big = reinterpret_cast<double *>(ws + b.off_part_big);
    a.dgamma = h.dgamma; a.dbeta = h.dbeta;
    a.pe_gamma_sq = h.pe_gamma_sq; a.pe_beta_sq = h.pe_beta_sq; a.big_sq = h.big_sq;
    a.n_slots = h.n_slots; a.gs = h.gs; a.G1 = h.G1; a.n_ex = h.n_ex; a.ex_gs = h.ex_gs; a.D = b.D; a.ntile = b.ntile;
    a.accumulate = h.accumulate;
    return a;
}

// grid (ntile, most examples + groups of any layer, layers): workgroups beyond a layer's own count leave at once
__global__ __launch_bounds__(kTile) void reduce_groups_batch_kernel(BatchArgs b)
{
    const ReduceArgs a = batch_layer_args(b, blockIdx.z);
    if ((int)blockIdx.y >= reduce_groups_count(a)) return;
    reduce_groups_body(a, blockIdx.y, blockIdx.x);
}

// grid (layers)
__global__ __launch_bounds__(1024) void reduce_final_batch_kernel(BatchArgs b)
{
    const ReduceArgs a = batch_layer_args(b, blockIdx.x);
    if (a.G1 == 1 && a.n_ex == 0 && !a.big_sq) return;
    reduce_final_body(a);
}

// Level 2 for large shapes: grid ntile, 256 threads, one column per thread.
__global__ __launch_bounds__(kTile) void reduce_final_tiles_kernel(ReduceArgs a)
{
    __shared__ double slots[2][4];
    const int tid = threadIdx.x, tile = blockIdx.x;
    const int col = tile * kTile + tid;
    double s0 = 0.0, s1 = 0.0;
    if (col < a.D) {
        sum_groups(a.grp, a.G1, a.D, col, s0, s1);
        if (a.accumulate) {
            s0 += (double)a.dgamma[col];
            if (a.dbeta) s1 += (double)a.dbeta[col];
        }
        a.dgamma[col] = (float)s0;
        if (a.dbeta) a.dbeta[col] = (float)s1;
    }
    const double d0 = (double)(float)s0, d1 = (double)(float)s1;
    const double q0 = block_sum_f64(d0 * d0, slots[0]);
    const double q1 = block_sum_f64(d1 * d1, slots[1]);
    if (tid == 0) {
        a.part_big[tile * 2] = q0;
        a.part_big[tile * 2 + 1] = q1;
    }
}

// Level 3 for large shapes: one workgroup.
__global__ __launch_bounds__(256) void reduce_scalars_kernel(ReduceArgs a)
{
    const int tid = threadIdx.x;
    finish_scalars(a, tid, 256);
    if (a.big_sq && tid < (a.dbeta ? 2 : 1)) {
        double t2 = 0.0;
        for (int t = 0; t < a.ntile; ++t) t2 += a.part_big[t * 2 + tid];
        a.big_sq[tid] = (float)t2;
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
