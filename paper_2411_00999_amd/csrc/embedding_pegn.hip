// Embedding-layer simultaneous per-example gradient norms (Appendix B, embedding-layer algorithm) for gfx950:
//   w_b[v,d] = sum_{t: ids[b,t] = v} g[b,t,d]     (steps 1-2; the one-hot tensor and [B,V,D] are never formed)
//   s[b]     = sum_{v,d} w_b[v,d]^2               (step 3)
//   w'[v,d]  = sum_b w_b[v,d]                     (step 4)
// The positions p = b*T + t are sorted by id (stable, so positions ascend inside an id and the rows of one
// example are adjacent): a "run" is the rows of one id in one example, a "segment" all runs of one id.
// Kernel A gives every run to a wave (columns spread over its lanes): the run's sum, squared, is that
// example's share of step 3; if the run is the id's only one it is also the row of w'.  Otherwise the sum is
// parked in the workspace and kernel B adds an id's parked sums in example order (at most B of them).
// Every row of g is read once, an id that fills half the batch still costs no wave more than one example's
// worth of rows, and nothing is atomic: results are bitwise reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstring>
#include <rocprim/device/device_radix_sort.hpp>

#include "../../include/lnpegn.h"
#include "lnpegn_device.h"

namespace lnpegn {
namespace {

constexpr int kColBlock = 512;      // columns per wave: 8 per lane
constexpr int kChunk = 8;           // sorted positions whose segment heads one wave looks after
constexpr int kWavesPerBlock = 4;
constexpr int kNormBlocks = 1024;   // workgroups of the ||w'||^2 pass in accumulate mode

__global__ __launch_bounds__(256) void emb_prepare_kernel(const void *ids, int ids_i64, uint32_t *keys,
                                                          uint32_t *vals, float *scratch, int64_t n,
                                                          int64_t nscratch, int V)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) {
        const int64_t id = ids_i64 ? static_cast<const int64_t *>(ids)[i] : (int64_t) static_cast<const int32_t *>(ids)[i];
        keys[i] = (id >= 0 && id < V) ? (uint32_t)id : (uint32_t)V;    // out of range: sorted behind, skipped
        vals[i] = (uint32_t)i;
    }
    for (int64_t j = i; j < nscratch; j += (int64_t)gridDim.x * 256) scratch[j] = 0.f;
}

__global__ __launch_bounds__(256) void emb_fill_kernel(float *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0.f;
}

// eight columns of one row, added into sub: 16-byte loads when the row allows, element loads otherwise
__device__ __forceinline__ void add_row(const bf16_t *g, int64_t p, int D, int c0, bool vec, float (&sub)[8])
{
    const bf16_t *row = g + p * D + c0;
    if (vec) {
        const uint4 r = *reinterpret_cast<const uint4 *>(row);
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sub[2 * i] += __builtin_bit_cast(float, w[i] << 16);
            sub[2 * i + 1] += __builtin_bit_cast(float, w[i] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (c0 + i < D) sub[i] += load_elem<bf16_t>(row, i);
    }
}

// the same eight columns as raw 16-byte loads, for callers that want several rows in flight
template <typename T>
struct Row8;
template <>
struct Row8<bf16_t> {
    uint4 a;
};
template <>
struct Row8<float> {
    float4 a, b;
};
__device__ __forceinline__ Row8<bf16_t> load_row8(const bf16_t *g, int64_t p, int D, int c0)
{
    return Row8<bf16_t>{*reinterpret_cast<const uint4 *>(g + p * D + c0)};
}
__device__ __forceinline__ Row8<float> load_row8(const float *g, int64_t p, int D, int c0)
{
    const float *row = g + p * D + c0;
    return Row8<float>{*reinterpret_cast<const float4 *>(row), *reinterpret_cast<const float4 *>(row + 4)};
}
__device__ __forceinline__ void unpack_row8(const Row8<bf16_t> &r, float (&f)[8])
{
    const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __builtin_bit_cast(float, w[i] << 16);
        f[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void unpack_row8(const Row8<float> &r, float (&f)[8])
{
    f[0] = r.a.x; f[1] = r.a.y; f[2] = r.a.z; f[3] = r.a.w;
    f[4] = r.b.x; f[5] = r.b.y; f[6] = r.b.z; f[7] = r.b.w;
}

__device__ __forceinline__ void add_row(const float *g, int64_t p, int D, int c0, bool vec, float (&sub)[8])
{
    const float *row = g + p * D + c0;
    if (vec) {
        const float4 lo = *reinterpret_cast<const float4 *>(row), hi = *reinterpret_cast<const float4 *>(row + 4);
        sub[0] += lo.x; sub[1] += lo.y; sub[2] += lo.z; sub[3] += lo.w;
        sub[4] += hi.x; sub[5] += hi.y; sub[6] += hi.z; sub[7] += hi.w;
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (c0 + i < D) sub[i] += row[i];
    }
}

// eight fp32 columns of a row: out[k] = (add ? row[k] : 0) + in[k], stored; returns the sum of squares
__device__ __forceinline__ float put_row(float *row, const float (&in)[8], int c0, int D, bool add)
{
    float sq = 0.f;
    if (c0 + 8 <= D && (reinterpret_cast<uintptr_t>(row) & 15u) == 0) {
        float4 lo = make_float4(in[0], in[1], in[2], in[3]), hi = make_float4(in[4], in[5], in[6], in[7]);
        if (add) {
            const float4 a = *reinterpret_cast<const float4 *>(row), b = *reinterpret_cast<const float4 *>(row + 4);
            lo.x += a.x; lo.y += a.y; lo.z += a.z; lo.w += a.w;
            hi.x += b.x; hi.y += b.y; hi.z += b.z; hi.w += b.w;
        }
        *reinterpret_cast<float4 *>(row) = lo;
        *reinterpret_cast<float4 *>(row + 4) = hi;
        sq = lo.x * lo.x + lo.y * lo.y + lo.z * lo.z + lo.w * lo.w + hi.x * hi.x + hi.y * hi.y + hi.z * hi.z + hi.w * hi.w;
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (c0 + k < D) {
                const float v = add ? row[k] + in[k] : in[k];
                row[k] = v;
                sq = fmaf(v, v, sq);
            }
    }
    return sq;
}

__device__ __forceinline__ uint32_t lane_value(uint32_t v, int lane)      // lane is wave-uniform
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

// One window of the sorted list: lane l looks at sorted position i + l.  Returns how many of the leading
// positions satisfy same(key, example), 0..64, and leaves each lane's position value in val.
struct Window {
    uint32_t key, val, ex;
};
__device__ __forceinline__ Window window_at(const uint32_t *keys, const uint32_t *vals, int64_t i, int64_t n,
                                             int Tn, int lane)
{
    Window w;
    const bool in = i + lane < n;
    w.key = in ? keys[i + lane] : 0xffffffffu;
    w.val = in ? vals[i + lane] : 0u;
    w.ex = w.val / (uint32_t)Tn;
    return w;
}
__device__ __forceinline__ int leading(bool pred)
{
    const uint64_t not_pred = ~__ballot(pred);
    return not_pred ? __builtin_ctzll(not_pred) : 64;
}

// Kernel A.  keys/vals: positions sorted by id.  A wave looks after the runs whose first row is among its
// kChunk sorted positions, and streams their rows eight at a time in sorted order, closing a run wherever
// the next position starts another.  contrib [ncb][n]: the run's share of s[b], stored at the run's first
// position, zero elsewhere.  runsum [n][D]: the sums of runs that are not their id's only run, at the same
// index.  bigpart [ncb][n]: squared norm of a finished row of w', at the segment's first position (not
// when accumulating).
template <typename T>
__global__ __launch_bounds__(64 * kWavesPerBlock) void emb_runs_kernel(
    const T *g, const uint32_t *keys, const uint32_t *vals, float *w, float *runsum, float *contrib, float *bigpart,
    int64_t n, int Tn, int D, int V, int accumulate, int vec_ok)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // the waves of a workgroup take the same positions and neighbouring column blocks: a row of g is then
    // read whole by one workgroup at one time
    const int64_t i0 = (int64_t)blockIdx.x * kChunk;
    const int cb = blockIdx.y * kWavesPerBlock + wave, c0 = cb * kColBlock + lane * 8;
    if (i0 >= n || cb * kColBlock >= D) return;
    const bool has_cols = c0 < D;
    const bool vec = vec_ok && c0 + 8 <= D;
    float sub[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) sub[k] = 0.f;
    bool in_run = false;                 // a run of this wave is open (its sum so far is in sub)
    uint32_t cur_first = 0, cur_key = 0;
    bool cur_seg_head = false;
    int64_t pos = i0;                    // next sorted position to look at
    while (true) {
        // lane l looks at sorted position pos - 1 + l: lane 0 is the position before, lanes 1..62 are
        // handled in this round, lane 63 is only looked at as "what follows lane 62"
        const int64_t q = pos - 1 + lane;
        const bool in = q >= 0 && q < n;
        const uint32_t key = in ? keys[q] : 0xffffffffu, val = in ? vals[q] : 0u;
        const uint32_t ex = val / (uint32_t)Tn;
        const uint32_t pkey = (uint32_t)__shfl_up((int)key, 1), pex = (uint32_t)__shfl_up((int)ex, 1);
        const bool valid = key < (uint32_t)V;
        const uint64_t m_valid = __ballot(valid);
        const uint64_t m_head = __ballot(valid && lane >= 1 && (key != pkey || ex != pex));     // starts a run
        const uint64_t m_seg = __ballot(valid && lane >= 1 && key != pkey);                     // starts a segment
        // the lanes this wave handles now: from the first run head of its chunk (or lane 1 if a run is
        // open) up to the lane before the first head that belongs to a later chunk, an invalid key, or 63
        const int64_t chunk_end = i0 + kChunk;
        int l = 1;
        if (!in_run) {
            const uint64_t h = m_head & ~(uint64_t)1;
            if (!h) {
                // no run starts in this round; rows seen belong to a run of an earlier chunk
                if (!(m_valid >> 62 & 1) || pos - 1 + 62 >= chunk_end) return;
                pos += 62;
                continue;
            }
            l = __builtin_ctzll(h);
            if (pos - 1 + l >= chunk_end) return;
        }
        // end: first lane >= l that is invalid, or a head at a position >= chunk_end
        int e = l;
        while (e <= 62) {
            if (!(m_valid >> e & 1)) break;
            if ((m_head >> e & 1) && pos - 1 + e >= chunk_end) break;
            ++e;
        }
        // rows l .. e-1, eight in flight: the loads carry no condition (a row past the end repeats the last
        // one and is dropped afterwards), so that all eight are issued before the first is waited for
        for (int r = l; r < e; r += 8) {
            float part[8][8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int k = 0; k < 8; ++k) part[u][k] = 0.f;
            if (vec) {                                           // lanes whose eight columns are a whole vector
                Row8<T> raw[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int t = r + u < e ? r + u : e - 1;
                    raw[u] = load_row8(g, (int64_t)lane_value(val, t), D, c0);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) unpack_row8(raw[u], part[u]);
            } else if (has_cols) {                               // ragged or unaligned columns: element loads
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (r + u < e) add_row(g, (int64_t)lane_value(val, r + u), D, c0, false, part[u]);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = r + u;
                if (t >= e) break;
                if (m_head >> t & 1) {                           // this row opens a run
                    in_run = true;
                    cur_first = lane_value(val, t);
                    cur_key = lane_value(key, t);
                    cur_seg_head = (m_seg >> t & 1) != 0;
#pragma unroll
                    for (int k = 0; k < 8; ++k) sub[k] = 0.f;
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) sub[k] += part[u][k];
                // the run ends here if the next position is invalid or opens another run; lane 63's
                // successor is unknown, which is why lane 62 is the last one handled in a round
                const bool next_valid = (m_valid >> (t + 1) & 1) != 0;
                if (next_valid && !(m_head >> (t + 1) & 1)) continue;
                const uint32_t next_key = next_valid ? lane_value(key, t + 1) : 0xffffffffu;
                float sq = 0.f;
#pragma unroll
                for (int k = 0; k < 8; ++k) sq = fmaf(sub[k], sub[k], sq);
                sq = wave_sum(sq);
                if (lane == 0) contrib[(int64_t)cb * n + cur_first] = sq;
                if (cur_seg_head && next_key != cur_key) {      // the id's only run: this is the row of w'
                    float wsq = has_cols ? put_row(w + (int64_t)cur_key * D + c0, sub, c0, D, accumulate != 0) : 0.f;
                    if (!accumulate) {
                        wsq = wave_sum(wsq);
                        if (lane == 0) bigpart[(int64_t)cb * n + cur_first] = wsq;
                    }
                } else if (has_cols) {
                    put_row(runsum + (int64_t)cur_first * D + c0, sub, c0, D, false);
                }
                in_run = false;
            }
        }
        if (e <= 62) return;              // stopped at an invalid key or at a later chunk's run
        pos += 62;                        // lane 62 was the last handled: it becomes lane 0 of the next round
    }
}

// Kernel B.  A wave looks after the segments (ids) whose first row is among its kChunk sorted positions and
// that have more than one run: the row of w' is the sum of the runs' parked sums, in example order.
__global__ __launch_bounds__(64 * kWavesPerBlock) void emb_ids_kernel(
    const uint32_t *keys, const uint32_t *vals, float *w, const float *runsum, float *bigpart, int64_t n, int Tn,
    int D, int V, int accumulate)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t i0 = (int64_t)blockIdx.x * kChunk;
    const int cb = blockIdx.y * kWavesPerBlock + wave, c0 = cb * kColBlock + lane * 8;
    if (cb * kColBlock >= D) return;
    const bool has_cols = c0 < D;
    const bool runsum_vec = c0 + 8 <= D && D % 4 == 0 && (reinterpret_cast<uintptr_t>(runsum) & 15u) == 0;
    for (int64_t i = i0; i < i0 + kChunk && i < n; ++i) {
        const uint32_t v = keys[i];
        if (v >= (uint32_t)V) break;
        if (i > 0 && keys[i - 1] == v) continue;                // not the head of a segment
        float tot[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) tot[k] = 0.f;
        // first the number of runs (positions only); an id with one run was finished by kernel A
        int runs = 0;
        for (int pass = 0; pass < 2; ++pass) {
            if (pass == 1 && runs < 2) break;
            int64_t j = i;
            uint32_t prev_ex = 0xffffffffu;                      // example of the position before the window
            int len;
            do {
                const Window win = window_at(keys, vals, j, n, Tn, lane);
                len = leading(win.key == v);
                // a position heads a run if the one before it belongs to another example
                uint32_t before = (uint32_t)__shfl_up((int)win.ex, 1);
                if (lane == 0) before = prev_ex;
                uint64_t heads = __ballot(lane < len && win.ex != before);
                if (pass == 0) {
                    runs += __popcll(heads);
                } else {
                    while (heads) {                              // parked sums, in example order
                        const int r = __builtin_ctzll(heads);
                        heads &= heads - 1;
                        if (has_cols) add_row(runsum, (int64_t)lane_value(win.val, r), D, c0, runsum_vec, tot);
                    }
                }
                if (len > 0) prev_ex = lane_value(win.ex, len - 1);
                j += len;
            } while (len == 64);
        }
        if (runs < 2) continue;
        float wsq = has_cols ? put_row(w + (int64_t)v * D + c0, tot, c0, D, accumulate != 0) : 0.f;
        if (!accumulate) {
            wsq = wave_sum(wsq);
            if (lane == 0) bigpart[(int64_t)cb * n + vals[i]] = wsq;
        }
    }
}

// partial sums of squares of w (accumulate mode: every row counts, not only those touched)
__global__ __launch_bounds__(256) void emb_wnorm_kernel(const float *w, int64_t n, double *part)
{
    __shared__ double slots[4];
    double t = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        t += (double)w[i] * (double)w[i];
    t = block_sum_f64(t, slots);
    if (threadIdx.x == 0) part[blockIdx.x] = t;
}

// s[b] = sum over column blocks and positions of example b of contrib; big_sq from its parts.  fp64, fixed order.
__global__ __launch_bounds__(1024) void emb_final_kernel(const float *contrib, const float *bigpart,
                                                         const double *wpart, int nwpart, float *s, float *big_sq,
                                                         int B, int Tn, int ncb, int64_t n)
{
    __shared__ double slots[16];
    const int b = blockIdx.x;
    double t = 0.0;
    if (b < B) {
        for (int c = 0; c < ncb; ++c)
            for (int i = threadIdx.x; i < Tn; i += 1024) t += (double)contrib[(int64_t)c * n + (int64_t)b * Tn + i];
        t = block_sum_f64(t, slots);
        if (threadIdx.x == 0) s[b] = (float)t;
    } else if (big_sq) {
        if (wpart) {
            for (int i = threadIdx.x; i < nwpart; i += 1024) t += wpart[i];
        } else {
            double t1 = 0.0, t2 = 0.0, t3 = 0.0;               // four loads in flight; the order stays fixed
            const int64_t m = (int64_t)ncb * n;
            int64_t i = threadIdx.x;
            for (; i + 3072 < m; i += 4096) {
                t += (double)bigpart[i];
                t1 += (double)bigpart[i + 1024];
                t2 += (double)bigpart[i + 2048];
                t3 += (double)bigpart[i + 3072];
            }
            for (; i < m; i += 1024) t += (double)bigpart[i];
            t = (t + t1) + (t2 + t3);
        }
        t = block_sum_f64(t, slots);
        if (threadIdx.x == 0) big_sq[0] = (float)t;
    }
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int key_bits(int V)
{
    int bits = 1;
    while (bits < 32 && ((uint64_t)1 << bits) <= (uint64_t)V) ++bits;   // keys run up to V inclusive
    return bits;
}

struct EmbPlan {
    int64_t n;
    int ncb;
    size_t off_keys_in, off_keys_out, off_vals_in, off_vals_out, off_contrib, off_bigpart, off_wpart, off_temp, off_runsum;
    size_t temp_bytes, bytes;
};

bool emb_shape_ok(int B, int T, int D, int V)
{
    return B > 0 && T > 0 && D > 0 && V > 0 && (int64_t)B * T < ((int64_t)1 << 31) && V < (1 << 30);
}

// The sort's own temporary storage is sized by the library for the current device.
hipError_t make_emb_plan(int B, int T, int D, int V, EmbPlan &p)
{
    p.n = (int64_t)B * T;
    p.ncb = (D + kColBlock - 1) / kColBlock;
    size_t temp = 0;
    const hipError_t e = rocprim::radix_sort_pairs(nullptr, temp, (const uint32_t *)nullptr, (uint32_t *)nullptr,
                                                   (const uint32_t *)nullptr, (uint32_t *)nullptr, (size_t)p.n, 0,
                                                   key_bits(V), (hipStream_t)0);
    if (e != hipSuccess) return e;
    const size_t arr = align256((size_t)p.n * sizeof(uint32_t)), f = align256((size_t)p.ncb * p.n * sizeof(float));
    p.off_keys_in = 0;
    p.off_keys_out = p.off_keys_in + arr;
    p.off_vals_in = p.off_keys_out + arr;
    p.off_vals_out = p.off_vals_in + arr;
    p.off_contrib = p.off_vals_out + arr;
    p.off_bigpart = p.off_contrib + f;            // directly behind contrib: one fill clears both
    p.off_wpart = p.off_bigpart + f;
    p.off_temp = p.off_wpart + align256(kNormBlocks * sizeof(double));
    p.temp_bytes = temp;
    p.off_runsum = p.off_temp + align256(temp);
    p.bytes = p.off_runsum + align256((size_t)p.n * D * sizeof(float));
    return hipSuccess;
}

}  // namespace
}  // namespace lnpegn

using namespace lnpegn;

extern "C" {

size_t embedding_pegn_workspace_bytes(int B, int T, int D, int V)
{
    if (!emb_shape_ok(B, T, D, V)) return 0;
    EmbPlan p;
    return make_emb_plan(B, T, D, V, p) == hipSuccess ? p.bytes : 0;
}

int embedding_pegn(const void *ids, int ids_are_int64, const void *g, float *w, float *s, float *big_sq, int B, int T,
                   int D, int V, lnpegn_dtype dt, void *workspace, size_t workspace_bytes, unsigned flags, void *stream)
{
    if (!emb_shape_ok(B, T, D, V) || !ids || !g || !w || !s || !workspace) return LNPEGN_EINVAL;
    if (flags & ~(unsigned)LNPEGN_ACCUMULATE) return LNPEGN_EINVAL;
    if (dt != LNPEGN_F32 && dt != LNPEGN_BF16) return LNPEGN_EUNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return LNPEGN_EINVAL;
    EmbPlan p;
    if (make_emb_plan(B, T, D, V, p) != hipSuccess) return LNPEGN_EHIP;
    if (workspace_bytes < p.bytes) return LNPEGN_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int accumulate = (flags & LNPEGN_ACCUMULATE) ? 1 : 0;
    char *ws = static_cast<char *>(workspace);
    uint32_t *keys_in = reinterpret_cast<uint32_t *>(ws + p.off_keys_in);
    uint32_t *keys_out = reinterpret_cast<uint32_t *>(ws + p.off_keys_out);
    uint32_t *vals_in = reinterpret_cast<uint32_t *>(ws + p.off_vals_in);
    uint32_t *vals_out = reinterpret_cast<uint32_t *>(ws + p.off_vals_out);
    float *contrib = reinterpret_cast<float *>(ws + p.off_contrib);
    float *bigpart = reinterpret_cast<float *>(ws + p.off_bigpart);
    double *wpart = reinterpret_cast<double *>(ws + p.off_wpart);
    const int64_t nscratch = (int64_t)((p.off_wpart - p.off_contrib) / sizeof(float));
    const unsigned nblk = (unsigned)((p.n + 255) / 256);
    emb_prepare_kernel<<<dim3(nblk), dim3(256), 0, st>>>(ids, ids_are_int64, keys_in, vals_in, contrib, p.n, nscratch, V);
    if (hipGetLastError() != hipSuccess) return LNPEGN_EHIP;
    size_t temp = p.temp_bytes;
    if (rocprim::radix_sort_pairs(ws + p.off_temp, temp, keys_in, keys_out, vals_in, vals_out, (size_t)p.n, 0,
                                  key_bits(V), st) != hipSuccess)
        return LNPEGN_EHIP;
    if (!accumulate) {
        const int64_t nw = (int64_t)V * D;
        const unsigned fb = (unsigned)(nw / 256 / 8 + 1 < 65536 ? nw / 256 / 8 + 1 : 65536);
        emb_fill_kernel<<<dim3(fb), dim3(256), 0, st>>>(w, nw);
        if (hipGetLastError() != hipSuccess) return LNPEGN_EHIP;
    }
    const int esz = dt == LNPEGN_BF16 ? 2 : 4;
    // 8 columns per lane: 16 bytes of bf16, 32 bytes of fp32; rows must keep that alignment
    const int vec_ok = ((reinterpret_cast<uintptr_t>(g) & 15u) == 0 && ((int64_t)D * esz) % 16 == 0) ? 1 : 0;
    const dim3 grid((unsigned)((p.n + kChunk - 1) / kChunk), (unsigned)((p.ncb + kWavesPerBlock - 1) / kWavesPerBlock));
    float *runsum = reinterpret_cast<float *>(ws + p.off_runsum);
    if (dt == LNPEGN_BF16)
        emb_runs_kernel<bf16_t><<<grid, dim3(64 * kWavesPerBlock), 0, st>>>(
            static_cast<const bf16_t *>(g), keys_out, vals_out, w, runsum, contrib, bigpart, p.n, T, D, V, accumulate,
            vec_ok);
    else
        emb_runs_kernel<float><<<grid, dim3(64 * kWavesPerBlock), 0, st>>>(
            static_cast<const float *>(g), keys_out, vals_out, w, runsum, contrib, bigpart, p.n, T, D, V, accumulate,
            vec_ok);
    if (hipGetLastError() != hipSuccess) return LNPEGN_EHIP;
    emb_ids_kernel<<<grid, dim3(64 * kWavesPerBlock), 0, st>>>(keys_out, vals_out, w, runsum, bigpart, p.n, T, D, V,
                                                              accumulate);
    if (hipGetLastError() != hipSuccess) return LNPEGN_EHIP;
    const bool wnorm = accumulate && big_sq;
    if (wnorm) {
        emb_wnorm_kernel<<<dim3(kNormBlocks), dim3(256), 0, st>>>(w, (int64_t)V * D, wpart);
        if (hipGetLastError() != hipSuccess) return LNPEGN_EHIP;
    }
    emb_final_kernel<<<dim3(B + 1), dim3(1024), 0, st>>>(contrib, bigpart, wnorm ? wpart : nullptr, kNormBlocks, s,
                                                         big_sq, B, T, p.ncb, p.n);
    return hipGetLastError() == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

}  // extern "C"
