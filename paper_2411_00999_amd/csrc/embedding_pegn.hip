// Embedding-layer simultaneous per-example gradient norms (Appendix B, embedding-layer algorithm) for gfx950:
//   w_b[v,d] = sum_{t: ids[b,t] = v} g[b,t,d]     (steps 1-2; the one-hot tensor and [B,V,D] are never formed)
//   s[b]     = sum_{v,d} w_b[v,d]^2               (step 3)
//   w'[v,d]  = sum_b w_b[v,d]                     (step 4)
// The positions p = b*T + t are sorted by id (stable, so positions ascend inside an id and the rows of one
// example are adjacent): a "segment" is all positions of one id, a "run" those of one id in one example, a
// "piece" at most kPiece consecutive sorted positions of one run (a run is cut wherever the sorted index is a
// multiple of kPiece).  Kernel A reads g, every row once.  An id with at most kShort positions is finished
// there by one wave (each run's share of step 3, the row of w').  A longer id is handed out piece by piece:
// a piece that is a whole run yields that run's share at once, the piece sums are parked in the workspace,
// and kernel B (two launches: per run, then per id) adds the parked sums in sorted order, finding them by
// binary search of the sorted list rather than by walking it.  No wave reads more than kChunk + kPiece rows
// however skewed the ids are, and nothing is atomic: results are bitwise reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstring>
#include <mutex>
#include <rocprim/device/device_radix_sort.hpp>

#include "../../include/lnpegn.h"
#include "lnpegn_device.h"

namespace lnpegn {
int g_emb_run_blocks = 4096;        // workgroups of kernel A per column group (each loops over its chunks)
namespace {

constexpr int kColBlock = 512;      // columns per wave: 8 per lane
constexpr int kChunk = 16;          // sorted positions whose piece heads one wave looks after
constexpr int kPiece = 32;          // longest piece; kChunk + kPiece + 1 lanes of one 64-lane window cover a wave's work
constexpr int kWavesPerBlock = 4;
constexpr int kNormBlocks = 2048;   // workgroups of the ||w'||^2 pass in accumulate mode

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

// ---------------------------------------------------------------------------------------
// Sort of the (id, position) pairs for batches of up to kSortTiles * kSortTile positions, in two launches.
// A pair travels as one 64-bit word, id in the upper half and position in the lower: the words are distinct, so
// any correct sort of them is the stable sort by id.  (1) Every workgroup sorts one tile of kSortTile words in LDS
// (bitonic network).  (2) The place of a word in the whole order is the number of words below it: its index in
// its own tile plus one binary search in each other tile; each thread places one word.
// ---------------------------------------------------------------------------------------
constexpr int kSortTile = 2048;
constexpr int kSortTiles = 64;
constexpr uint64_t kSortPad = ~(uint64_t)0;

constexpr int kSortThreads = kSortTile / 2;   // one compare-exchange per thread and stage

__global__ __launch_bounds__(kSortThreads) void emb_tile_sort_kernel(const void *ids, int ids_i64, int64_t n, int V,
                                                                     uint64_t *tiles, float *scratch, int64_t nscratch)
{
    __shared__ uint64_t a[kSortTile];
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int i = tid + h * kSortThreads;
        const int64_t p = base + i;
        uint64_t word = kSortPad;
        if (p < n) {
            const int64_t id = ids_i64 ? static_cast<const int64_t *>(ids)[p] : (int64_t) static_cast<const int32_t *>(ids)[p];
            const uint32_t key = (id >= 0 && id < V) ? (uint32_t)id : (uint32_t)V;   // out of range: sorted behind, skipped
            word = ((uint64_t)key << 32) | (uint32_t)p;
        }
        a[i] = word;
    }
    // the scratch arrays of the call are cleared here too (grid-stride), which saves a launch
    for (int64_t j = (int64_t)blockIdx.x * kSortThreads + tid; j < nscratch; j += (int64_t)gridDim.x * kSortThreads)
        scratch[j] = 0.f;
    for (int k = 2; k <= kSortTile; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            __syncthreads();
            const int lo = ((tid & ~(j - 1)) << 1) | (tid & (j - 1)), hi = lo + j;   // j is a power of two
            const uint64_t x = a[lo], y = a[hi];
            const bool ascending = (lo & k) == 0;
            if ((x > y) == ascending) {
                a[lo] = y;
                a[hi] = x;
            }
        }
    }
    __syncthreads();
    tiles[base + tid] = a[tid];
    tiles[base + tid + kSortThreads] = a[tid + kSortThreads];
}

// Each thread places one word: sixteen binary searches (one per other tile) advance together, step by step, so
// that sixteen independent loads are in flight instead of one chain of twelve dependent ones after another.
__global__ __launch_bounds__(256) void emb_rank_kernel(const uint64_t *tiles, int ntiles, int64_t n, int V,
                                                       uint32_t *sorted_ids, uint32_t *sorted_pos, uint8_t *present)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;     // index into the tiles array
    if (i >= (int64_t)ntiles * kSortTile) return;
    const uint64_t word = tiles[i];
    if (word == kSortPad) return;
    const int mine = (int)(i / kSortTile);
    int64_t rank = i - (int64_t)mine * kSortTile;
    constexpr int kGroup = 16;
    for (int t0 = 0; t0 < ntiles; t0 += kGroup) {
        const uint64_t *tile[kGroup];
        int pos[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int t = t0 + u < ntiles ? t0 + u : mine;          // a tile that does not exist: searched, not counted
            tile[u] = tiles + (int64_t)t * kSortTile;
            pos[u] = 0;
        }
        // words of each tile below `word` (the tiles are sorted, kSortTile long): branch-free lower bound
#pragma unroll
        for (int step = kSortTile / 2; step > 0; step >>= 1) {
#pragma unroll
            for (int u = 0; u < kGroup; ++u) pos[u] += tile[u][pos[u] + step - 1] < word ? step : 0;
        }
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const int below = pos[u] + (tile[u][pos[u]] < word ? 1 : 0);
            rank += (t0 + u < ntiles && t0 + u != mine) ? below : 0;
        }
    }
    const uint32_t key = (uint32_t)(word >> 32);
    sorted_ids[rank] = key;
    sorted_pos[rank] = (uint32_t)word;
    if (present && key < (uint32_t)V) present[key] = 1;
}

// present[v] = 1 for every id that occurs (out-of-range ids carry the key V and are left out).  Plain byte
// stores of the same value: the result does not depend on the order.  `present` was cleared by the launch before.
__global__ __launch_bounds__(256) void emb_mark_kernel(const uint32_t *keys, int64_t n, int V, uint8_t *present)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) {
        const uint32_t k = keys[i];
        if (k < (uint32_t)V) present[k] = 1;
    }
}

// Clears the scratch arrays of a call whose keys are already sorted (the sorting call's prepare kernel does it
// otherwise).
__global__ __launch_bounds__(256) void emb_clear_kernel(float *scratch, int64_t nscratch)
{
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < nscratch; j += (int64_t)gridDim.x * 256) scratch[j] = 0.f;
}

// Zero fill of the rows of w' that no id selects (the rows of ids that occur are written, whole, by the run and
// id kernels, so the fill and those kernels touch different rows and may run side by side).  Streaming stores:
// the zeros are not wanted in any cache (the rows read next are g's), and lines left dirty in the memory-side
// cache would be written back one by one under the reads that follow.
__global__ __launch_bounds__(256) void emb_fill_kernel(float *p, int64_t V, int D, const uint8_t *present)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t n = V * D;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if ((reinterpret_cast<uintptr_t>(p) & 15u) == 0 && D % 4 == 0) {
        typedef __attribute__((ext_vector_type(4))) float f32x4;
        f32x4 *p4 = reinterpret_cast<f32x4 *>(p);
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        const int d4 = D / 4;
        for (; i < n / 4; i += stride)
            if (!present[i / d4]) __builtin_nontemporal_store(zero, p4 + i);
        return;
    }
    for (; i < n; i += stride)
        if (!present[i / D]) p[i] = 0.f;
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
// stream: the row will not be read again soon (a row of w'): streaming stores, kept out of the caches
__device__ __forceinline__ float put_row(float *row, const float (&in)[8], int c0, int D, bool add, bool stream = false)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    float sq = 0.f;
    if (c0 + 8 <= D && (reinterpret_cast<uintptr_t>(row) & 15u) == 0) {
        float4 lo = make_float4(in[0], in[1], in[2], in[3]), hi = make_float4(in[4], in[5], in[6], in[7]);
        if (add) {
            const float4 a = *reinterpret_cast<const float4 *>(row), b = *reinterpret_cast<const float4 *>(row + 4);
            lo.x += a.x; lo.y += a.y; lo.z += a.z; lo.w += a.w;
            hi.x += b.x; hi.y += b.y; hi.z += b.z; hi.w += b.w;
        }
        if (stream) {
            __builtin_nontemporal_store(f32x4{lo.x, lo.y, lo.z, lo.w}, reinterpret_cast<f32x4 *>(row));
            __builtin_nontemporal_store(f32x4{hi.x, hi.y, hi.z, hi.w}, reinterpret_cast<f32x4 *>(row + 4));
        } else {
            *reinterpret_cast<float4 *>(row) = lo;
            *reinterpret_cast<float4 *>(row + 4) = hi;
        }
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

// element u (wave-uniform, known at run time) of an array that lives in registers: a switch, so that the array
// is never indexed by a variable (which would move it to scratch memory)
template <typename R>
__device__ __forceinline__ R pick_row(const R (&a)[16], int u)
{
    switch (u) {
        case 0: return a[0];   case 1: return a[1];   case 2: return a[2];   case 3: return a[3];
        case 4: return a[4];   case 5: return a[5];   case 6: return a[6];   case 7: return a[7];
        case 8: return a[8];   case 9: return a[9];   case 10: return a[10]; case 11: return a[11];
        case 12: return a[12]; case 13: return a[13]; case 14: return a[14]; default: return a[15];
    }
}
template <typename R>
__device__ __forceinline__ R pick_row(const R (&a)[8], int u)
{
    switch (u) {
        case 0: return a[0]; case 1: return a[1]; case 2: return a[2]; case 3: return a[3];
        case 4: return a[4]; case 5: return a[5]; case 6: return a[6]; default: return a[7];
    }
}
template <typename R>
__device__ __forceinline__ R pick_row(const R (&a)[1], int)
{
    return a[0];
}
template <int N>
__device__ __forceinline__ void pick_floats(const float (&a)[N][8], int u, float (&f)[8])
{
#pragma unroll
    for (int k = 0; k < 8; ++k) f[k] = a[0][k];
#pragma unroll
    for (int j = 1; j < N; ++j)
        if (u == j) {
#pragma unroll
            for (int k = 0; k < 8; ++k) f[k] = a[j][k];
        }
}

// Kernel A.  keys/vals: positions sorted by id.  Ownership: a short segment (at most kShort positions)
// belongs whole to the wave whose kChunk sorted positions hold its first one, and that wave finishes the id
// (every run's share of s[b], the row of w').  A longer segment is handed out piece by piece to the waves
// whose positions hold the pieces' first rows; a piece that is a whole run yields that run's share of s[b],
// every sum is parked (unless the piece is the id's only one) and the id is marked for kernel B.
// A wave sees kShort positions back (to tell whether a piece in its chunk belongs to a short segment that an
// earlier wave owns) and far enough ahead for anything that starts in its chunk; rows are streamed sixteen
// (fp32: eight) at a time.  contrib [ncb][n]: a run's share of s[b], at the run's first position, zero elsewhere.
// runsum [n][D]: parked sums, at the piece's first position.  multi [n]: set at the sorted index of the first
// position of a long id that has parked sums; multi_run [n]: of a run that has several pieces.
// bigpart [ncb][n]: squared norm of a finished row of w', at the segment's first position (not when
// accumulating).
constexpr int kShort = 12;
static_assert(kShort + kChunk + kPiece < 63 && kShort + kChunk + kShort < 63, "one 64-lane window must cover a wave's work");

// kVec: every lane that has columns has eight whole ones behind an aligned 16-byte boundary (D % 8 == 0 and
// aligned rows); rows are then fetched as vectors, sixteen bf16 rows or eight fp32 rows in flight.
template <typename T, bool kVec>
__global__ __launch_bounds__(64 * kWavesPerBlock) void emb_runs_kernel(
    const T *g, const uint32_t *keys, const uint32_t *vals, float *w, float *runsum, float *contrib, float *bigpart,
    uint32_t *multi, uint32_t *multi_run, int64_t n, int Tn, int D, int V, int accumulate)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // the waves of a workgroup take the same positions and neighbouring column blocks: a row of g is then
    // read whole by one workgroup at one time
    const int cb = blockIdx.y * kWavesPerBlock + wave, c0 = cb * kColBlock + lane * 8;
    if (cb * kColBlock >= D) return;
    const bool has_cols = c0 < D;
    const int c_load = has_cols ? c0 : 0;                        // lanes without columns fetch what lane 0 does
    constexpr int kRows = kVec && sizeof(T) == 2 ? 16 : 8;       // rows in flight
    // A workgroup takes chunks blockIdx.x, blockIdx.x + gridDim.x, ...; the next chunk's part of the sorted list
    // is fetched while this chunk's rows are on their way.
    // Lane l looks at sorted position i0 - kShort - 1 + l: lane 0 only serves as "the position before",
    // lanes kShort+1 .. kShort+kChunk are the chunk.
    const int64_t nchunks = (n + kChunk - 1) / kChunk;
    auto look = [&](int64_t chunk, uint32_t &k, uint32_t &p) {
        const int64_t q = chunk * kChunk - kShort - 1 + lane;
        const bool in = chunk < nchunks && q >= 0 && q < n;
        k = in ? keys[q] : 0xffffffffu;
        p = in ? vals[q] : 0u;
    };
    uint32_t key_next, val_next;
    look(blockIdx.x, key_next, val_next);
    for (int64_t chunk = blockIdx.x; chunk < nchunks; chunk += gridDim.x) {
    const int64_t i0 = chunk * kChunk;
    const int64_t q = i0 - kShort - 1 + lane;
    const uint32_t key = key_next, val = val_next;
    look(chunk + gridDim.x, key_next, val_next);
    const uint32_t ex = val / (uint32_t)Tn;
    const uint32_t pkey = (uint32_t)__shfl_up((int)key, 1), pex = (uint32_t)__shfl_up((int)ex, 1);
    const bool valid = key < (uint32_t)V;
    const uint64_t m_valid = __ballot(valid);
    const uint64_t m_head = __ballot(valid && lane >= 1 && (key != pkey || ex != pex));     // starts a run
    const uint64_t m_seg = __ballot(valid && lane >= 1 && key != pkey);                     // starts a segment
    const uint64_t m_piece = m_head | __ballot(valid && lane >= 1 && q % kPiece == 0);      // starts a piece
    // is this lane's segment long?  Its first position is the nearest segment head at or below the lane
    // (not in the window: it lies more than kShort back), its end the next segment head or invalid key
    // (not in the window: more than kShort ahead of anything this wave may own).
    const uint64_t upto = ((uint64_t)2 << lane) - 1;
    const uint64_t heads_below = m_seg & upto, ends_above = (m_seg | ~m_valid) & ~upto;
    const int seg_first = heads_below ? 63 - __builtin_clzll(heads_below) : -1;
    const int seg_end = ends_above ? __builtin_ctzll(ends_above) : 64;
    const uint64_t m_long = __ballot(valid && (seg_first < 0 || seg_end - seg_first > kShort));
    const uint64_t m_own = m_seg | (m_piece & m_long);                                      // starts something to own
    const uint64_t chunk_lanes = (((uint64_t)1 << kChunk) - 1) << (kShort + 1);
    if (!(m_own & chunk_lanes)) continue;                        // nothing starts here
    const int l = __builtin_ctzll(m_own & chunk_lanes);
    // rows l .. e-1: up to the first invalid key or the first thing that starts behind the chunk
    const uint64_t behind = ~(((uint64_t)2 << (kShort + kChunk)) - 1);
    const uint64_t stop = (~m_valid & ~(((uint64_t)2 << l) - 1)) | (m_own & behind);
    int e = stop ? __builtin_ctzll(stop) : 63;
    if (e > 63) e = 63;

    // What happens at a row, as masks over the lanes: the masks are shifted so that bit u is row r + u of the
    // batch in hand, and a batch in which nothing happens is plain additions.
    const uint64_t next_starts_run = (m_head | ~m_valid) >> 1, next_starts_seg = (m_seg | ~m_valid) >> 1;
    const uint64_t next_starts_piece = (m_piece | ~m_valid) >> 1;
    uint64_t b_opens_id = m_seg >> l;                                        // first row of an id
    uint64_t b_opens = ((m_long & m_piece) | (~m_long & m_head)) >> l;       // first row of a long id's piece, or of a run
    uint64_t b_run_head = m_head >> l;
    uint64_t b_short_run_ends = (~m_long & next_starts_run) >> l;            // last row of a short id's run
    uint64_t b_piece_ends = (m_long & next_starts_piece) >> l;               // last row of a long id's piece
    uint64_t b_run_ends = next_starts_run >> l, b_seg_ends = next_starts_seg >> l;

    float sub[8], tot[8];                // the open run or piece; the short id's runs so far
#pragma unroll
    for (int k = 0; k < 8; ++k) sub[k] = tot[k] = 0.f;
    uint32_t first = 0, cur_key = 0, first_idx = 0, id_first = 0;
    bool run_head = false, seg_head = false;
    // kRows rows in flight: the loads carry no condition (a row past the end repeats the last one and is
    // dropped afterwards), so that all are issued before the first is waited for
    for (int r = l; r < e; r += kRows) {
        Row8<T> raw[kVec ? kRows : 1];
        float part[kVec ? 1 : kRows][8];
        if constexpr (kVec) {
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const int t = r + u < e ? r + u : e - 1;
                raw[u] = load_row8(g, (int64_t)lane_value(val, t), D, c_load);
            }
        } else {                                                 // ragged or unaligned columns: element loads
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
#pragma unroll
                for (int k = 0; k < 8; ++k) part[u][k] = 0.f;
                if (has_cols && r + u < e) add_row(g, (int64_t)lane_value(val, r + u), D, c0, false, part[u]);
            }
        }
        auto row = [&](int u, float (&f)[8]) {
            if constexpr (kVec) {
                unpack_row8(raw[u], f);
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) f[k] = part[u][k];
            }
        };
        const int rows = e - r < kRows ? e - r : kRows;
        const uint32_t in_batch = (1u << rows) - 1u;
        if (!((uint32_t)(b_opens | b_short_run_ends | b_piece_ends) & in_batch)) {
#pragma unroll
            for (int u = 0; u < kRows; ++u)
                if (u < rows) {
                    float f[8];
                    row(u, f);
#pragma unroll
                    for (int k = 0; k < 8; ++k) sub[k] += f[k];
                }
            b_opens_id >>= kRows; b_opens >>= kRows; b_run_head >>= kRows; b_short_run_ends >>= kRows;
            b_piece_ends >>= kRows; b_run_ends >>= kRows; b_seg_ends >>= kRows;
            continue;
        }
        // Something opens or closes in this batch: one row at a time, in a loop that is not unrolled (its body,
        // sixteen times over, would not fit the instruction cache); bit 0 of every mask is the row in hand.
#pragma nounroll
        for (int u = 0; u < rows; ++u) {
            const int t = r + u;
            float f[8];
            if constexpr (kVec) {
                unpack_row8(pick_row(raw, u), f);
            } else {
                pick_floats(part, u, f);
            }
            if (b_opens_id & 1) {                                // this row opens an id
                id_first = lane_value(val, t);
#pragma unroll
                for (int k = 0; k < 8; ++k) tot[k] = 0.f;
            }
            if (b_opens & 1) {                                   // ... a piece of a long id, or a run
                first = lane_value(val, t);
                first_idx = (uint32_t)(i0 - kShort - 1 + t);
                cur_key = lane_value(key, t);
                run_head = (b_run_head & 1) != 0;
                seg_head = (b_opens_id & 1) != 0;
#pragma unroll
                for (int k = 0; k < 8; ++k) sub[k] = 0.f;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) sub[k] += f[k];
            const bool short_run_ends = (b_short_run_ends & 1) != 0, piece_ends = (b_piece_ends & 1) != 0;
            if (short_run_ends || piece_ends) {
                const bool seg_end_here = (b_seg_ends & 1) != 0, run_end_here = (b_run_ends & 1) != 0;
                // a short id's run: its share of s[b] now, the row of w' when the id is complete.  A long id's
                // piece: the share of s[b] if it is a whole run, the row of w' if it is the id's only piece,
                // parked otherwise.
                const bool whole_run = short_run_ends || (run_head && run_end_here);
                const bool to_w = short_run_ends ? seg_end_here : (whole_run && seg_head && seg_end_here);
                const bool park = piece_ends && !to_w;
                float sq = 0.f, wsq = 0.f, out[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    sq = fmaf(sub[k], sub[k], sq);
                    if (short_run_ends) tot[k] += sub[k];
                    out[k] = short_run_ends ? tot[k] : sub[k];
                }
                if (!has_cols) sq = 0.f;                         // such lanes hold a copy of lane 0's columns
                if (has_cols && (to_w || park)) {
                    float *dst = to_w ? w + (int64_t)cur_key * D + c0 : runsum + (int64_t)first * D + c0;
                    wsq = put_row(dst, out, c0, D, to_w && accumulate != 0, to_w);
                }
                if (whole_run) {
                    wave_sum2(sq, wsq);                          // one exchange for both
                    if (lane == 0) {
                        contrib[(int64_t)cb * n + first] = sq;
                        if (to_w && !accumulate) bigpart[(int64_t)cb * n + (short_run_ends ? id_first : first)] = wsq;
                    }
                }
                if (park && cb == 0 && lane == 0) {
                    if (seg_head) multi[first_idx] = 1u;
                    if (run_head && !run_end_here) multi_run[first_idx] = 1u;
                }
            }
            b_opens_id >>= 1; b_opens >>= 1; b_run_head >>= 1; b_short_run_ends >>= 1;
            b_piece_ends >>= 1; b_run_ends >>= 1; b_seg_ends >>= 1;
        }
    }
    }   // chunks
}

// First index in [lo, n) whose (id, position) pair is not below (v, target); every lane searches for its own
// target, the loop runs until the slowest lane is done (about log2(n) dependent loads).
__device__ __forceinline__ int64_t lower_bound_pair(const uint32_t *keys, const uint32_t *vals, int64_t lo, int64_t n,
                                                    uint32_t v, uint32_t target)
{
    int64_t len = n - lo;
    while (__any(len > 0)) {
        const int64_t half = len >> 1, m = lo + half;
        bool below = false;
        if (len > 0) {
            const uint32_t k = keys[m], p = vals[m];
            below = k < v || (k == v && p < target);
        }
        lo = below ? m + 1 : lo;
        len = below ? len - half - 1 : half;
    }
    return lo;
}

// The same for one target that the whole wave shares: every round the 64 lanes probe 64 positions that cut the
// range into 65 parts, and the number of probes below the target says which part to keep: three rounds of
// loads for 32768 positions instead of fifteen.  [lo, hi) is wave-uniform; every lane must be active.
__device__ __forceinline__ int64_t wave_lower_bound_pair(const uint32_t *keys, const uint32_t *vals, int64_t lo,
                                                         int64_t hi, uint32_t v, uint32_t target, int lane)
{
    while (hi > lo) {
        const int64_t len = hi - lo;
        // probe j sits at lo + floor((j + 1) * len / 65), below hi; when len < 65 some probes repeat a position or
        // sit at lo, which keeps the count monotone
        const int64_t at = len <= 64 ? lo + (lane < len ? lane : len - 1) : lo + ((int64_t)(lane + 1) * len) / 65;
        const uint32_t k = keys[at], p = vals[at];
        const bool below = k < v || (k == v && p < target);
        const int c = __builtin_popcountll(__ballot(below));        // probes are in order, so these are the first c
        if (len <= 64) return lo + (c < len ? c : len);
        const int64_t new_lo = c == 0 ? lo : lo + ((int64_t)c * len) / 65 + 1;
        const int64_t new_hi = c == 64 ? hi : lo + ((int64_t)(c + 1) * len) / 65;
        lo = new_lo;
        hi = new_hi;
    }
    return lo;
}

// Kernel B, two launches.  First per run (kIds = false): a wave looks after the runs of long ids whose first
// sorted position is among its kChunk positions and that kernel A marked as having several pieces; it adds
// the run's parked piece sums in sorted order, squares the result (the run's share of s[b]) and parks it in
// place of the run's first piece.  Then per id (kIds = true): a wave looks after the long ids whose first
// sorted position is among its positions and adds the parked run sums in example order: the row of w'.
// Neither walks the positions: the sorted list is searched.  A run's pieces start at its first position and
// at every multiple of kPiece below the run's end, which one search finds; an id's runs start where the
// searches for (id, b*T), one example per lane, land on that id and example.  The cost is logarithmic in
// the number of positions however long the id is.  Parked sums are loaded sixteen at a time.
template <bool kIds>
__global__ __launch_bounds__(64 * kWavesPerBlock) void emb_sums_kernel(
    const uint32_t *keys, const uint32_t *vals, float *w, float *runsum, float *contrib, float *bigpart,
    const uint32_t *marks_at, int64_t n, int Tn, int D, int V, int accumulate)
{
    constexpr int kBatch = 16;                                   // parked sums in flight
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t i0 = (int64_t)blockIdx.x * kChunk;
    const int cb = blockIdx.y * kWavesPerBlock + wave, c0 = cb * kColBlock + lane * 8;
    if (cb * kColBlock >= D) return;
    const bool has_cols = c0 < D;
    const bool runsum_vec = c0 + 8 <= D && D % 4 == 0 && (reinterpret_cast<uintptr_t>(runsum) & 15u) == 0;
    const int Bn = (int)(n / Tn);
    uint64_t marks = __ballot(lane < kChunk && i0 + lane < n && marks_at[i0 + lane < n ? i0 + lane : 0] != 0u);
    while (marks) {
        const int64_t i = i0 + __builtin_ctzll(marks);
        marks &= marks - 1;
        const uint32_t v = keys[i], p0 = vals[i], ex0 = p0 / (uint32_t)Tn;
        float acc[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = 0.f;
        // the parked sums at the positions held by the lanes of `take`, in lane order
        auto add_parked = [&](uint64_t take, uint32_t pos) {
            while (take) {
                uint32_t ent[kBatch];                            // all loads first, then the additions in order
                int cnt = 0;
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    if (take) {
                        ent[u] = lane_value(pos, __builtin_ctzll(take));
                        take &= take - 1;
                        ++cnt;
                    } else {
                        ent[u] = ent[u > 0 ? u - 1 : 0];
                    }
                }
                float add[kBatch][8];
                if (runsum_vec) {
                    Row8<float> raw[kBatch];
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) raw[u] = load_row8(runsum, (int64_t)ent[u], D, c0);
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) unpack_row8(raw[u], add[u]);
                } else {
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
#pragma unroll
                        for (int k = 0; k < 8; ++k) add[u][k] = 0.f;
                        if (has_cols && u < cnt) add_row(runsum, (int64_t)ent[u], D, c0, false, add[u]);
                    }
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u)
                    if (u < cnt) {
#pragma unroll
                        for (int k = 0; k < 8; ++k) acc[k] += add[u][k];
                    }
            }
        };
        if constexpr (kIds) {
            // the id's positions end where (v + 1, 0) would go; the examples' runs are searched for inside them
            const int64_t seg_end = wave_lower_bound_pair(keys, vals, i, n, v + 1u, 0u, lane);
            for (int b0 = 0; b0 < Bn; b0 += 64) {
                const int b = b0 + lane;
                const uint32_t target = (uint32_t)(b < Bn ? b : 0) * (uint32_t)Tn;
                const int64_t at = lower_bound_pair(keys, vals, i, seg_end, v, target);
                const uint32_t k = at < n ? keys[at] : 0xffffffffu, pos = at < n ? vals[at] : 0u;
                add_parked(__ballot(b < Bn && k == v && pos - target < (uint32_t)Tn), pos);
            }
            float wsq = has_cols ? put_row(w + (int64_t)v * D + c0, acc, c0, D, accumulate != 0, true) : 0.f;
            if (!accumulate) {
                wsq = wave_sum(wsq);
                if (lane == 0) bigpart[(int64_t)cb * n + p0] = wsq;
            }
        } else {
            const int64_t end = wave_lower_bound_pair(keys, vals, i, n, v, (ex0 + 1u) * (uint32_t)Tn, lane);
            const int64_t h1 = (i / kPiece + 1) * kPiece;        // the run's second piece, if it gets that far
            const int64_t npieces = 1 + (end > h1 ? (end - h1 + kPiece - 1) / kPiece : 0);
            for (int64_t u0 = 0; u0 < npieces; u0 += 64) {
                const int64_t u = u0 + lane, at = u == 0 ? i : h1 + (u - 1) * kPiece;
                const bool ok = u < npieces;
                add_parked(__ballot(ok), ok ? vals[at] : 0u);
            }
            float sq = has_cols ? put_row(runsum + (int64_t)p0 * D + c0, acc, c0, D, false) : 0.f;
            sq = wave_sum(sq);
            if (lane == 0) contrib[(int64_t)cb * n + p0] = sq;
        }
    }
}

// partial sums of squares of w (accumulate mode: every row counts, not only those touched).  Four 16-byte
// loads in flight per thread; every thread's own order of additions is fixed.
__global__ __launch_bounds__(256) void emb_wnorm_kernel(const float *w, int64_t n, double *part)
{
    __shared__ double slots[4];
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double t = 0.0;
    if ((reinterpret_cast<uintptr_t>(w) & 15u) == 0) {
        const float4 *w4 = reinterpret_cast<const float4 *>(w);
        const int64_t n4 = n / 4;
        double t1 = 0.0, t2 = 0.0, t3 = 0.0;
        auto sq4 = [](const float4 &v) {
            return (double)v.x * v.x + (double)v.y * v.y + (double)v.z * v.z + (double)v.w * v.w;
        };
        for (; i + 3 * stride < n4; i += 4 * stride) {
            const float4 a = w4[i], b = w4[i + stride], c = w4[i + 2 * stride], d = w4[i + 3 * stride];
            t += sq4(a); t1 += sq4(b); t2 += sq4(c); t3 += sq4(d);
        }
        for (; i < n4; i += stride) t += sq4(w4[i]);
        t = (t + t1) + (t2 + t3);
        i = n4 * 4 + (int64_t)blockIdx.x * 256 + threadIdx.x;
    }
    for (; i < n; i += stride) t += (double)w[i] * (double)w[i];
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
            // sixteen 16-byte loads in flight per thread; every thread's order of additions is fixed
            double part[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) part[u] = 0.0;
            const int64_t m = (int64_t)ncb * n, m4 = m / 4;       // bigpart is 256-byte aligned
            const float4 *big4 = reinterpret_cast<const float4 *>(bigpart);
            auto sum4 = [](const float4 &q) { return ((double)q.x + (double)q.y) + ((double)q.z + (double)q.w); };
            int64_t i = threadIdx.x;
            for (; i + 15 * 1024 < m4; i += 16 * 1024) {
                float4 q[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) q[u] = big4[i + u * 1024];
#pragma unroll
                for (int u = 0; u < 16; ++u) part[u] += sum4(q[u]);
            }
            for (; i < m4; i += 1024) part[0] += sum4(big4[i]);
            for (i = m4 * 4 + threadIdx.x; i < m; i += 1024) part[1] += (double)bigpart[i];
#pragma unroll
            for (int u = 0; u < 16; ++u) t += part[u];
        }
        t = block_sum_f64(t, slots);
        if (threadIdx.x == 0) big_sq[0] = (float)t;
    }
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }


// The zero fill of w' (bandwidth bound) has nothing to do with the sort (a dozen tiny launches): it runs on a
// side stream of the library's own, forked from and joined to the caller's stream with events, so the two
// overlap.  One side stream and event pair per device, made at the first call there and kept; calls that
// share a device share them (the events order each call's fill with that call's own work).
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    std::mutex in_use;   // held by a call from its fork to its join: the two events are recorded and waited
                         // on as pairs, which another thread's call on the same device must not interleave
};
constexpr int kMaxDevices = 64;
SideStream g_side[kMaxDevices];
std::mutex g_side_mutex;

SideStream *side_stream()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_side_mutex);
    SideStream &s = g_side[dev];
    if (!s.stream) {
        hipStream_t st = nullptr;
        hipEvent_t a = nullptr, b = nullptr;
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) return nullptr;   // default priority
        if (hipEventCreateWithFlags(&a, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&b, hipEventDisableTiming) != hipSuccess) {
            (void)hipStreamDestroy(st);
            if (a) (void)hipEventDestroy(a);
            return nullptr;
        }
        s.stream = st; s.fork = a; s.join = b;
    }
    return &s;
}

int key_bits(int V)
{
    int bits = 1;
    while (bits < 32 && ((uint64_t)1 << bits) <= (uint64_t)V) ++bits;   // keys run up to V inclusive
    return bits;
}

struct EmbPlan {
    int64_t n;
    int ncb;
    size_t off_keys_in, off_keys_out, off_vals_in, off_vals_out, off_contrib, off_bigpart, off_multi, off_multi_run, off_present, off_wpart, off_tiles, off_temp, off_runsum;
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
    p.off_bigpart = p.off_contrib + f;            // directly behind contrib, the marks behind that: one fill
    p.off_multi = p.off_bigpart + f;              // clears all three
    p.off_multi_run = p.off_multi + arr;
    p.off_present = p.off_multi_run + arr;        // one byte per vocabulary row, cleared with the rest
    p.off_wpart = p.off_present + align256((size_t)V);
    p.off_tiles = p.off_wpart + align256(kNormBlocks * sizeof(double));
    const int64_t ntiles = (p.n + kSortTile - 1) / kSortTile;
    p.off_temp = p.off_tiles + (ntiles <= kSortTiles ? align256((size_t)ntiles * kSortTile * sizeof(uint64_t)) : 0);
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

// The call behind embedding_pegn and embedding_pegn_presorted.  With `ids`: keys are made and sorted here (the
// zero fill runs beside the sort).  With sorted_ids / sorted_pos: the caller sorted them earlier
// (embedding_sort_ids), the scratch is cleared here and the fill runs beside the run and id kernels.
static int run_embedding(const void *ids, int ids_are_int64, const uint32_t *sorted_ids, const uint32_t *sorted_pos,
                         const void *g, float *w, float *s, float *big_sq, int B, int T, int D, int V, lnpegn_dtype dt,
                         void *workspace, size_t workspace_bytes, unsigned flags, void *stream)
{
    if (!emb_shape_ok(B, T, D, V) || !g || !w || !s || !workspace) return LNPEGN_EINVAL;
    if (!ids && (!sorted_ids || !sorted_pos)) return LNPEGN_EINVAL;
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
    uint32_t *vals_in = reinterpret_cast<uint32_t *>(ws + p.off_vals_in);
    const uint32_t *keys_out = ids ? reinterpret_cast<uint32_t *>(ws + p.off_keys_out) : sorted_ids;
    const uint32_t *vals_out = ids ? reinterpret_cast<uint32_t *>(ws + p.off_vals_out) : sorted_pos;
    float *contrib = reinterpret_cast<float *>(ws + p.off_contrib);
    float *bigpart = reinterpret_cast<float *>(ws + p.off_bigpart);
    uint32_t *multi = reinterpret_cast<uint32_t *>(ws + p.off_multi);
    uint32_t *multi_run = reinterpret_cast<uint32_t *>(ws + p.off_multi_run);
    uint8_t *present = reinterpret_cast<uint8_t *>(ws + p.off_present);
    double *wpart = reinterpret_cast<double *>(ws + p.off_wpart);
    const int64_t nscratch = (int64_t)((p.off_wpart - p.off_contrib) / sizeof(float));
    const unsigned nblk = (unsigned)((p.n + 255) / 256);

    const int ntiles = (int)((p.n + kSortTile - 1) / kSortTile);
    const bool own_sort = ids && ntiles <= kSortTiles;
    uint64_t *tiles = reinterpret_cast<uint64_t *>(ws + p.off_tiles);
    // 1. scratch cleared, the ids sorted (two launches of our own for up to kSortTiles * kSortTile positions; the
    //    library's radix sort beyond that, after the fork), and the ids that occur marked for the fill
    if (own_sort) {
        if (launch(emb_tile_sort_kernel, dim3(ntiles), dim3(kSortThreads), 0, st, ids, ids_are_int64, p.n, V, tiles, contrib, nscratch) != hipSuccess) return LNPEGN_EHIP;
        if (launch(emb_rank_kernel, dim3(ntiles * (kSortTile / 256)), dim3(256), 0, st, tiles, ntiles, p.n, V,
                   const_cast<uint32_t *>(keys_out), const_cast<uint32_t *>(vals_out), accumulate ? nullptr : present) != hipSuccess)
            return LNPEGN_EHIP;
    } else if (ids) {
        if (launch(emb_prepare_kernel, dim3(nblk), dim3(256), 0, st, ids, ids_are_int64, keys_in, vals_in, contrib, p.n, nscratch, V) != hipSuccess) return LNPEGN_EHIP;
    } else {
        const unsigned cb = (unsigned)(nscratch / 256 / 4 + 1 < 4096 ? nscratch / 256 / 4 + 1 : 4096);
        if (launch(emb_clear_kernel, dim3(cb), dim3(256), 0, st, contrib, nscratch) != hipSuccess) return LNPEGN_EHIP;
    }
    // 2. fork: the fill of the rows no id selects, on the side stream (on the caller's stream if there is none)
    SideStream *side = accumulate ? nullptr : side_stream();
    std::unique_lock<std::mutex> side_lock;
    if (side) side_lock = std::unique_lock<std::mutex>(side->in_use);
    if (!accumulate) {
        if (!own_sort &&
            launch(emb_mark_kernel, dim3(nblk), dim3(256), 0, st, ids ? keys_in : keys_out, p.n, V, present) != hipSuccess)
            return LNPEGN_EHIP;
        hipStream_t fs = st;
        if (side) {
            if (hipEventRecord(side->fork, st) != hipSuccess || hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess)
                return LNPEGN_EHIP;
            fs = side->stream;
        }
        const int64_t nw = (int64_t)V * D;
        const unsigned fb = (unsigned)(nw / 256 / 8 + 1 < 65536 ? nw / 256 / 8 + 1 : 65536);
        if (launch(emb_fill_kernel, dim3(fb), dim3(256), 0, fs, w, (int64_t)V, D, present) != hipSuccess) return LNPEGN_EHIP;
        if (side && hipEventRecord(side->join, fs) != hipSuccess) return LNPEGN_EHIP;
    }
    // 3. the library's sort for batches beyond our own
    if (ids && !own_sort) {
        size_t temp = p.temp_bytes;
        if (rocprim::radix_sort_pairs(ws + p.off_temp, temp, keys_in, const_cast<uint32_t *>(keys_out), vals_in,
                                      const_cast<uint32_t *>(vals_out), (size_t)p.n, 0, key_bits(V), st) != hipSuccess)
            return LNPEGN_EHIP;
    }
    // 4. runs, then the marked runs and ids: these write the rows of the ids that occur, the fill the others
    const int esz = dt == LNPEGN_BF16 ? 2 : 4;
    // 8 columns per lane: 16 bytes of bf16, 32 bytes of fp32; rows must keep that alignment
    const int vec_ok = ((reinterpret_cast<uintptr_t>(g) & 15u) == 0 && ((int64_t)D * esz) % 16 == 0) ? 1 : 0;
    const dim3 grid((unsigned)((p.n + kChunk - 1) / kChunk), (unsigned)((p.ncb + kWavesPerBlock - 1) / kWavesPerBlock));
    const dim3 grid_runs(grid.x < (unsigned)g_emb_run_blocks ? grid.x : (unsigned)g_emb_run_blocks, grid.y);
    float *runsum = reinterpret_cast<float *>(ws + p.off_runsum);
    const bool vec = vec_ok && D % 8 == 0;
    hipError_t runs_status = hipSuccess;
    auto runs = [&](auto kernel, auto *gp) {
        runs_status = launch(kernel, grid_runs, dim3(64 * kWavesPerBlock), 0, st, gp, keys_out, vals_out, w, runsum, contrib, bigpart, multi, multi_run, p.n, T, D, V, accumulate);
    };
    if (dt == LNPEGN_BF16) {
        if (vec) runs(emb_runs_kernel<bf16_t, true>, static_cast<const bf16_t *>(g));
        else runs(emb_runs_kernel<bf16_t, false>, static_cast<const bf16_t *>(g));
    } else {
        if (vec) runs(emb_runs_kernel<float, true>, static_cast<const float *>(g));
        else runs(emb_runs_kernel<float, false>, static_cast<const float *>(g));
    }
    if (runs_status != hipSuccess) return LNPEGN_EHIP;
    if (launch(emb_sums_kernel<false>, grid, dim3(64 * kWavesPerBlock), 0, st, keys_out, vals_out, w, runsum, contrib, bigpart, multi_run, p.n, T, D, V, accumulate) != hipSuccess) return LNPEGN_EHIP;
    if (launch(emb_sums_kernel<true>, grid, dim3(64 * kWavesPerBlock), 0, st, keys_out, vals_out, w, runsum, contrib, bigpart, multi, p.n, T, D, V, accumulate) != hipSuccess) return LNPEGN_EHIP;
    // 5. join: w' is complete on the caller's stream from here
    if (side && hipStreamWaitEvent(st, side->join, 0) != hipSuccess) return LNPEGN_EHIP;
    if (side) side_lock.unlock();
    const bool wnorm = accumulate && big_sq;
    if (wnorm) {
        if (launch(emb_wnorm_kernel, dim3(kNormBlocks), dim3(256), 0, st, w, (int64_t)V * D, wpart) != hipSuccess) return LNPEGN_EHIP;
    }
    return launch(emb_final_kernel, dim3(B + 1), dim3(1024), 0, st, contrib, bigpart, wnorm ? wpart : nullptr, kNormBlocks, s, big_sq, B, T, p.ncb, p.n) == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

int embedding_pegn(const void *ids, int ids_are_int64, const void *g, float *w, float *s, float *big_sq, int B, int T,
                   int D, int V, lnpegn_dtype dt, void *workspace, size_t workspace_bytes, unsigned flags, void *stream)
{
    if (!ids) return LNPEGN_EINVAL;
    return run_embedding(ids, ids_are_int64, nullptr, nullptr, g, w, s, big_sq, B, T, D, V, dt, workspace,
                         workspace_bytes, flags, stream);
}

int embedding_sort_ids(const void *ids, int ids_are_int64, int B, int T, int V, uint32_t *sorted_ids,
                       uint32_t *sorted_pos, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!emb_shape_ok(B, T, 1, V) || !ids || !sorted_ids || !sorted_pos || !workspace) return LNPEGN_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return LNPEGN_EINVAL;
    EmbPlan p;
    if (make_emb_plan(B, T, 1, V, p) != hipSuccess) return LNPEGN_EHIP;
    if (workspace_bytes < p.bytes) return LNPEGN_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    uint32_t *keys_in = reinterpret_cast<uint32_t *>(ws + p.off_keys_in);
    uint32_t *vals_in = reinterpret_cast<uint32_t *>(ws + p.off_vals_in);
    const int ntiles = (int)((p.n + kSortTile - 1) / kSortTile);
    if (ntiles <= kSortTiles) {
        uint64_t *tiles = reinterpret_cast<uint64_t *>(ws + p.off_tiles);
        if (launch(emb_tile_sort_kernel, dim3(ntiles), dim3(kSortThreads), 0, st, ids, ids_are_int64, p.n, V, tiles,
                   static_cast<float *>(nullptr), (int64_t)0) != hipSuccess)
            return LNPEGN_EHIP;
        return launch(emb_rank_kernel, dim3(ntiles * (kSortTile / 256)), dim3(256), 0, st, tiles, ntiles, p.n, V, sorted_ids,
                      sorted_pos, static_cast<uint8_t *>(nullptr)) == hipSuccess
                   ? LNPEGN_OK
                   : LNPEGN_EHIP;
    }
    const unsigned nblk = (unsigned)((p.n + 255) / 256);
    if (launch(emb_prepare_kernel, dim3(nblk), dim3(256), 0, st, ids, ids_are_int64, keys_in, vals_in,
               static_cast<float *>(nullptr), p.n, (int64_t)0, V) != hipSuccess)
        return LNPEGN_EHIP;
    size_t temp = p.temp_bytes;
    return rocprim::radix_sort_pairs(ws + p.off_temp, temp, keys_in, sorted_ids, vals_in, sorted_pos, (size_t)p.n, 0,
                                     key_bits(V), st) == hipSuccess
               ? LNPEGN_OK
               : LNPEGN_EHIP;
}

int embedding_pegn_presorted(const uint32_t *sorted_ids, const uint32_t *sorted_pos, const void *g, float *w, float *s,
                             float *big_sq, int B, int T, int D, int V, lnpegn_dtype dt, void *workspace,
                             size_t workspace_bytes, unsigned flags, void *stream)
{
    if (!sorted_ids || !sorted_pos) return LNPEGN_EINVAL;
    return run_embedding(nullptr, 0, sorted_ids, sorted_pos, g, w, s, big_sq, B, T, D, V, dt, workspace,
                         workspace_bytes, flags, stream);
}

}  // extern "C"
