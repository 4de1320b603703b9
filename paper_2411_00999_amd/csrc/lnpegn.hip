// C ABI of the lnpegn library (declared in include/lnpegn.h): argument validation, launch
// planning and kernel launches.  No allocation, no synchronisation, no state between calls
// apart from the process-wide launch-shape overrides of lnpegn_set_tuning() and the per-device
// address of the fixed scratch of ln_bwd_pegn_static.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/lnpegn.h"
#include "lnpegn_finalize.h"
#include "lnpegn_tracker.h"
#include "lnpegn_launch.h"
#include "lnpegn_rows.h"

// Scratch of ln_bwd_pegn_static: the workspace of a backward call, held by the library itself so that the
// call allocates nothing.  One copy per GPU the library runs on, kept until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; kernels are given the address it returns.
constexpr size_t kStaticScratchBytes = LNPEGN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace lnpegn {
thread_local int g_last_hip_error = 0;   // hipError_t behind this thread's latest LNPEGN_EHIP from a row kernel launch
extern int g_emb_run_blocks;   // embedding_pegn.hip: workgroups of its run kernel per column group
namespace {

// launch-shape overrides (0 = automatic)
int g_chunks_pegn = 0;
int g_chunks_plain = 0;
int g_waves = 0;
int g_vpt_max = 0;          // cap on 16-byte vectors per lane and array (0: automatic)
int g_xcd = -1;        // hand neighbouring chunks to the same XCD: 0 never, 1 always, -1 automatic
int g_blocked = -1;    // chunks of consecutive rows: 0 never, 1 always, -1 automatic
int g_dx_cached = -1;  // dx stores write-back instead of streaming: 0 never, 1 always, -1 automatic
int g_stagger = -1;   // rows between the sweep starts of consecutive examples (-1 = automatic)
// one-shot profiling events around the row kernel (null = disarmed)
hipEvent_t g_ev_start = nullptr;
hipEvent_t g_ev_stop = nullptr;

constexpr int kMaxChunks = 16384;
constexpr int kCUs = 256;           // MI355X
constexpr int kGroups = 16;         // groups of chunks in the reduction that gives the batch gradients
constexpr int64_t kSmallFinal = 32768;  // G1*D up to which one workgroup finishes the reduction
constexpr size_t kAlign = 256;

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

struct Plan {
    // row kernel
    bool plain;       // no per-example outputs: the plain backward's kernel
    bool fast;        // vectorised kernels usable (shape-wise; pointer alignment checked apart)
    bool sync;        // several waves per row
    int vpt;          // 16-byte vectors per lane
    int S, R;         // waves per row, row groups per workgroup
    int max_threads;  // launch bound of the instantiation
    int nvec;
    int64_t Tp;       // rows per partition example
    int C;            // chunks per partition example
    int64_t n_slots;  // chunks in all
    int rows_per;     // > 0: a chunk is a block of that many consecutive rows; 0: every C-th row of its example
    int64_t stagger;  // rows between the sweep starts of consecutive examples
    int xcd_chunks;   // > 0: chunks per XCD (an example's chunks share an L2); 0: chunks in launch order
    size_t lds_bytes;
    // reduction
    int ntile;
    int gs, G1;       // chunks per group, groups
    bool emit_pe;     // row kernel writes the per-example norms (a chunk is a whole example)
    int n_ex;         // examples whose norms the reduction takes from their chunks' sums (0 or B)
    // workspace layout (byte offsets); everything but `part` depends on B and D only, so that a
    // batched reduction can address any layer of the same shape
    size_t off_grp, off_part_s, off_part_big, off_part, total;
};
constexpr size_t kHeaderBytes = 256;

// Chunks per example, given W workgroups resident at a time.  W/B of them fill one round of workgroups when B
// divides W; when they would leave much of a round empty (B*C/W below 0.85, or a last round that is less than a
// third full), the example is cut finer, into three rounds or more: many short workgroups even out by themselves,
// at the price of one more flush of column sums per chunk.  Measured, bf16 D=1024, us per launch, W/B chunks ->
// this choice: B=300 T=100 39.6 -> 33.3, B=260 T=128 44.6 -> 38.6, B=600 T=64 47.7 -> 45.5, B=513 T=64
// 40.0 -> 37.0, B=384 T=64 30.0 -> 29.1, B=200 T=128 31.4 -> 30.2; D=2048: B=300 T=100 104.5 -> 77.9, B=600 T=64
// 105.3 -> 91.5; D=4096: B=300 T=100 170.1 -> 153.5.  (B=700 T=48 and B=1000 T=32, whose second round is more
// than a third full, are faster with one chunk per example: 35.8 against 36.9 and 34.1 against 35.2.)
int64_t chunks_per_example(int64_t B, int64_t T, int64_t W)
{
    const int64_t c0 = W / B > 1 ? W / B : 1;
    const int64_t n = B * c0, full = n / W, rest = n % W;   // rounds that are full, workgroups in the last one
    const bool fits = n <= W ? 20 * n >= 17 * W
                             : rest == 0 || full >= 3 || (full == 1 && 10 * rest >= 3 * W);
    if (fits) return c0;
    const int64_t c3 = (3 * W + B - 1) / B;         // three rounds
    return (c3 <= 16 && T / c3 >= 16) ? c3 : c0;    // ... unless that leaves a chunk fewer than 16 rows
}

// `vector_ok`: the 16-byte aligned fast kernels will run (else the generic kernel does).
Plan make_plan(int B, int T, int D, lnpegn_dtype dt, bool pegn, bool vector_ok)
{
    Plan p{};
    p.plain = !pegn;
    const int E = dt == LNPEGN_BF16 ? 8 : 4;
    const int64_t N = (int64_t)B * T;
    int vpt_max = 16 / E;                            // 16 elements per lane ...
    if (g_vpt_max > 0 && g_vpt_max < vpt_max) vpt_max = g_vpt_max;
    // ... up to 32 for rows beyond eight waves of 16 (D > 8192): eight waves of 24 or 32 elements per lane
    if (D % E == 0 && D / E > 64 * vpt_max * 8) vpt_max = 32 / E;
    p.fast = vector_ok && (D % E == 0) && (D / E <= 64 * vpt_max * 8);
    p.nvec = p.fast ? D / E : 0;
    p.sync = false;
    p.vpt = 1;
    p.S = 1;
    p.R = 4;
    p.max_threads = 256;
    int waves_per_simd = 4;                          // resident waves per SIMD to aim for
    if (p.fast) {
        p.S = vpt_max > 16 / E ? 8 : ceil_div(p.nvec, 64 * vpt_max);   // beyond 16 elements per lane: always eight waves
        p.vpt = ceil_div(p.nvec, 64 * p.S);
        p.sync = p.S > 1;
        const int elems = p.vpt * E;                 // per lane
        waves_per_simd = elems > 8 ? 2 : 4;          // measured: more waves of 16-element lanes only add contention
        // launch bound of the instantiation that will run: 256 threads for S = 1, 2, 4; 512 else
        const int max_waves = (elems <= 8 && p.S <= 2) ? 4 : 8;
        // row groups per workgroup.  Wide lanes: six waves per workgroup, one workgroup per CU (measured, B*T =
        // 32768 rows: bf16 D=2048 69.2 -> 66.9 us per-example and 69.0 -> 65.4 plain against four waves; fp32
        // D=2048 151.7 -> 145.6 and 133 -> 131; eight waves are slower than six; no difference where a row
        // already takes four or eight waves).
        // (rows that one wave covers stay at four row groups: six made the short kernels of B=8 T=1024 D=768 and
        // B=512 T=64 D=1024 3-10 % slower)
        // (fp32 rows of four waves: two row groups, measured with the per-example sweeps, 288.7 -> 273.8 us)
        // (rows of two waves with lanes left over, D=1280, 1536 or 1600 in bf16, have fewer bytes in flight per
        // wave and take four row groups: D=1280 64.5 -> 52.0 us, D=1536 65.0 -> 55.3; rows of three waves take two:
        // bf16 D=3072 147.7 -> 111.5 per-example and 107.6 -> 100.3 plain, fp32 D=3072 216.3 -> 205.1)
        const bool full = p.nvec == 64 * p.S * p.vpt;
        int R = g_waves > 0 ? g_waves / p.S
                : (elems > 8 && p.S == 2) ? (full ? 3 : 4)
                : p.S == 3 ? 2
                : (pegn && E == 4 && p.S == 4 && p.vpt >= 3) ? 2
                : (p.S >= 4 ? 1 : 4 / p.S);
        if (R < 1) R = 1;
        while (R > 1 && R * p.S > max_waves) --R;
        p.R = R;
        p.max_threads = 64 * max_waves;
    }
    const int nwaves = p.fast ? p.R * p.S : 4;
    // one full round of resident workgroups unless told otherwise
    int target = pegn ? g_chunks_pegn : g_chunks_plain;
    if (target <= 0) {
        int per_cu = (waves_per_simd * 4) / nwaves > 0 ? (waves_per_simd * 4) / nwaves : 1;
        // Per-example sweeps, measured on B*T = 32768 rows (bf16, us per launch, fewer / more chunks):
        //   rows of one wave   (D=768: 34.8 / 29.3, D=1024: 39.6 / 38.8)    two workgroups of four waves per CU
        //   rows of two waves  (D=2048: six waves per workgroup)             one workgroup per CU
        //   rows of four waves (D=4096: 138.9 / 147.8)                       one workgroup per CU: half as many
        //       chunks per example keep each example's moving window of memory half as wide
        //   rows of eight waves (D=8192: 279.6 / 268.0)                      two rounds of workgroups: the second
        //       round starts where the first finishes, which evens out the CUs' unequal memory throughput
        // ... as long as a chunk keeps a hundred rows or so (short launches want the parallelism more).
        if (pegn && p.fast && p.S == 4 && waves_per_simd == 2 && per_cu > 1 && !(E == 4 && p.vpt >= 3) &&
            N / ((int64_t)kCUs * (per_cu / 2)) >= 96)
            per_cu /= 2;
        //   fp32 rows of two and four waves (lanes of four vectors; D=2048: 140.5 / 137.9, D=4096 with two row
        //       groups: 290.8 / 273.8) also take two rounds
        const bool wide_f32 = E == 4 && p.vpt >= 3 && p.S >= 2;
        //   rows of six and seven waves likewise (bf16 D=6144: 224.6 / 216.9)
        if (pegn && p.fast && (p.S >= 6 || wide_f32) && N / ((int64_t)kCUs * 2) >= 32) per_cu = 2;
        target = kCUs * per_cu;
    }
    // rows per chunk at least: two per row group, and four in all -- a chunk ends with a write of its 2*D column
    // sums, which is as many bytes as four bf16 rows carry
    const int rows_min = p.fast ? (2 * p.R > 4 ? 2 * p.R : 4) : 4;
    const int R = p.fast ? p.R : 1;
    // Prefer a chunk count that gives every chunk the same number of rows, a multiple of R: no
    // partial last iteration.  Searched downwards, never below 3/4 of the first choice.
    auto even_chunks = [&](int64_t c, int64_t rows) {
        for (int64_t t = c; t >= 1 && 4 * t >= 3 * c; --t)
            if (rows % (t * R) == 0) return t;
        return c;
    };
    if (pegn) {
        p.Tp = T;
        int64_t c = g_chunks_pegn > 0 || !p.fast ? target / B : chunks_per_example(B, T, target);
        // Long launches over fp32 rows of 16 elements per lane: several rounds of shorter workgroups, which even
        // out the CUs' unequal progress (measured, us per launch, one round -> this: B=16 T=2048 D=2048
        // 138.3 -> 134.3, B=8 T=4096 D=2048 137.2 -> 134.2, B=16 T=4096 D=2048 280.9 -> 265.9, B=16 T=2048 D=1024
        // 75.2 -> 72.0, B=16 T=2048 D=4096 279.6 -> 265.1 with two rounds and 283.3 with four; half as many rows,
        // B=16 T=1024 D=2048, are faster in one round, 72.8 against 74.0, and so are bf16 rows: D=2048 68.8 -> 71.2
        // with two rounds).
        // (fp32 D=1280 96.4 -> 93.1, D=1536 112.3 -> 109.2)
        if (g_chunks_pegn <= 0 && p.fast && E == 4 && p.vpt >= 3 && p.S <= 4 && N >= 32768 && B * c <= target) {
            int64_t rounds = p.S == 4 ? 2 : 4;
            while (rounds > 1 && T / (c * rounds) < 16) rounds /= 2;
            c *= rounds;
        }
        const int64_t cmax = T / rows_min > 1 ? T / rows_min : 1;
        if (c > cmax) c = cmax;
        if (c < 1) c = 1;
        p.C = (int)even_chunks(c, T);
        p.n_slots = (int64_t)B * p.C;
        // A chunk that is a whole short example, two or more of them per CU, rows of one wave: eight rows at a
        // time (measured, bf16 D=1024: B=512 T=64 35.8 -> 35.0 us, B=1024 T=32 35.2 -> 34.1, B=700 T=48
        // 37.8 -> 35.7; fp32 B=512 T=64 D=1024 77.5 -> 73.9; with fewer examples than that four rows are faster).
        if (p.fast && g_waves <= 0 && p.C == 1 && p.S == 1 && p.vpt * E > 8 && B >= 2 * kCUs && T >= 32) p.R = 8;
    } else {
        p.Tp = N;
        int64_t c = target;
        const int64_t cmax = N / rows_min > 1 ? N / rows_min : 1;
        if (c > cmax) c = cmax;
        p.C = (int)even_chunks(c, N);
        p.n_slots = p.C;
    }
    // The chunks of an example take every C-th row each, so that together they sweep the example as one narrow
    // window of memory: the fastest pattern as long as the examples, i.e. the windows, are few.  With more than 32
    // examples every chunk takes a block of consecutive rows instead: a few percent behind the best case of
    // the other pattern but without its bad cases (measured, us per launch, every C-th row / blocks: bf16 D=2048,
    // B*T = 32768: B=16 67.5 / 73.6, B=32 70.6 / 73.8, B=64 89.7 / 73.8; D=1024: B=64 48.9 / 37.3, B=128
    // 41.3 / 36.0, B=256 35.2 / 36.0).  The plain backward always has one window (D=2048: 67.3 / 73.2).
    const bool blocked = g_blocked >= 0 ? g_blocked != 0 : pegn && B > 32;
    p.rows_per = (blocked && p.C > 1) ? ceil_div(p.Tp, p.C) : 0;
    // Every example's sweep starts 5T/4B rows after its predecessor's; none when that is less than a row (measured
    // with a chunk per example, bf16 D=1024, no shift / one row: B=512 T=128 76.0 / 96.3 us, B=260 T=128 44.7 / 50.9,
    // B=1000 T=32 35.2 / 39.4, B=512 T=64 36.1 / 35.8).
    p.stagger = g_stagger >= 0 ? (pegn ? g_stagger : 0) : (!pegn || p.rows_per > 0) ? 0 : 5 * (int64_t)T / (4 * (int64_t)B);
    // measured: grouping an example's chunks on one XCD helps wide rows (S >= 4) and is neutral otherwise
    const bool xcd = g_xcd >= 0 ? g_xcd != 0 : p.S >= 4;
    p.xcd_chunks = (xcd && p.fast && p.n_slots % 8 == 0 && p.n_slots / 8 <= INT32_MAX) ? (int)(p.n_slots / 8) : 0;
    {
        const int nw = p.fast ? p.R * p.S : 4;
        const size_t xchg = (size_t)((10 * nw + 2 * p.S + 3) & ~3) * sizeof(float);
        const size_t merge = p.fast && p.R > 1 ? (size_t)nw * 2 * p.vpt * E * kWave * sizeof(float) : 0;
        p.lds_bytes = xchg + (merge > 512 ? merge : 512);
    }
    p.emit_pe = pegn && p.fast && p.C == 1;
    p.n_ex = pegn && !p.emit_pe ? B : 0;
    p.gs = ceil_div(p.n_slots, kGroups);
    p.G1 = ceil_div(p.n_slots, p.gs);
    p.ntile = ceil_div(D, kTile);
    const size_t vec_bytes = (size_t)2 * D * sizeof(float);
    size_t off = kHeaderBytes;            // the layout up to `part` does not depend on the path taken
    p.off_grp = off;       off += align_up((size_t)kGroups * vec_bytes);
    p.off_part_s = off;    off += align_up((size_t)B * p.ntile * 2 * sizeof(double));
    p.off_part_big = off;  off += align_up((size_t)p.ntile * 2 * sizeof(double));
    p.off_part = off;      off += align_up((size_t)p.n_slots * vec_bytes);
    p.total = off;
    return p;
}

bool shape_ok(int B, int T, int D) { return B > 0 && T > 0 && D > 0; }

// Device address of `scratch` on the current device, looked up once per device and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr || reinterpret_cast<uintptr_t>(ptr) % kAlign) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
bool dtype_ok(int dt) { return dt == LNPEGN_F32 || dt == LNPEGN_BF16; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int run_bwd(bool pegn, bool defer, bool accumulate, bool rms, const void *x, const void *dy, const void *gamma, const float *mean,
            const float *rstd, void *dx, float *dgamma, float *dbeta, float *pe_gamma_sq,
            float *pe_beta_sq, float *big_sq, int B, int T, int D, int dt, int gamma_dt, float eps,
            void *workspace, size_t workspace_bytes, void *stream)
{
    if (!shape_ok(B, T, D) || !(eps >= 0.f)) return LNPEGN_EINVAL;
    if (!dtype_ok(dt) || !dtype_ok(gamma_dt)) return LNPEGN_EUNSUPPORTED;
    if (!x || !dy || !gamma || !dx || !dgamma || (!rms && !dbeta)) return LNPEGN_EINVAL;
    if (pegn && (!pe_gamma_sq || (!rms && !pe_beta_sq))) return LNPEGN_EINVAL;
    if (!rms && (mean == nullptr) != (rstd == nullptr)) return LNPEGN_EINVAL;
    if (dx == x) return LNPEGN_EINVAL;
    if ((int64_t)B * T > INT32_MAX) return LNPEGN_EINVAL;   // row indices are 32-bit
    const bool vector_ok = aligned16(x) && aligned16(dy) && aligned16(dx) && aligned16(gamma);
    const Plan p = make_plan(B, T, D, (lnpegn_dtype)dt, pegn, vector_ok);
    if (!workspace || workspace_bytes < p.total) return LNPEGN_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return LNPEGN_EINVAL;
    if (p.n_slots > INT32_MAX) return LNPEGN_EINVAL;

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *part = reinterpret_cast<float *>(ws + p.off_part);

    RowArgs a{};
    a.x = x; a.dy = dy; a.gamma = gamma; a.mean = mean; a.rstd = rstd; a.dx = dx;
    a.part = part; a.pe_gamma_sq = pe_gamma_sq; a.pe_beta_sq = pe_beta_sq;
    a.Tp = p.Tp; a.C = p.C; a.D = D; a.nvec = p.nvec;
    a.rows_per = p.rows_per; a.stagger = p.stagger; a.xcd_chunks = p.xcd_chunks;
    a.S = p.S; a.gamma_is_f32 = gamma_dt == LNPEGN_F32; a.emit_pe = p.emit_pe; a.rms = rms;
    a.eps = eps; a.inv_D = 1.0f / (float)D;
    if (defer) {
        a.defer = reinterpret_cast<DeferHeader *>(ws);
        a.hdr = DeferHeader{dgamma, dbeta, pe_gamma_sq, pe_beta_sq, pegn ? big_sq : nullptr,
                            (int)p.n_slots, p.gs, p.G1, p.n_ex, p.C, accumulate ? 1 : 0};
    }

    const bool saved = rstd != nullptr;
    const RowLaunch rl{s, g_ev_start, g_ev_stop};
    g_ev_start = g_ev_stop = nullptr;
    RowShape rs{};
    rs.plain = p.plain; rs.fast = p.fast; rs.vpt = p.vpt; rs.S = p.S; rs.R = p.R; rs.nvec = p.nvec;
    rs.n_slots = p.n_slots; rs.lds_bytes = p.lds_bytes;
    // measured (size of dx in MiB: streaming / write-through, us per launch, one layer at a time): 32: 23.2 / 22.1,
    // 64: 39.1 / 36.6 and 41.2 / 35.9, 96: 57.3 / 54.2, 128: 69.6 / 68.6, 192: 108.3 / 109.6.  At 128 MiB the
    // write-through stores are still draining when the next layer starts: 48 such layers back to back take 3.46 ms
    // against 3.41 ms with streaming stores, so the switch is at 96 MiB.
    rs.dx_cached = g_dx_cached >= 0 ? g_dx_cached != 0
                                    : (int64_t)B * T * D * (dt == LNPEGN_BF16 ? 2 : 4) <= ((int64_t)96 << 20);
    const hipError_t e = dt == LNPEGN_BF16 ? (saved ? launch_rows_bf16_saved(rs, a, rl) : launch_rows_bf16_recompute(rs, a, rl))
                                           : (saved ? launch_rows_f32_saved(rs, a, rl) : launch_rows_f32_recompute(rs, a, rl));
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return LNPEGN_EHIP;
    }
    if (defer) return LNPEGN_OK;   // lnpegn_reduce_deferred finishes the job

    // ---- the levels above the chunks (fixed-order sums) ----
    ReduceArgs ra{};
    ra.part = part;
    ra.grp = reinterpret_cast<float *>(ws + p.off_grp);
    ra.part_s = reinterpret_cast<double *>(ws + p.off_part_s);
    ra.part_big = reinterpret_cast<double *>(ws + p.off_part_big);
    ra.dgamma = dgamma; ra.dbeta = dbeta;
    ra.pe_gamma_sq = pe_gamma_sq; ra.pe_beta_sq = pe_beta_sq;
    ra.big_sq = pegn ? big_sq : nullptr;
    ra.n_slots = (int)p.n_slots; ra.gs = p.gs; ra.G1 = p.G1; ra.n_ex = p.n_ex; ra.ex_gs = p.C; ra.D = D; ra.ntile = p.ntile;
    ra.accumulate = accumulate;
    if (launch(reduce_groups_kernel, dim3((unsigned)p.ntile, (unsigned)reduce_groups_count(ra)), dim3(kTile), 0, s, ra) != hipSuccess) return LNPEGN_EHIP;
    const bool need_scalars = p.n_ex > 0 || ra.big_sq != nullptr;
    if (p.G1 == 1 || (int64_t)p.G1 * D <= kSmallFinal) {
        if (p.G1 > 1 || need_scalars) {
            if (launch(reduce_final_small_kernel, dim3(1), dim3(1024), 0, s, ra) != hipSuccess) return LNPEGN_EHIP;
        }
    } else {
        if (launch(reduce_final_tiles_kernel, dim3((unsigned)p.ntile), dim3(kTile), 0, s, ra) != hipSuccess) return LNPEGN_EHIP;
        if (need_scalars) {
            if (launch(reduce_scalars_kernel, dim3(1), dim3(256), 0, s, ra) != hipSuccess) return LNPEGN_EHIP;
        }
    }
    return LNPEGN_OK;
}

// Streaming yardstick: every lane moves 4 x 16 bytes per array, one workgroup per 16 KiB.
template <int kMode>
__global__ __launch_bounds__(256) void stream_probe_kernel(const uint4 *a, const uint4 *b, uint4 *out,
                                                           int64_t nvec)
{
    const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    uint4 va[4], vb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t v = base + i * 256;
        if (v < nvec) {
            va[i] = a[v];
            if (kMode == 1) vb[i] = b[v];
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t v = base + i * 256;
        if (v < nvec) {
            uint4 o = va[i];
            if (kMode == 1) {
                o.x ^= vb[i].x; o.y ^= vb[i].y; o.z ^= vb[i].z; o.w ^= vb[i].w;
            }
            out[v] = o;
        }
    }
}

// The same with one vector per lane and array, streaming loads and stores, one workgroup per 4 KiB: the
// fastest plain streaming kernel found on this part (the workgroups are dealt out in address order and
// never loop, so the window of memory in use stays narrow).
__global__ __launch_bounds__(256) void stream_probe_oneshot_kernel(const uint4 *a, const uint4 *b, uint4 *out,
                                                                   int64_t nvec)
{
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v < nvec) {
        const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a) + v);
        const u32x4 y = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(b) + v);
        __builtin_nontemporal_store(x ^ y, reinterpret_cast<u32x4 *>(out) + v);
    }
}

template <typename T, bool kWriteY>
hipError_t launch_fwd(FwdArgs a, bool vector_ok, hipStream_t s)
{
    constexpr int E = Vec<T>::kElems;
    const int D = a.D;
    const int64_t N = a.N;
    const bool fast = vector_ok && (D % E == 0) && (D / E <= 64 * (16 / E) * 16);   // up to 16 waves share a row
    if (!fast) {
        const unsigned grid = (unsigned)(N < 4096 ? N : 4096);
        return launch(ln_fwd_generic_kernel<T, kWriteY>, dim3(grid), dim3(256), 0, s, a);
    }
    a.nvec = D / E;
    if (a.nvec <= 64 * (16 / E)) {
        const int vpt = ceil_div(a.nvec, 64);
        const int64_t want = (N + 3) / 4;
        const dim3 grid((unsigned)(want < 4096 ? want : 4096)), block(256);
        switch (vpt) {
            case 1: return launch(ln_fwd_kernel<T, 1, false, kWriteY>, grid, block, 0, s, a);
            case 2: return launch(ln_fwd_kernel<T, 2, false, kWriteY>, grid, block, 0, s, a);
            case 3: return launch(ln_fwd_kernel<T, 3, false, kWriteY>, grid, block, 0, s, a);
            case 4: return launch(ln_fwd_kernel<T, 4, false, kWriteY>, grid, block, 0, s, a);
            default: return hipErrorInvalidValue;
        }
    } else {
        const int waves = ceil_div(a.nvec, 64 * (16 / E));
        const int vpt = ceil_div(a.nvec, 64 * waves);
        // measured (B*T = 32768 rows, bf16): 16 resident waves per CU for rows of 2 and 4 waves (D=2048: 47.8 us
        // against 52.6 with twice as many; D=4096: 92.3 against 95.2), the full 32 for rows of 8 (D=8192: 181 against 190)
        const int64_t cap = waves <= 4 ? 4096 / waves : 4096;
        const dim3 grid((unsigned)(N < cap ? N : cap)), block(64 * waves);
        switch (vpt) {
            case 1: return launch(ln_fwd_kernel<T, 1, true, kWriteY>, grid, block, 0, s, a);
            case 2: return launch(ln_fwd_kernel<T, 2, true, kWriteY>, grid, block, 0, s, a);
            case 3: return launch(ln_fwd_kernel<T, 3, true, kWriteY>, grid, block, 0, s, a);
            case 4: return launch(ln_fwd_kernel<T, 4, true, kWriteY>, grid, block, 0, s, a);
            default: return hipErrorInvalidValue;
        }
    }
}

}  // namespace
}  // namespace lnpegn

using namespace lnpegn;

extern "C" {

size_t lnpegn_workspace_bytes(int B, int T, int D, lnpegn_dtype dt)
{
    if (!shape_ok(B, T, D) || !dtype_ok(dt)) return 0;
    size_t need = 0;
    for (int pegn = 0; pegn < 2; ++pegn)
        for (int vec = 0; vec < 2; ++vec) {
            const size_t t = make_plan(B, T, D, dt, pegn != 0, vec != 0).total;
            if (t > need) need = t;
        }
    return need;
}

int lnpegn_plan_query(int B, int T, int D, lnpegn_dtype dt, int per_example, int aligned, int64_t *out, int n_out)
{
    if (!shape_ok(B, T, D) || !out || n_out < 0) return LNPEGN_EINVAL;
    if (!dtype_ok(dt)) return LNPEGN_EUNSUPPORTED;
    const Plan p = make_plan(B, T, D, dt, per_example != 0, aligned != 0);
    const int64_t v[LNPEGN_PLAN_FIELDS] = {
        p.fast ? 1 : 0, p.S, p.fast ? p.R : 1, p.vpt, p.C, p.n_slots, p.rows_per, p.stagger, p.xcd_chunks,
        (int64_t)p.lds_bytes, p.emit_pe ? 1 : 0, p.n_ex, p.G1, p.gs, (int64_t)p.total, p.Tp};
    for (int i = 0; i < n_out && i < LNPEGN_PLAN_FIELDS; ++i) out[i] = v[i];
    return LNPEGN_OK;
}

int lnpegn_last_hip_error(void) { return g_last_hip_error; }

const char *lnpegn_status_string(int status)
{
    switch (status) {
        case LNPEGN_OK: return "ok";
        case LNPEGN_EINVAL: return "invalid argument";
        case LNPEGN_EUNSUPPORTED: return "unsupported dtype";
        case LNPEGN_EWORKSPACE: return "workspace missing or too small";
        case LNPEGN_EHIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int ln_fwd_stats(const void *x, float *mean, float *rstd, int B, int T, int D, lnpegn_dtype dt,
                 float eps, void *stream)
{
    if (!shape_ok(B, T, D) || !(eps >= 0.f)) return LNPEGN_EINVAL;
    if (!dtype_ok(dt)) return LNPEGN_EUNSUPPORTED;
    if (!x || !mean || !rstd) return LNPEGN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    FwdArgs a{};
    a.x = x; a.mean = mean; a.rstd = rstd; a.N = (int64_t)B * T; a.D = D; a.eps = eps;
    a.inv_D = 1.0f / (float)D;
    const hipError_t e = dt == LNPEGN_BF16 ? launch_fwd<bf16_t, false>(a, aligned16(x), s)
                                           : launch_fwd<float, false>(a, aligned16(x), s);
    return e == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

int ln_fwd(const void *x, const void *gamma, const void *beta, void *y, float *mean, float *rstd, int B,
           int T, int D, lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *stream)
{
    if (!shape_ok(B, T, D) || !(eps >= 0.f)) return LNPEGN_EINVAL;
    if (!dtype_ok(dt) || !dtype_ok(gamma_dt)) return LNPEGN_EUNSUPPORTED;
    if (!x || !gamma || !beta || !y) return LNPEGN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    FwdArgs a{};
    a.x = x; a.gamma = gamma; a.beta = beta; a.y = y; a.mean = mean; a.rstd = rstd;
    a.N = (int64_t)B * T; a.D = D; a.gamma_is_f32 = gamma_dt == LNPEGN_F32; a.eps = eps;
    a.inv_D = 1.0f / (float)D;
    const bool vec = aligned16(x) && aligned16(y) && aligned16(gamma) && aligned16(beta);
    const hipError_t e = dt == LNPEGN_BF16 ? launch_fwd<bf16_t, true>(a, vec, s)
                                           : launch_fwd<float, true>(a, vec, s);
    return e == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

int ln_bwd(const void *x, const void *dy, const void *gamma, const float *mean, const float *rstd,
           void *dx, float *dgamma, float *dbeta, int B, int T, int D, lnpegn_dtype dt,
           lnpegn_dtype gamma_dt, float eps, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_bwd(false, false, false, false, x, dy, gamma, mean, rstd, dx, dgamma, dbeta, nullptr, nullptr, nullptr, B, T,
                   D, dt, gamma_dt, eps, workspace, workspace_bytes, stream);
}

int ln_bwd_pegn(const void *x, const void *dy, const void *gamma, const float *mean,
                const float *rstd, void *dx, float *dgamma, float *dbeta, float *pe_gamma_sq,
                float *pe_beta_sq, float *big_sq, int B, int T, int D, lnpegn_dtype dt,
                lnpegn_dtype gamma_dt, float eps, void *workspace, size_t workspace_bytes,
                void *stream)
{
    return run_bwd(true, false, false, false, x, dy, gamma, mean, rstd, dx, dgamma, dbeta, pe_gamma_sq, pe_beta_sq, big_sq,
                   B, T, D, dt, gamma_dt, eps, workspace, workspace_bytes, stream);
}

int ln_bwd_pegn_static(const void *x, const void *dy, const void *gamma, const float *mean, const float *rstd,
                       void *dx, float *dgamma, float *dbeta, float *pe_gamma_sq, float *pe_beta_sq, float *big_sq,
                       int B, int T, int D, lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *stream)
{
    // validate the shape against the fixed scratch before touching the device
    if (!shape_ok(B, T, D) || !(eps >= 0.f)) return LNPEGN_EINVAL;
    if (!dtype_ok(dt) || !dtype_ok(gamma_dt)) return LNPEGN_EUNSUPPORTED;
    const bool vector_ok = aligned16(x) && aligned16(dy) && aligned16(dx) && aligned16(gamma);
    if (make_plan(B, T, D, dt, true, vector_ok).total > kStaticScratchBytes) return LNPEGN_EWORKSPACE;
    void *ws = nullptr;
    const hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return LNPEGN_EHIP;
    }
    return run_bwd(true, false, false, false, x, dy, gamma, mean, rstd, dx, dgamma, dbeta, pe_gamma_sq, pe_beta_sq, big_sq,
                   B, T, D, dt, gamma_dt, eps, ws, kStaticScratchBytes, stream);
}

int ln_bwd_deferred(const void *x, const void *dy, const void *gamma, const float *mean,
                    const float *rstd, void *dx, float *dgamma, float *dbeta, int B, int T, int D,
                    lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    return run_bwd(false, true, false, false, x, dy, gamma, mean, rstd, dx, dgamma, dbeta, nullptr, nullptr, nullptr, B,
                   T, D, dt, gamma_dt, eps, workspace, workspace_bytes, stream);
}

int ln_bwd_pegn_deferred(const void *x, const void *dy, const void *gamma, const float *mean,
                         const float *rstd, void *dx, float *dgamma, float *dbeta,
                         float *pe_gamma_sq, float *pe_beta_sq, float *big_sq, int B, int T, int D,
                         lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *workspace,
                         size_t workspace_bytes, void *stream)
{
    return run_bwd(true, true, false, false, x, dy, gamma, mean, rstd, dx, dgamma, dbeta, pe_gamma_sq, pe_beta_sq,
                   big_sq, B, T, D, dt, gamma_dt, eps, workspace, workspace_bytes, stream);
}

int ln_bwd_ex(const void *x, const void *dy, const void *gamma, const float *mean, const float *rstd,
              void *dx, float *dgamma, float *dbeta, float *pe_gamma_sq, float *pe_beta_sq, float *big_sq,
              int B, int T, int D, lnpegn_dtype dt, lnpegn_dtype gamma_dt, float eps, void *workspace,
              size_t workspace_bytes, unsigned flags, void *stream)
{
    if (flags & ~(unsigned)(LNPEGN_PER_EXAMPLE | LNPEGN_DEFER | LNPEGN_ACCUMULATE)) return LNPEGN_EINVAL;
    const bool pegn = (flags & LNPEGN_PER_EXAMPLE) != 0;
    return run_bwd(pegn, (flags & LNPEGN_DEFER) != 0, (flags & LNPEGN_ACCUMULATE) != 0, false, x, dy, gamma, mean,
                   rstd, dx, dgamma, dbeta, pegn ? pe_gamma_sq : nullptr, pegn ? pe_beta_sq : nullptr,
                   pegn ? big_sq : nullptr, B, T, D, dt, gamma_dt, eps, workspace, workspace_bytes, stream);
}

int rms_fwd(const void *x, const void *gamma, void *y, float *rstd, int B, int T, int D, lnpegn_dtype dt,
            lnpegn_dtype gamma_dt, float eps, void *stream)
{
    if (!shape_ok(B, T, D) || !(eps >= 0.f)) return LNPEGN_EINVAL;
    if (!dtype_ok(dt) || !dtype_ok(gamma_dt)) return LNPEGN_EUNSUPPORTED;
    if (!x || !gamma || !y) return LNPEGN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    FwdArgs a{};
    a.x = x; a.gamma = gamma; a.beta = nullptr; a.y = y; a.mean = nullptr; a.rstd = rstd;
    a.N = (int64_t)B * T; a.D = D; a.gamma_is_f32 = gamma_dt == LNPEGN_F32; a.rms = 1; a.eps = eps;
    a.inv_D = 1.0f / (float)D;
    const bool vec = aligned16(x) && aligned16(y) && aligned16(gamma);
    const hipError_t e = dt == LNPEGN_BF16 ? launch_fwd<bf16_t, true>(a, vec, s)
                                           : launch_fwd<float, true>(a, vec, s);
    return e == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

int rms_bwd_ex(const void *x, const void *dy, const void *gamma, const float *rstd, void *dx, float *dgamma,
               float *pe_gamma_sq, float *big_sq, int B, int T, int D, lnpegn_dtype dt, lnpegn_dtype gamma_dt,
               float eps, void *workspace, size_t workspace_bytes, unsigned flags, void *stream)
{
    if (flags & ~(unsigned)(LNPEGN_PER_EXAMPLE | LNPEGN_DEFER | LNPEGN_ACCUMULATE)) return LNPEGN_EINVAL;
    const bool pegn = (flags & LNPEGN_PER_EXAMPLE) != 0;
    return run_bwd(pegn, (flags & LNPEGN_DEFER) != 0, (flags & LNPEGN_ACCUMULATE) != 0, true, x, dy, gamma,
                   nullptr, rstd, dx, dgamma, nullptr, pegn ? pe_gamma_sq : nullptr, nullptr,
                   pegn ? big_sq : nullptr, B, T, D, dt, gamma_dt, eps, workspace, workspace_bytes, stream);
}

int lnpegn_reduce_deferred(void *const *workspaces, int n, int B, int T, int D, lnpegn_dtype dt,
                           void *stream)
{
    if (!workspaces || n <= 0 || !shape_ok(B, T, D)) return LNPEGN_EINVAL;
    if (!dtype_ok(dt)) return LNPEGN_EUNSUPPORTED;
    for (int i = 0; i < n; ++i)
        if (!workspaces[i] || reinterpret_cast<uintptr_t>(workspaces[i]) % kAlign) return LNPEGN_EINVAL;
    const Plan p = make_plan(B, T, D, dt, true, true);   // the offsets used depend on B and D only
    const int g1_max = B + kGroups;     // an example each, then the groups
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int first = 0; first < n; first += kBatchMax) {
        BatchArgs b{};
        b.n = n - first < kBatchMax ? n - first : kBatchMax;
        for (int i = 0; i < b.n; ++i) b.ws[i] = static_cast<char *>(workspaces[first + i]);
        b.D = D; b.ntile = p.ntile;
        b.off_grp = p.off_grp; b.off_part_s = p.off_part_s; b.off_part_big = p.off_part_big;
        b.off_part = p.off_part;
        if (launch(reduce_groups_batch_kernel, dim3((unsigned)p.ntile, (unsigned)g1_max, (unsigned)b.n), dim3(kTile), 0, s, b) != hipSuccess) return LNPEGN_EHIP;
        if (launch(reduce_final_batch_kernel, dim3((unsigned)b.n), dim3(1024), 0, s, b) != hipSuccess) return LNPEGN_EHIP;
    }
    return LNPEGN_OK;
}

int gns_estimate(const float *pe_sq, const float *big_sq, int n_groups, int B, float pe_scale,
                 float *out, void *stream)
{
    if (!pe_sq || !big_sq || !out || n_groups <= 0 || B <= 1) return LNPEGN_EINVAL;
    return launch(gns_estimate_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream),  pe_sq, big_sq, n_groups, B, pe_scale, out) == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

int gns_ema_update(double *state, const float *records, int n, double alpha, float *smoothed, void *stream)
{
    if (!state || !records || n <= 0 || !(alpha >= 0.0 && alpha < 1.0)) return LNPEGN_EINVAL;
    return launch(gns_ema_update_kernel, dim3((n + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),  state, records, n, alpha, smoothed) == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

int gns_offline(const float *records, int64_t n, float *out, void *stream)
{
    if (!records || !out || n < 2) return LNPEGN_EINVAL;
    return launch(gns_offline_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), records, n, out) == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

int gns_linear_accum_steps(int64_t tokens_seen, int64_t ramp_tokens, int accum_final)
{
    if (tokens_seen < 0 || ramp_tokens < 0 || accum_final < 1) return -LNPEGN_EINVAL;
    if (ramp_tokens == 0 || tokens_seen >= ramp_tokens) return accum_final;
    const __int128 num = (__int128)accum_final * tokens_seen;
    const int64_t a = (int64_t)((num + ramp_tokens - 1) / ramp_tokens);
    return a < 1 ? 1 : (a > accum_final ? accum_final : (int)a);
}

int lnpegn_set_tuning(int key, int value)
{
    if (value < 0) return LNPEGN_EINVAL;
    switch (key) {
        case 0:
            if (value > kMaxChunks) return LNPEGN_EINVAL;
            g_chunks_pegn = value;
            return LNPEGN_OK;
        case 1:
            if (value > kMaxChunks) return LNPEGN_EINVAL;
            g_chunks_plain = value;
            return LNPEGN_OK;
        case 2:
            if (value > 16) return LNPEGN_EINVAL;
            g_waves = value;
            return LNPEGN_OK;
        case 3:
            g_stagger = value == 0 ? -1 : value - 1;
            return LNPEGN_OK;
        case 4:
            if (value > 2) return LNPEGN_EINVAL;
            g_xcd = value - 1;          // 0 automatic, 1 never, 2 always
            return LNPEGN_OK;
        case 5:
            if (value > 4) return LNPEGN_EINVAL;
            g_vpt_max = value;
            return LNPEGN_OK;
        case 6:
            if (value < 1 || value > 65535) return LNPEGN_EINVAL;
            g_emb_run_blocks = value;
            return LNPEGN_OK;
        case 7:
            if (value > 2) return LNPEGN_EINVAL;
            g_dx_cached = value - 1;
            return LNPEGN_OK;
        case 8:
            if (value > 2) return LNPEGN_EINVAL;
            g_blocked = value - 1;
            return LNPEGN_OK;
        default: return LNPEGN_EINVAL;
    }
}

int lnpegn_stream_probe(const void *a, const void *b, void *out, size_t bytes, int mode, void *stream)
{
    if (!a || !out || (mode >= 1 && !b) || bytes == 0 || bytes % 16) return LNPEGN_EINVAL;
    if (mode < 0 || mode > 2) return LNPEGN_EINVAL;
    if (!aligned16(a) || !aligned16(out) || (mode >= 1 && !aligned16(b))) return LNPEGN_EINVAL;
    const int64_t nvec = (int64_t)(bytes / 16);
    const int64_t blocks = mode == 2 ? (nvec + 255) / 256 : (nvec + 1023) / 1024;
    if (blocks > INT32_MAX) return LNPEGN_EINVAL;
    hipEvent_t ev_start = g_ev_start, ev_stop = g_ev_stop;
    g_ev_start = g_ev_stop = nullptr;
    const uint4 *pa = static_cast<const uint4 *>(a), *pb = static_cast<const uint4 *>(b);
    uint4 *po = static_cast<uint4 *>(out);
    int64_t n = nvec;
    void *args[] = {&pa, &pb, &po, &n};
    const void *fn = mode == 0   ? reinterpret_cast<const void *>(stream_probe_kernel<0>)
                     : mode == 1 ? reinterpret_cast<const void *>(stream_probe_kernel<1>)
                                 : reinterpret_cast<const void *>(stream_probe_oneshot_kernel);
    const hipError_t e = hipExtLaunchKernel(fn, dim3((unsigned)blocks), dim3(256), args, 0,
                                            static_cast<hipStream_t>(stream), ev_start, ev_stop, 0);
    return e == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

int lnpegn_set_profile_events(void *start_event, void *stop_event)
{
    if ((start_event == nullptr) != (stop_event == nullptr)) return LNPEGN_EINVAL;
    g_ev_start = static_cast<hipEvent_t>(start_event);
    g_ev_stop = static_cast<hipEvent_t>(stop_event);
    return LNPEGN_OK;
}

}  // extern "C"
