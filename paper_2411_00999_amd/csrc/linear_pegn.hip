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
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// Workgroup tile: (WM*MI*32) (k) x (WN*NI*32) (l) outputs, 64 positions t per stage, WM x WN waves, each
// wave MI x NI MFMA tiles of 32 x 32 (v_mfma_f32_32x32x16_bf16).
//
// A stage sits in LDS the way it sits in memory, [t][column]: 64 rows of x followed by 64 rows of g.
// It gets there by loads that write LDS directly (no registers in between), three stages deep: one
// being multiplied, one landed or landing, one just issued.  The MFMA operand of a lane is 8
// consecutive t of ONE column, i.e. a column of that layout; the transposing LDS read
// (ds_read_b64_tr_b16: 16 lanes read a 4 x 16 block as 4 rows, each lane receives one column of it)
// delivers exactly that, two reads per operand.  The four rows of such a block are a whole row pitch
// apart, which is a multiple of all banks, so the 16-byte chunks of row r are stored at chunk index
// c ^ 4*(r & 3); a direct-to-LDS load writes a wave's 64 chunks contiguously, so the swizzle is applied
// by choosing which chunk of memory each lane fetches.
constexpr int kBufs = 3, kMaxSplit = 64;
#define LIN_STR2(x) #x
#define LIN_STR(x) LIN_STR2(x)
#define LIN_XROW 512   // bytes per LDS row of x and of g, as literals for the assembly below
#define LIN_GROW 256

// kElem: bytes per element (2: bf16, 4: fp32).  A stage is 64 positions of bf16 or 32 of fp32: the same
// 48 KiB either way.
template <int WM, int WN, int MI, int NI, int kElem>
struct LinCfg {
    static constexpr int kWaves = WM * WN, kThreads = 64 * kWaves;
    static constexpr int kTileK = WM * MI * 32, kTileL = WN * NI * 32;
    static constexpr int kStageT = 128 / kElem;
    static constexpr int kXRow = kTileK * kElem, kGRow = kTileL * kElem;  // bytes per LDS row
    static constexpr int kXBytes = kStageT * kXRow, kGBytes = kStageT * kGRow;
    static constexpr int kStageBytes = kXBytes + kGBytes;
    static constexpr int kXLoads = kXBytes / 1024, kLoads = kStageBytes / 1024;   // direct loads of 1 KiB
    static constexpr int kLoadsPerWave = kLoads / kWaves;
    static_assert(kLoads % kWaves == 0, "loads must divide evenly over the waves");
    static_assert(kXRow >= 256 && kGRow >= 256 && kXRow <= 1024 && kGRow <= 1024, "row of 16..64 chunks");
    static_assert(kBufs * kStageBytes <= 160 * 1024, "three stages must fit in LDS");
};
// 8 waves (two per SIMD, so one can issue MFMAs while the other waits for LDS), each 64 x 64: 256 x 128
// per workgroup.  Measured against 4 waves of 128 x 64 (one per SIMD, fewer LDS reads per MFMA): the
// lone wave cannot cover its own LDS latency and is 30 % slower.
#define LIN_CFG 4, 2, 2, 2
typedef LinCfg<LIN_CFG, 2> Cfg;          // tile shape and wave count are the same for both element types
typedef LinCfg<LIN_CFG, 4> CfgF32;

struct LinArgs {
    const char *x;          // [B,T,K] bf16 or fp32
    const char *g;          // [B,T,L]
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

// One direct-to-LDS load: every active lane moves 16 bytes from base + voff to LDS address
// lds_addr + 16*lane.  Written in assembly so that the compiler does not know of it: it would make the
// wave wait for the data before the next barrier, and the point is to wait two stages later.
__device__ __forceinline__ void load_to_lds(uint32_t lds_addr, uint32_t voff, const void *base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
}

template <typename C, int WM, int WN, int MI, int NI, int kElem>
__device__ __forceinline__ void linear_pegn_body(const LinArgs &a)
{
    constexpr bool kF32 = kElem == 4;
    constexpr int kStageT = C::kStageT, kPerChunk = 16 / kElem;       // elements per 16-byte chunk
    constexpr int kWaves = C::kWaves, kLoadsPerWave = C::kLoadsPerWave, kStageBytes = C::kStageBytes;
    constexpr int kXRow = C::kXRow, kGRow = C::kGRow, kXBytes = C::kXBytes;
    constexpr int kXChunks = kXRow / 16, kGChunks = kGRow / 16;       // 16-byte chunks per row
    constexpr int kXRowsPerLoad = 64 / kXChunks, kGRowsPerLoad = 64 / kGChunks;
    __shared__ __align__(1024) unsigned char lds[kBufs * kStageBytes];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: branches on it are scalar
    const int ntiles = a.tiles_k * a.tiles_l;
    const int tile = xcd_spread(blockIdx.x, ntiles);
    const int split = blockIdx.y;
    const int k0 = (tile % a.tiles_k) * C::kTileK, l0 = (tile / a.tiles_k) * C::kTileL;
    const int b_begin = split * a.b_per_split;
    const int b_end = b_begin + a.b_per_split < a.B ? b_begin + a.b_per_split : a.B;
    const int nst = (a.T + kStageT - 1) / kStageT;
    const int nstages = (b_end - b_begin) * nst;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;

    // ---- loading: a stage is kLoads loads of 1 KiB; wave w issues loads w*kLoadsPerWave .. +kLoadsPerWave-1.
    // The first kXLoads are rows of x, the rest rows of g.  Per load and lane: the row and the chunk of
    // memory that belongs at this lane's LDS position.
    uint32_t voff[kLoadsPerWave];        // byte offset from the stage's first element of x (or g)
    int lrow[kLoadsPerWave];             // row within the stage
    bool lcol_ok[kLoadsPerWave];         // the chunk's columns exist (edge tiles)
#pragma unroll
    for (int n = 0; n < kLoadsPerWave; ++n) {
        const int i = wave * kLoadsPerWave + n;
        // fp32 operands are read back one element per lane along a row, which needs no swizzle
        if (i < C::kXLoads) {
            const int r = kXRowsPerLoad * i + lane / kXChunks;
            const int c = kF32 ? lane % kXChunks : (lane % kXChunks) ^ ((r & 3) << 2);
            lrow[n] = r;
            lcol_ok[n] = k0 + c * kPerChunk < a.K;
            voff[n] = (uint32_t)(((int64_t)r * a.K + c * kPerChunk) * kElem);
        } else {
            const int r = kGRowsPerLoad * (i - C::kXLoads) + lane / kGChunks;
            const int c = kF32 ? lane % kGChunks : (lane % kGChunks) ^ ((r & 3) << 2);
            lrow[n] = r;
            lcol_ok[n] = l0 + c * kPerChunk < a.L;
            voff[n] = (uint32_t)(((int64_t)r * a.L + c * kPerChunk) * kElem);
        }
    }
    // A workgroup whose tile lies inside the matrix, on examples that are whole stages long, never has
    // a lane without data: it issues the same number of loads per wave at every stage and may count on
    // that when it waits.  Any other workgroup masks lanes, zero-fills their chunks and waits for all.
    const bool regular = a.T % kStageT == 0 && k0 + C::kTileK <= a.K && l0 + C::kTileL <= a.L;
    // The stage to fetch next is tracked by two running pointers: rows are contiguous in memory, within
    // an example and from one example to the next, so a stage is 64 rows further unless it is the short
    // last stage of an example.
    int fs = 0;                                                // stage within the example
    const int last_rows = a.T - (nst - 1) * kStageT;           // rows of an example's last stage (64 if whole)
    const char *xs = a.x + ((int64_t)b_begin * a.T * a.K + k0) * kElem, *gs = a.g + ((int64_t)b_begin * a.T * a.L + l0) * kElem;
    auto fetch = [&](int buf) {
        const uint32_t dst = lds_base + buf * kStageBytes + wave * kLoadsPerWave * 1024;
        if (regular) {
#pragma unroll
            for (int n = 0; n < kLoadsPerWave; ++n)
                load_to_lds(dst + n * 1024, voff[n],
                            wave * kLoadsPerWave + n < C::kXLoads ? (const void *)xs : (const void *)gs);
        } else {
            const int rows_left = fs == nst - 1 ? last_rows : kStageT;
#pragma unroll
            for (int n = 0; n < kLoadsPerWave; ++n) {
                if (lcol_ok[n] && lrow[n] < rows_left)
                    load_to_lds(dst + n * 1024, voff[n],
                                wave * kLoadsPerWave + n < C::kXLoads ? (const void *)xs : (const void *)gs);
                else
                    *reinterpret_cast<u32x4_t *>(lds + buf * kStageBytes + (wave * kLoadsPerWave + n) * 1024 +
                                                 lane * 16) = u32x4_t{0u, 0u, 0u, 0u};
            }
        }
        const int rows = fs == nst - 1 ? last_rows : kStageT;
        xs += (int64_t)rows * a.K * kElem;
        gs += (int64_t)rows * a.L * kElem;
        fs = fs == nst - 1 ? 0 : fs + 1;
    };

    // ---- multiplying: wave (wm, wn) owns outputs k0 + wm*MI*32 .. , l0 + wn*NI*32 .. .
    // For a transposing read, lane s of a 16-lane group reads row s/4 of the block, columns 4*(s%4) .. +3;
    // group g of the wave takes columns (g%2)*16 .. +15 of the 32 and positions (g/2)*8 .. +7 of the 16.
    const int wm = wave % WM, wn = wave / WM;
    const int s16 = lane & 15, grp = lane >> 4;
    const int rr = (grp >> 1) * 8 + (s16 >> 2);                // row within the 16 positions (first of two reads)
    uint32_t a_addr[MI], b_addr[NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int q = (wm * MI + i) * 4 + (grp & 1) * 2 + ((s16 & 3) >> 1);
        a_addr[i] = rr * kXRow + ((q ^ ((s16 >> 2) << 2)) * 16) + (s16 & 1) * 8;
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int q = (wn * NI + i) * 4 + (grp & 1) * 2 + ((s16 & 3) >> 1);
        b_addr[i] = kXBytes + rr * kGRow + ((q ^ ((s16 >> 2) << 2)) * 16) + (s16 & 1) * 8;
    }
    f32x16_t acc[MI][NI], tot[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                acc[mi][ni][i] = 0.f;
                tot[mi][ni][i] = 0.f;
            }
    // The transposing reads are written in assembly: the compiler's own selection of that instruction
    // takes no immediate offset (two VALU additions per read), and here the reads of the next 16
    // positions are issued, with immediate offsets off four per-stage addresses, before the MFMAs of the
    // current 16 start.  A block first waits for the reads issued by the block before it; the operands
    // those delivered are passed through it ("+v") so that no MFMA using them can be moved above the wait.
    static_assert(MI == 2 && NI == 2, "the read blocks below are written for 2 x 2 MFMA tiles per wave");
    static_assert(kF32 || (kXRow == LIN_XROW && kGRow == LIN_GROW), "row pitches used in the assembly");
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
    struct Frags {
        u32x2_t a0l, a0h, a1l, a1h, b0l, b0h, b1l, b1h;
    };
#define LIN_READS(KK)                                                                                          \
    "ds_read_b64_tr_b16 %0, %8 offset:" LIN_STR((KK) * 16 * LIN_XROW) "\n\t"                                    \
    "ds_read_b64_tr_b16 %1, %8 offset:" LIN_STR((KK) * 16 * LIN_XROW + 4 * LIN_XROW) "\n\t"                      \
    "ds_read_b64_tr_b16 %2, %9 offset:" LIN_STR((KK) * 16 * LIN_XROW) "\n\t"                                    \
    "ds_read_b64_tr_b16 %3, %9 offset:" LIN_STR((KK) * 16 * LIN_XROW + 4 * LIN_XROW) "\n\t"                      \
    "ds_read_b64_tr_b16 %4, %10 offset:" LIN_STR((KK) * 16 * LIN_GROW) "\n\t"                                   \
    "ds_read_b64_tr_b16 %5, %10 offset:" LIN_STR((KK) * 16 * LIN_GROW + 4 * LIN_GROW) "\n\t"                     \
    "ds_read_b64_tr_b16 %6, %11 offset:" LIN_STR((KK) * 16 * LIN_GROW) "\n\t"                                   \
    "ds_read_b64_tr_b16 %7, %11 offset:" LIN_STR((KK) * 16 * LIN_GROW + 4 * LIN_GROW)
#define LIN_OUTS(F)                                                                                            \
    "=&v"(F.a0l), "=&v"(F.a0h), "=&v"(F.a1l), "=&v"(F.a1h), "=&v"(F.b0l), "=&v"(F.b0h), "=&v"(F.b1l), "=&v"(F.b1h)
#define LIN_KEEP(F)                                                                                            \
    "+v"(F.a0l), "+v"(F.a0h), "+v"(F.a1l), "+v"(F.a1h), "+v"(F.b0l), "+v"(F.b0h), "+v"(F.b1l), "+v"(F.b1h)
    auto mfmas = [&](const Frags &f) {
        const bf16x8_t fa[2] = {
            __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(f.a0l, f.a0h, 0, 1, 2, 3)),
            __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(f.a1l, f.a1h, 0, 1, 2, 3))};
        const bf16x8_t fb2[2] = {
            __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(f.b0l, f.b0h, 0, 1, 2, 3)),
            __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(f.b1l, f.b1h, 0, 1, 2, 3))};
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb2[ni], acc[mi][ni], 0, 0, 0);
    };
    auto multiply_bf16 = [&](int buf, bool refill, int refill_buf) {
        const uint32_t base = lds_base + buf * kStageBytes;
        const uint32_t pa0 = base + a_addr[0], pa1 = base + a_addr[1], pb0 = base + b_addr[0], pb1 = base + b_addr[1];
        Frags f0, f1;
        asm volatile(LIN_READS(0) : LIN_OUTS(f0) : "v"(pa0), "v"(pa1), "v"(pb0), "v"(pb1) : "memory");
        asm volatile(LIN_READS(1) : LIN_OUTS(f1) : "v"(pa0), "v"(pa1), "v"(pb0), "v"(pb1) : "memory");
        asm volatile("s_waitcnt lgkmcnt(8)" : LIN_KEEP(f0) : : "memory");
        mfmas(f0);
        asm volatile(LIN_READS(2) : LIN_OUTS(f0) : "v"(pa0), "v"(pa1), "v"(pb0), "v"(pb1) : "memory");
        if (refill) fetch(refill_buf);                         // stage st+2 goes out in the shadow of those MFMAs
        asm volatile("s_waitcnt lgkmcnt(8)" : LIN_KEEP(f1) : : "memory");
        mfmas(f1);
        asm volatile(LIN_READS(3) : LIN_OUTS(f1) : "v"(pa0), "v"(pa1), "v"(pb0), "v"(pb1) : "memory");
        asm volatile("s_waitcnt lgkmcnt(8)" : LIN_KEEP(f0) : : "memory");
        mfmas(f0);
        asm volatile("s_waitcnt lgkmcnt(0)" : LIN_KEEP(f1) : : "memory");
        mfmas(f1);
    };
#undef LIN_READS
#undef LIN_OUTS
#undef LIN_KEEP
    // fp32 operands (v_mfma_f32_32x32x2_f32: lane l holds row l%32 of A, column l%32 of B, position l/32 of
    // the two): one element per lane straight off a row of the stage, no transposition and no swizzle;
    // every read is one per-stage address plus an immediate.
    typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
    typedef __attribute__((address_space(3))) float lds_float_t;
    uint32_t fa_addr[MI], fb_addr[NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) fa_addr[i] = (lane >> 5) * kXRow + ((wm * MI + i) * 32 + (lane & 31)) * 4;
#pragma unroll
    for (int i = 0; i < NI; ++i) fb_addr[i] = kXBytes + (lane >> 5) * kGRow + ((wn * NI + i) * 32 + (lane & 31)) * 4;
    auto multiply_f32 = [&](int buf, bool refill, int refill_buf) {
        const lds_byte_t *base = (const lds_byte_t *)lds + buf * kStageBytes;
        const lds_byte_t *pa[MI], *pb[NI];
#pragma unroll
        for (int i = 0; i < MI; ++i) pa[i] = base + fa_addr[i];
#pragma unroll
        for (int i = 0; i < NI; ++i) pb[i] = base + fb_addr[i];
#pragma unroll
        for (int ks = 0; ks < kStageT / 2; ++ks) {
            float fa[MI], fb2[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[i] = *(const lds_float_t *)(pa[i] + ks * 2 * kXRow);
#pragma unroll
            for (int i = 0; i < NI; ++i) fb2[i] = *(const lds_float_t *)(pb[i] + ks * 2 * kGRow);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[mi], fb2[ni], acc[mi][ni], 0, 0, 0);
            if (ks == 1 && refill) fetch(refill_buf);          // stage st+2 goes out in the shadow of the MFMAs
        }
    };
    auto multiply = [&](int buf, bool refill, int refill_buf) {
        if constexpr (kF32) multiply_f32(buf, refill, refill_buf);
        else multiply_bf16(buf, refill, refill_buf);
    };
    int cb = b_begin, cs = 0;                                  // the stage being multiplied
    auto boundary = [&]() {
        if (++cs < nst) return;
        cs = 0;
        // example boundary: step 2 on this wave's part, then fold it into the total (step 3)
        float ssq = 0.f;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
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

    // ---- pipeline: before multiplying stage st a wave waits for its own loads of that stage (those of
    // stage st+1, issued later, may still be under way), the barrier then says that every wave's part has
    // landed and that stage st-1 has been read by all, so its buffer can take stage st+2.
    if (nstages > 0) fetch(0);
    if (nstages > 1) fetch(1);
    int cur = 0, nxt2 = 2;                                     // buffers of stage st and of stage st+2
    for (int st = 0; st < nstages; ++st) {
        if (regular && st + 1 < nstages)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerWave) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        multiply(cur, st + 2 < nstages, nxt2);
        cur = cur == kBufs - 1 ? 0 : cur + 1;
        nxt2 = nxt2 == kBufs - 1 ? 0 : nxt2 + 1;
        boundary();
    }

    // ---- write the total: lane holds rows (i/4)*8 + (lane/32)*4 + i%4, column lane%32 of each 32x32 tile
    float *out = a.out + (a.nsplit > 1 ? (int64_t)split * a.K * a.L : 0);
    double bsq = 0.0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int l = l0 + (wn * NI + ni) * 32 + (lane & 31);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int k = k0 + (wm * MI + mi) * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
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

template <int kElem>
__global__ __launch_bounds__(Cfg::kThreads) void linear_pegn_kernel(LinArgs a)
{
    linear_pegn_body<LinCfg<LIN_CFG, kElem>, LIN_CFG, kElem>(a);
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
    const int per_chunk = dt == LNPEGN_BF16 ? 8 : 4;          // elements per 16-byte vector
    p.mfma = K % per_chunk == 0 && L % per_chunk == 0 && aligned;
    if (p.mfma) {
        p.tiles_k = (K + Cfg::kTileK - 1) / Cfg::kTileK;
        p.tiles_l = (L + Cfg::kTileL - 1) / Cfg::kTileL;
        const int ntiles = p.tiles_k * p.tiles_l;
        // enough workgroups for 256 CUs: split the examples when the output has few tiles
        int want = (256 + ntiles - 1) / ntiles;
        if (want > B) want = B;
        if (want > kMaxSplit) want = kMaxSplit;
        p.b_per_split = (B + want - 1) / want;
        p.nsplit = (B + p.b_per_split - 1) / p.b_per_split;
        p.nparts = ntiles * Cfg::kWaves;
        p.nbig = p.nsplit == 1 ? (int64_t)ntiles * Cfg::kWaves : ((int64_t)K * L + 255) / 256;
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
        a.x = static_cast<const char *>(x);
        a.g = static_cast<const char *>(g);
        a.out = p.nsplit > 1 ? part_w : w;
        a.tile_s = part_s;
        a.tile_big = part_big;
        a.B = B; a.T = T; a.K = K; a.L = L;
        a.tiles_k = p.tiles_k; a.tiles_l = p.tiles_l; a.nsplit = p.nsplit; a.b_per_split = p.b_per_split;
        a.accumulate = accumulate;
        const dim3 grid(p.tiles_k * p.tiles_l, p.nsplit), block(Cfg::kThreads);
        if ((dt == LNPEGN_BF16 ? launch(linear_pegn_kernel<2>, grid, block, 0, st, a)
                               : launch(linear_pegn_kernel<4>, grid, block, 0, st, a)) != hipSuccess)
            return LNPEGN_EHIP;
        if (p.nsplit > 1) {
            const int64_t n = (int64_t)K * L;
            if (launch(linear_sum_splits_kernel, dim3((unsigned)p.nbig), dim3(256), 0, st, part_w, w, part_big, n, p.nsplit, accumulate) != hipSuccess) return LNPEGN_EHIP;
        }
    } else {
        const dim3 grid(p.tiles_l, p.tiles_k);
        const hipError_t e =
            dt == LNPEGN_BF16
                ? launch(linear_pegn_generic_kernel<bf16_t>, grid, dim3(256), 0, st, static_cast<const bf16_t *>(x),
                         static_cast<const bf16_t *>(g), w, part_s, part_big, B, T, K, L, accumulate)
                : launch(linear_pegn_generic_kernel<float>, grid, dim3(256), 0, st, static_cast<const float *>(x),
                         static_cast<const float *>(g), w, part_s, part_big, B, T, K, L, accumulate);
        if (e != hipSuccess) return LNPEGN_EHIP;
    }
    return launch(linear_final_kernel, dim3(B + 1), dim3(1024), 0, st, part_s, p.nparts, part_big, p.nbig, s, big_sq, B) == hipSuccess ? LNPEGN_OK : LNPEGN_EHIP;
}

}  // extern "C"
