// One quarter of the row-kernel instantiations: compiled four times, with
//   -DLNPEGN_INST_BF16=0|1   storage type of x, dy, dx (fp32 | bf16)
//   -DLNPEGN_INST_SAVED=0|1  row statistics recomputed | taken from ln_fwd_stats
// each defining the launch function of that quarter (lnpegn_launch.h).
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include "lnpegn_launch.h"

#if !defined(LNPEGN_INST_BF16) || !defined(LNPEGN_INST_SAVED)
#error "compile with -DLNPEGN_INST_BF16=0|1 -DLNPEGN_INST_SAVED=0|1"
#endif

namespace lnpegn {
namespace {

#if LNPEGN_INST_BF16
using InstT = bf16_t;
#else
using InstT = float;
#endif
constexpr bool kInstSaved = LNPEGN_INST_SAVED != 0;

template <typename K>
hipError_t launch_row_kernel(K kernel, dim3 grid, dim3 block, size_t lds, const RowLaunch &rl,
                             const RowArgs &a)
{
    RowArgs copy = a;
    void *args[] = {&copy};
    if (rl.ev_start)
        return hipExtLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, args, lds,
                                  rl.stream, rl.ev_start, rl.ev_stop, 0);
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, args, lds, rl.stream);
}

template <int kVpt, int kS, bool kFull>
hipError_t launch_variant(const RowShape &p, const RowArgs &a, const RowLaunch &rl)
{
    const dim3 grid((unsigned)p.n_slots), block(64 * p.R * p.S);
    auto go = [&](auto kernel) { return launch_row_kernel(kernel, grid, block, p.lds_bytes, rl, a); };
    if (p.plain)
        return p.dx_cached ? go(ln_bwd_plain_rows_kernel<InstT, kVpt, kInstSaved, kS, kFull, true>)
                           : go(ln_bwd_plain_rows_kernel<InstT, kVpt, kInstSaved, kS, kFull, false>);
    return p.dx_cached ? go(ln_bwd_rows_kernel<InstT, kVpt, kInstSaved, kS, kFull, true>)
                       : go(ln_bwd_rows_kernel<InstT, kVpt, kInstSaved, kS, kFull, false>);
}

template <int kVpt>
hipError_t launch_vpt(const RowShape &p, const RowArgs &a, const RowLaunch &rl)
{
    const bool full = p.nvec == 64 * p.S * kVpt;
    switch (p.S) {
        case 1: return full ? launch_variant<kVpt, 1, true>(p, a, rl) : launch_variant<kVpt, 1, false>(p, a, rl);
        case 2: return full ? launch_variant<kVpt, 2, true>(p, a, rl) : launch_variant<kVpt, 2, false>(p, a, rl);
        case 4: return full ? launch_variant<kVpt, 4, true>(p, a, rl) : launch_variant<kVpt, 4, false>(p, a, rl);
        case 8: return full ? launch_variant<kVpt, 8, true>(p, a, rl) : launch_variant<kVpt, 8, false>(p, a, rl);
        default: return full ? launch_variant<kVpt, 0, true>(p, a, rl) : launch_variant<kVpt, 0, false>(p, a, rl);
    }
}

hipError_t launch_inst(const RowShape &p, const RowArgs &a, const RowLaunch &rl)
{
    if (!p.fast)
        return launch_row_kernel(ln_bwd_rows_generic_kernel<InstT, kInstSaved>, dim3((unsigned)p.n_slots),
                                 dim3(256), 0, rl, a);
    // up to 16 elements per lane (2 vectors of 8 bf16, 4 vectors of 4 fp32) at any number of waves per row;
    // 24 or 32 elements per lane only for rows of eight waves (D > 8192)
    constexpr int kBase = 16 / Vec<InstT>::kElems;
    if (p.vpt > kBase) {
        if (p.S != 8) return hipErrorInvalidValue;
        const bool full = p.nvec == 64 * 8 * p.vpt;
#define LNPEGN_WIDE(V) \
    case V: return full ? launch_variant<V, 8, true>(p, a, rl) : launch_variant<V, 8, false>(p, a, rl)
        switch (p.vpt) {
            LNPEGN_WIDE(kBase + 1);
            LNPEGN_WIDE(kBase + 2);
            default: break;
        }
        if constexpr (kBase == 4) {
            switch (p.vpt) {
                LNPEGN_WIDE(7);
                LNPEGN_WIDE(8);
                default: break;
            }
        }
#undef LNPEGN_WIDE
        return hipErrorInvalidValue;
    }
    if constexpr (Vec<InstT>::kElems == 4) {
        if (p.vpt == 3) return launch_vpt<3>(p, a, rl);
        if (p.vpt == 4) return launch_vpt<4>(p, a, rl);
    }
    if (p.vpt == 1) return launch_vpt<1>(p, a, rl);
    if (p.vpt == 2) return launch_vpt<2>(p, a, rl);
    return hipErrorInvalidValue;
}

}  // namespace

#if LNPEGN_INST_BF16 && LNPEGN_INST_SAVED
hipError_t launch_rows_bf16_saved(const RowShape &p, const RowArgs &a, const RowLaunch &rl) { return launch_inst(p, a, rl); }
#elif LNPEGN_INST_BF16
hipError_t launch_rows_bf16_recompute(const RowShape &p, const RowArgs &a, const RowLaunch &rl) { return launch_inst(p, a, rl); }
#elif LNPEGN_INST_SAVED
hipError_t launch_rows_f32_saved(const RowShape &p, const RowArgs &a, const RowLaunch &rl) { return launch_inst(p, a, rl); }
#else
hipError_t launch_rows_f32_recompute(const RowShape &p, const RowArgs &a, const RowLaunch &rl) { return launch_inst(p, a, rl); }
#endif

}  // namespace lnpegn
