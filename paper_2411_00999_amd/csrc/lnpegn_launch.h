// Launch interface between the C ABI (lnpegn.hip) and the row-kernel instantiations, which are
// compiled as four translation units (storage type x saved/recomputed statistics) from
// lnpegn_rows_inst.hip so that they build side by side.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lnpegn_rows.h"

namespace lnpegn {

// The part of a launch plan the row kernels' dispatch needs.
struct RowShape {
    bool plain;       // no per-example outputs: the plain backward's kernel
    bool fast;        // vectorised kernels (else the generic kernel)
    bool dx_cached;   // dx stored write-back instead of streaming
    int vpt;          // 16-byte vectors per lane
    int S, R;         // waves per row, row groups per workgroup
    int nvec;
    int64_t n_slots;  // chunks = workgroups
    size_t lds_bytes;
};

// One launch of a row kernel.  When profiling events are given they are attached to this very
// dispatch, so their elapsed time is the kernel's own execution time.
struct RowLaunch {
    hipStream_t stream;
    hipEvent_t ev_start, ev_stop;
};

hipError_t launch_rows_bf16_saved(const RowShape &p, const RowArgs &a, const RowLaunch &rl);
hipError_t launch_rows_bf16_recompute(const RowShape &p, const RowArgs &a, const RowLaunch &rl);
hipError_t launch_rows_f32_saved(const RowShape &p, const RowArgs &a, const RowLaunch &rl);
hipError_t launch_rows_f32_recompute(const RowShape &p, const RowArgs &a, const RowLaunch &rl);

}  // namespace lnpegn
