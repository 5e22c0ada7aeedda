// Host-side launcher template, included by the instantiation units next to the kernel.
#pragma once
#include "ucl_kernel.h"
#include "ucl_variants.h"

namespace ucl {

template <class Cfg>
hipError_t launch_cfg(const KParams &p, const GroupTable *gt, int grid, hipStream_t stream) {
    if constexpr (Cfg::MODE == 1) {
        hipLaunchKernelGGL(ucl_tile_kernel<Cfg>, dim3(grid), dim3(kThreads), 0, stream, p, *gt);
    } else {
        (void)gt;
        hipLaunchKernelGGL(ucl_tile_kernel<Cfg>, dim3(grid), dim3(kThreads), 0, stream, p, NoGroupTable{});
    }
    return hipGetLastError();
}

// Workgroups of the variant that one CU holds at a time, as the runtime computes it from the registers and
// LDS the compiled kernel uses (a host-side query, asked once: no device work, no allocation).
template <class Cfg>
int resident_cfg() {
    static const int cached = [] {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, ucl_tile_kernel<Cfg>, kThreads, 0) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = 1;
        }
        return n;
    }();
    return cached;
}

template <class Cfg>
constexpr VariantDesc describe() {
    return VariantDesc{Cfg::TM, Cfg::TN, Cfg::TK, Cfg::STAGES, Cfg::DT, Cfg::MODE, Cfg::LA, Cfg::LB,
                       Cfg::LDS_BYTES, Cfg::SCHED, Cfg::MIN_WAVES, Cfg::HALO ? Cfg::PATCH_C : 0, &launch_cfg<Cfg>, &resident_cfg<Cfg>};
}

}  // namespace ucl
