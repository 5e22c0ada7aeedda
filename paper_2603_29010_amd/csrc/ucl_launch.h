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

template <class Cfg>
constexpr VariantDesc describe() {
    return VariantDesc{Cfg::TM, Cfg::TN, Cfg::TK, Cfg::STAGES, Cfg::DT, Cfg::MODE, Cfg::LA, Cfg::LB,
                       Cfg::LDS_BYTES, Cfg::PERSIST ? 1 : 0, Cfg::MIN_WAVES, &launch_cfg<Cfg>};
}

}  // namespace ucl
