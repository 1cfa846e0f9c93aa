// Translation unit of the fused ISTA decoder for one value of MT (tiles of m): compile with -DCSAT_TU_MT=<1..16>.
#include "csat_ista_fused.h"
#include "csat_ista_fused2.h"
#include "csat_launch.h"

#ifndef CSAT_TU_MT
#error "compile with -DCSAT_TU_MT=<tiles of m>"
#endif
#define CSAT_CAT2(a, b) a##b
#define CSAT_CAT(a, b) CSAT_CAT2(a, b)

namespace csat {

hipError_t CSAT_CAT(ista_fused_launch_mt, CSAT_TU_MT)(int variant, const IstaFusedArgs& a, unsigned grid, hipStream_t st) {
    constexpr int MT = CSAT_TU_MT;
    const size_t lds_bytes = variant >= 3 ? ista_fused2_lds_bytes(MT) : ista_fused_lds_bytes(MT);
    auto launch = [&](auto kernel) -> hipError_t {
        const hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), lds_bytes, st, a);
        return hipGetLastError();
    };
    if constexpr (MT >= 3 && MT <= 13) {      // (the two-chunk schedule: three to thirteen tiles of m)
        if (variant == 4) return launch(ista_fused2_kernel<MT, true>);
        if (variant == 3) return launch(ista_fused2_kernel<MT, false>);
    } else if (variant >= 3) {
        return hipErrorInvalidValue;
    }
    if (variant == 2) return launch(ista_fused_kernel<MT, false, true>);
    if (variant == 1) return launch(ista_fused_kernel<MT, true, false>);
    return launch(ista_fused_kernel<MT, false, false>);
}

}  // namespace csat
