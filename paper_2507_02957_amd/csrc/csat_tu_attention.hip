// Translation unit of the one-kernel compressed attention for one element type, with or without the output
// product: compile with -DCSAT_TU_BF16=<0|1> -DCSAT_TU_Z=<0|1|2|3> (2, 3: bf16 only, the product from packed fragments
// of V~ for d = 64 / 128).
#include "csat_attention.h"
#include "csat_launch.h"

#if !defined(CSAT_TU_BF16) || !defined(CSAT_TU_Z)
#error "compile with -DCSAT_TU_BF16=<0|1> -DCSAT_TU_Z=<0|1|2|3>"
#endif
#if CSAT_TU_BF16 && CSAT_TU_Z == 3
#define CSAT_TU_FN attention_fused_launch_bf16_z3
#elif CSAT_TU_BF16 && CSAT_TU_Z == 2
#define CSAT_TU_FN attention_fused_launch_bf16_z2
#elif CSAT_TU_BF16 && CSAT_TU_Z
#define CSAT_TU_FN attention_fused_launch_bf16_z1
#elif CSAT_TU_BF16
#define CSAT_TU_FN attention_fused_launch_bf16_z0
#elif CSAT_TU_Z
#define CSAT_TU_FN attention_fused_launch_f32_z1
#else
#define CSAT_TU_FN attention_fused_launch_f32_z0
#endif

namespace csat {

hipError_t CSAT_TU_FN(int mt, bool single, const AttentionArgs& a, unsigned grid, size_t lds_bytes, hipStream_t st) {
#if CSAT_TU_BF16
    typedef bf16_t T;
#else
    typedef float T;
#endif
    constexpr int Z = CSAT_TU_Z;
    auto launch = [&](auto kernel, int waves) -> hipError_t {
        const hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * waves), lds_bytes, st, a);
        return hipGetLastError();
    };
#define CSAT_ATTN(MTP_, SINGLE_) launch(attention_fused_kernel<T, MTP_, SINGLE_, Z>, attention_waves(MTP_, Z))
    switch (attention_mtp(mt, single)) {
        case 1: return CSAT_ATTN(1, true);
        case 2: return CSAT_ATTN(2, true);
        case 4: return CSAT_ATTN(4, true);
        case 8:
            if (single) return CSAT_ATTN(8, true);
            // (the two-sweep form with the product from packed fragments is not built: the host leaves Z to a product GEMM there)
            if constexpr (Z >= 2) return hipErrorInvalidValue;
            else return CSAT_ATTN(kAttnPanelTiles, false);
        case 13: return CSAT_ATTN(13, true);
        default: return CSAT_ATTN(16, true);
    }
#undef CSAT_ATTN
}

}  // namespace csat
