// Launchers of the kernel families that are compiled as translation units of their own (one per
// instantiation group, so that they build in parallel and a change to one family recompiles only it).
// Each returns the HIP error of its launch.
#pragma once
#include <hip/hip_runtime.h>

namespace csat {

struct IstaFusedArgs;
struct AttentionArgs;

// Fused ISTA decoder for MT tiles of m (csat_ista_fused.h, csat_ista_fused2.h).  variant: 0 dense state, 1 sparse
// state, 2 one 32-row tile per workgroup (thin); 3 and 4: dense and sparse state on the two-chunk schedule.  One function per MT, defined by csat_tu_ista_fused.hip
// compiled with -DCSAT_TU_MT=<MT>.
#define CSAT_DECLARE_FUSED(MT_) \
    hipError_t ista_fused_launch_mt##MT_(int variant, const IstaFusedArgs& a, unsigned grid, hipStream_t st);
CSAT_DECLARE_FUSED(1) CSAT_DECLARE_FUSED(2) CSAT_DECLARE_FUSED(3) CSAT_DECLARE_FUSED(4) CSAT_DECLARE_FUSED(5)
CSAT_DECLARE_FUSED(6) CSAT_DECLARE_FUSED(7) CSAT_DECLARE_FUSED(8) CSAT_DECLARE_FUSED(9) CSAT_DECLARE_FUSED(10)
CSAT_DECLARE_FUSED(11) CSAT_DECLARE_FUSED(12) CSAT_DECLARE_FUSED(13) CSAT_DECLARE_FUSED(14) CSAT_DECLARE_FUSED(15)
CSAT_DECLARE_FUSED(16)
#undef CSAT_DECLARE_FUSED

// Compressed attention in one kernel (csat_attention.h) for mt_total tiles of m; `single`: all of K~ is kept in
// registers and LDS at once.  One function per element type and per "with the output product", defined by
// csat_tu_attention.hip compiled with -DCSAT_TU_BF16=<0|1> -DCSAT_TU_Z=<0|1>.
hipError_t attention_fused_launch_f32_z0(int mt_total, bool single, const AttentionArgs& a, unsigned grid, size_t lds_bytes, hipStream_t st);
hipError_t attention_fused_launch_f32_z1(int mt_total, bool single, const AttentionArgs& a, unsigned grid, size_t lds_bytes, hipStream_t st);
hipError_t attention_fused_launch_bf16_z0(int mt_total, bool single, const AttentionArgs& a, unsigned grid, size_t lds_bytes, hipStream_t st);
hipError_t attention_fused_launch_bf16_z1(int mt_total, bool single, const AttentionArgs& a, unsigned grid, size_t lds_bytes, hipStream_t st);
// ... with the output product from V~ as packed fragments (a.Vf), d = 64 (z2) or 128 (z3)
hipError_t attention_fused_launch_bf16_z2(int mt_total, bool single, const AttentionArgs& a, unsigned grid, size_t lds_bytes, hipStream_t st);
hipError_t attention_fused_launch_bf16_z3(int mt_total, bool single, const AttentionArgs& a, unsigned grid, size_t lds_bytes, hipStream_t st);

}  // namespace csat
