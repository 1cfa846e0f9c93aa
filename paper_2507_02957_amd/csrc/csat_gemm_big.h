// Large-tile bf16 "NT" GEMM for the decoder's per-iteration GEMM pair when the fused decoder does
// not apply and for any other big bf16 contraction:  C[M,N] = sum_k A[M,k] * Bt[N,k].
//
// A workgroup of WM x WN wavefronts computes a (64*WM) x (128*WN) tile; each wavefront owns
// 64 x 128 = 2 x 4 MFMA tiles (128 accumulator registers) and reads 6 fragments per 8 MFMAs.
// Operand tiles are staged by direct global->LDS loads, KS columns of K per step, one request =
// 1 KB = 512/KS rows; the 16-byte slot of a row is XOR-swizzled with (row/2) so that the
// fragment reads of consecutive rows fall in different bank groups.  Two LDS stages.
//
// The shape in use is <4, 2, 64>: 256 x 256 tile, 8 wavefronts (two per SIMD, so one wavefront's
// staging requests and LDS waits are covered by the other's MFMAs), 128 KB of stages, one
// workgroup per CU.  <4, 1, 32> (256 x 128, two workgroups per CU) also instantiates.
//
// GemmArgs::a_kwrap carries the number of column tiles here (the grid is 1-D over tiles).
// Contract: K is a multiple of 64 (operands zero-padded to it), row pointers 16-byte aligned.
// Rows >= M / >= N are clamped to the last valid row (their products are discarded or overwritten
// by the epilogue's own bounds handling).
#pragma once
#include "csat_kernels.h"

namespace csat {

template <typename E, bool = has_tile_epilogue<E>::value> struct TilePre { struct type {}; };
template <typename E> struct TilePre<E, true> { using type = typename E::Pre; };
template <typename E>
__device__ __forceinline__ typename TilePre<E>::type tile_begin(const E& epi, long long r0w, long long c0w, int lane) {
    if constexpr (has_tile_epilogue<E>::value) return epi.begin(r0w, c0w, lane);
    else return {};
}

template <typename Epi, int WM, int WN, int KS>
struct BigGemmShape {
    static constexpr int kWaves = WM * WN, kThreads = 64 * kWaves;
    static constexpr int kRowsA = 64 * WM, kRowsB = 128 * WN;
    static constexpr int kRowBytes = 2 * KS;                       // one operand row of a stage
    static constexpr int kStage = (kRowsA + kRowsB) * kRowBytes;
    static constexpr int kOffB = kRowsA * kRowBytes;
    static constexpr size_t epilogue_bytes() {
        if constexpr (has_tile_epilogue<Epi>::value) return (size_t)kWaves * Epi::kStageBytes;
        else return 0;
    }
    static constexpr size_t kLdsBytes = 2 * kStage > epilogue_bytes() ? 2 * kStage : epilogue_bytes();
};

template <typename Epi, int WM, int WN, int KS>
__global__ __launch_bounds__(64 * WM * WN, 8 / (WM * WN)) void gemm_nt_bf16_big_kernel(GemmArgs g, Epi epi) {
    using S = BigGemmShape<Epi, WM, WN, KS>;
    constexpr int CPR = S::kRowBytes / 16;           // 16-byte chunks per staged row
    constexpr int RPB = 64 / CPR;                    // rows per 1 KB request
    constexpr int BLOCKS_A = S::kRowsA / RPB, BLOCKS = (S::kRowsA + S::kRowsB) / RPB;
    constexpr int BPW = BLOCKS / S::kWaves;          // requests per wavefront and stage
    constexpr int NGK = KS / 16;                     // MFMA k-slices per stage
    static_assert(BLOCKS % S::kWaves == 0, "requests must divide evenly over the wavefronts");
    static_assert(NGK == 2 || NGK == 4, "KS is 32 or 64");
    extern __shared__ uint4 lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lh = lane >> 5;
    const int z = blockIdx.z;
    // raster 0: blockIdx.x enumerates tiles column-fastest.  Workgroups go to the 8 XCDs (each with its
    // own L2) round-robin by index, so XCD x sees the column tiles x, x+8, ... of every row tile: right
    // when there are many column tiles (the column operand's share stays in that L2).
    // raster 1: all column tiles of a row tile run on one XCD (consecutive slots of that XCD), row tiles
    // round-robin over the XCDs: the A rows are fetched into one L2 instead of one per column tile, and
    // the workgroups of an XCD walk K of the column operand together.  Right for few column tiles.
    long long rowt, colt;
    const bool a_nt = (g.raster & kRasterStreamA) != 0;      // uniform: A rows go past the caches' recently-used end
    g.raster &= kRasterStreamA - 1;
    if (g.raster == 1) {
        const int slot = blockIdx.x >> 3;
        rowt = (long long)(slot / g.a_kwrap) * 8 + (blockIdx.x & 7);
        colt = slot % g.a_kwrap;
        if (rowt * S::kRowsA >= g.M) return;       // the grid is padded to whole groups of 8 row tiles
    } else if (g.raster >= 2) {
        // raster 2 + log2(CB): XCD x owns the column tiles [x tn/8, (x+1) tn/8) and walks them in groups of CB: within a
        // group row tile by row tile, so that the group's column operand (CB x 512 KB at K = 1024) stays in that L2
        // for the whole pass over the rows and a row tile's A panel is shared by CB workgroups running together.
        const int cb = 1 << (g.raster - 2), per_xcd = g.a_kwrap >> 3;
        const long long tm = gridDim.x / g.a_kwrap;
        const long long slot = blockIdx.x >> 3;
        const long long cg = slot / (tm * cb), rem = slot - cg * tm * cb;
        rowt = rem / cb;
        colt = (long long)(blockIdx.x & 7) * per_xcd + cg * cb + rem % cb;
    } else {
        rowt = blockIdx.x / g.a_kwrap;
        colt = blockIdx.x % g.a_kwrap;
    }
    const long long row0 = rowt * S::kRowsA, col0 = colt * S::kRowsB;
    const bf16_t* A = (const bf16_t*)g.A + (long long)z * g.strideA;
    const bf16_t* Bt = (const bf16_t*)g.Bt + (long long)z * g.strideB;
    const int ksteps = g.K / KS;
    const uint32_t lds0 = (uint32_t)(size_t)(lds_ptr_t)lds;

    // staging: this wavefront requests blocks wave*BPW .. wave*BPW+BPW-1 of the stage (A rows first,
    // then Bt rows).  Lane l: row l/CPR of the block, LDS slot l%CPR, which holds the row's 16-byte
    // chunk (l%CPR) ^ ((row/2)&(CPR-1)).
    const int drow = lane / CPR, dslot = lane % CPR;
    const bf16_t* src[BPW];
#pragma unroll
    for (int b = 0; b < BPW; ++b) {
        const int blk = wave * BPW + b;
        const bool isA = blk < BLOCKS_A;                           // uniform
        const int r = (isA ? blk : blk - BLOCKS_A) * RPB + drow;   // row inside the operand tile
        const int chunk = dslot ^ ((r >> 1) & (CPR - 1));
        long long gr = (isA ? row0 : col0) + r;
        const long long lim = isA ? g.M : g.N;
        if (gr >= lim) gr = lim - 1;
        src[b] = (isA ? A + gr * g.lda : Bt + gr * g.ldb) + chunk * 8;
    }
    auto stage = [&](int ks, int st) {
        char* dst = (char*)lds + st * S::kStage + wave * BPW * 1024;
#pragma unroll
        for (int b = 0; b < BPW; ++b) {
            if (a_nt && wave * BPW + b < BLOCKS_A)
                __builtin_amdgcn_global_load_lds((glb_ptr_t)(src[b] + (long long)ks * KS), (lds_ptr_t)(dst + b * 1024), 16, 0, 2);
            else
                __builtin_amdgcn_global_load_lds((glb_ptr_t)(src[b] + (long long)ks * KS), (lds_ptr_t)(dst + b * 1024), 16, 0, 0);
        }
    };

    // fragment addresses: row (tile base + li), 16-byte slot ((2*gk + lh) ^ ((li/2)&(CPR-1))) for k-slice gk
    uint32_t adA[NGK], adB[NGK];
#pragma unroll
    for (int gk = 0; gk < NGK; ++gk) {
        const uint32_t slot = (uint32_t)((2 * gk + lh) ^ ((li >> 1) & (CPR - 1))) * 16;
        adA[gk] = lds0 + (wm * 64 + li) * S::kRowBytes + slot;
        adB[gk] = lds0 + S::kOffB + (wn * 128 + li) * S::kRowBytes + slot;
    }

    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    if constexpr (has_acc_init<Epi>::value) epi.init(row0 + wm * 64, col0 + wn * 128, lane, acc);

    stage(0, 0);
    typename TilePre<Epi>::type pre = tile_begin(epi, row0 + wm * 64, col0 + wn * 128, lane);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        const uint32_t so = (ks & 1) * S::kStage;
        // the two wavefronts of a SIMD issue their staging requests at different points of the step
        // (the first at the top, the second after its second MFMA group): requests issued by both
        // at once leave the MFMA pipe idle
        const bool more = ks + 1 < ksteps;
        const bool early = wave < S::kWaves / 2;
        if (more && early) stage(ks + 1, (ks + 1) & 1);
        u32x4 fa[2][2], fb[2][4];
        auto fetch = [&](auto gkc) {
            constexpr int gk = decltype(gkc)::value;
            constexpr int T32 = 32 * S::kRowBytes;        // 32 rows further
            lds_read16<0>(fa[gk & 1][0], adA[gk] + so);
            lds_read16<T32>(fa[gk & 1][1], adA[gk] + so);
            lds_read16<0>(fb[gk & 1][0], adB[gk] + so);
            lds_read16<T32>(fb[gk & 1][1], adB[gk] + so);
            lds_read16<2 * T32>(fb[gk & 1][2], adB[gk] + so);
            lds_read16<3 * T32>(fb[gk & 1][3], adB[gk] + so);
        };
        auto compute = [&](auto gkc) {
            constexpr int gk = decltype(gkc)::value;
            if constexpr (gk + 1 < NGK) {
                fetch(std::integral_constant<int, gk + 1>{});
                asm volatile("s_waitcnt lgkmcnt(6)"
                             : "+v"(fa[gk & 1][0]), "+v"(fa[gk & 1][1]), "+v"(fb[gk & 1][0]), "+v"(fb[gk & 1][1]),
                               "+v"(fb[gk & 1][2]), "+v"(fb[gk & 1][3]));
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)"
                             : "+v"(fa[gk & 1][0]), "+v"(fa[gk & 1][1]), "+v"(fb[gk & 1][0]), "+v"(fb[gk & 1][1]),
                               "+v"(fb[gk & 1][2]), "+v"(fb[gk & 1][3]));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[gk & 1][i]),
                                                                        __builtin_bit_cast(bf16x8, fb[gk & 1][j]), acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (gk == 1) {
                if (more && !early) stage(ks + 1, (ks + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        fetch(std::integral_constant<int, 0>{});
        compute(std::integral_constant<int, 0>{});
        compute(std::integral_constant<int, 1>{});
        if constexpr (NGK == 4) {
            compute(std::integral_constant<int, 2>{});
            compute(std::integral_constant<int, 3>{});
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }

    // accumulator layout of the 32x32 MFMA: lane (li, lh), register v holds row 8*(v/4) + 4*lh + (v%4), column li
    if constexpr (has_tile_epilogue<Epi>::value) {
        // the stages are free now (last barrier passed): each wavefront takes a private piece
        char* stage_w = (char*)lds + wave * Epi::kStageBytes;
        const long long r0w = row0 + wm * 64, c0w = col0 + wn * 128;
        if constexpr (has_whole_epilogue<Epi>::value) {
            epi.whole(r0w, c0w, lane, acc, stage_w, pre);
        } else {
            epi.half(0, r0w, c0w, lane, acc[0], stage_w, pre);
            epi.half(1, r0w + 32, c0w, lane, acc[1], stage_w, pre);
        }
        epi.flush(r0w, c0w, lane, stage_w);
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const long long rt0 = row0 + wm * 64 + i * 32, ct0 = col0 + wn * 128 + j * 32;
#pragma unroll
                for (int v = 0; v < 16; ++v) epi(z, rt0 + 8 * (v / 4) + 4 * lh + (v % 4), ct0 + li, acc[i][j][v]);
            }
    }
}

}  // namespace csat
