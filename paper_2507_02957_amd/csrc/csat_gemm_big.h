// Large-tile bf16 "NT" GEMM for the decoder's per-iteration GEMM pair when the fused decoder does
// not apply (m > 512) and for any other big bf16 contraction:  C[M,N] = sum_k A[M,k] * Bt[N,k].
//
// 256 x 256 x 64 tile per workgroup of 8 wavefronts (two per SIMD, so one wavefront's staging
// requests and LDS waits are covered by the other's MFMAs); each wavefront owns 64 x 128 = 2 x 4
// MFMA tiles (128 accumulator registers) and reads 6 fragments per 8 MFMAs.  Operand tiles are
// staged by direct global->LDS loads, one request = 8 rows x 128 bytes; the 16-byte slot of a row
// is XOR-swizzled with (row/2)&7 so that the fragment reads of 16 consecutive rows fall in 16
// different bank groups.  Two LDS stages of 64 KB.
//
// GemmArgs::a_kwrap carries the number of column tiles here (the grid is 1-D over tiles).
// Contract: K is a multiple of 64 (operands zero-padded to it), row pointers 16-byte aligned.
// Rows >= M / >= N are clamped to the last valid row (their products are discarded or overwritten
// by the epilogue's own bounds handling).
#pragma once
#include "csat_kernels.h"

namespace csat {

constexpr int kBigTile = 256;
constexpr size_t kBigLdsBytes = 8 * 64 * 272;   // two 64 KB stages; the tiled epilogue restages 8 x 64 rows x 272 B

template <typename Epi>
__global__ __launch_bounds__(512) void gemm_nt_bf16_big_kernel(GemmArgs g, Epi epi) {
    extern __shared__ uint4 lds[];
    constexpr int STAGE = 65536, OFF_B = 32768;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // 0..7
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lh = lane >> 5;
    const int z = blockIdx.z;
    // blockIdx.x enumerates tiles column-fastest: the workgroups in flight together then cover all
    // column tiles of a few row tiles, so the wide operand (A rows) is fetched from HBM once and the
    // column operand stays in L2
    const long long row0 = (long long)(blockIdx.x / g.a_kwrap) * kBigTile, col0 = (long long)(blockIdx.x % g.a_kwrap) * kBigTile;
    const bf16_t* A = (const bf16_t*)g.A + (long long)z * g.strideA;
    const bf16_t* Bt = (const bf16_t*)g.Bt + (long long)z * g.strideB;
    const int ksteps = g.K / 64;
    const uint32_t lds0 = (uint32_t)(size_t)(lds_ptr_t)lds;

    // staging: a stage is 32 blocks of 8 rows per operand; this wavefront requests blocks
    // 4*wave .. 4*wave+3 of A and of Bt.  Lane l: row l/8 of the block, LDS slot l%8, which holds
    // the row's 16-byte chunk (l%8) ^ ((row/2)&7).
    const int drow = lane >> 3, dslot = lane & 7;
    const bf16_t* srcA[4];
    const bf16_t* srcB[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int r = (wave * 4 + b) * 8 + drow;                 // row inside the tile
        const int chunk = dslot ^ ((r >> 1) & 7);
        long long ga = row0 + r, gb = col0 + r;
        if (ga >= g.M) ga = g.M - 1;
        if (gb >= g.N) gb = g.N - 1;
        srcA[b] = A + ga * g.lda + chunk * 8;
        srcB[b] = Bt + gb * g.ldb + chunk * 8;
    }
    auto stage = [&](int ks, int st) {
        char* dA = (char*)lds + st * STAGE + wave * 4096;
        char* dB = dA + OFF_B;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            __builtin_amdgcn_global_load_lds((glb_ptr_t)(srcA[b] + (long long)ks * 64), (lds_ptr_t)(dA + b * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((glb_ptr_t)(srcB[b] + (long long)ks * 64), (lds_ptr_t)(dB + b * 1024), 16, 0, 0);
        }
    };

    // fragment addresses: row (tile base + li), 16-byte slot ((2*gk + lh) ^ ((li/2)&7)) for k group gk
    uint32_t adA[4], adB[4];
#pragma unroll
    for (int gk = 0; gk < 4; ++gk) {
        const uint32_t slot = (uint32_t)((2 * gk + lh) ^ ((li >> 1) & 7)) * 16;
        adA[gk] = lds0 + (wm * 64 + li) * 128 + slot;
        adB[gk] = lds0 + OFF_B + (wn * 128 + li) * 128 + slot;
    }

    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    stage(0, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        const uint32_t so = (ks & 1) * STAGE;
        if (ks + 1 < ksteps) stage(ks + 1, (ks + 1) & 1);
        u32x4 fa[2][2], fb[2][4];
        auto fetch = [&](auto gkc) {
            constexpr int gk = decltype(gkc)::value;
            lds_read16<0>(fa[gk & 1][0], adA[gk] + so);
            lds_read16<4096>(fa[gk & 1][1], adA[gk] + so);
            lds_read16<0>(fb[gk & 1][0], adB[gk] + so);
            lds_read16<4096>(fb[gk & 1][1], adB[gk] + so);
            lds_read16<8192>(fb[gk & 1][2], adB[gk] + so);
            lds_read16<12288>(fb[gk & 1][3], adB[gk] + so);
        };
        auto compute = [&](auto gkc) {
            constexpr int gk = decltype(gkc)::value;
            if constexpr (gk + 1 < 4) {
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
        };
        fetch(std::integral_constant<int, 0>{});
        compute(std::integral_constant<int, 0>{});
        compute(std::integral_constant<int, 1>{});
        compute(std::integral_constant<int, 2>{});
        compute(std::integral_constant<int, 3>{});
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }

    // accumulator layout of the 32x32 MFMA: lane (li, lh), register v holds row 8*(v/4) + 4*lh + (v%4), column li
    if constexpr (has_tile_epilogue<Epi>::value) {
        // the stages are free now (last barrier passed): each wavefront gets 64 x Epi::kPitch bytes
        char* stage_w = (char*)lds + wave * 64 * Epi::kPitch;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                epi.tile(z, row0 + wm * 64 + i * 32, col0 + wn * 128 + j * 32, lane, acc[i][j], stage_w, i, j);
        epi.flush(row0 + wm * 64, col0 + wn * 128, lane, stage_w);
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
