// Measurement K~ = Phi K, V~ = Phi V (section 3) for bf16 with d = 64 or 128, both products in one launch and
// straight from K and V as the caller holds them ([n, d] per head, d contiguous): no transposed copies.
//
// The contraction runs over n, which is the ROW index of K and V, so a B fragment of the MFMA (8 consecutive k for
// one column) is a column piece of the tile.  K and V tiles of KS rows go through LDS as they are, row-major, and
// the fragments come out with the transposing 8-byte LDS load: in each group of 16 lanes, lane 4e + q supplies the
// address of 4 consecutive elements of row e, and lane c receives column c of that 4 x 16 block.  The workgroup's
// rows of Phi go through LDS as well, KS columns per step (whole 128-byte lines of a row per load; a lane fetching
// its own fragment from global memory touches 32 lines per instruction and measured half as fast); an A fragment
// (8 consecutive k of one row) is 16 contiguous bytes there and feeds the d / 32 column tiles of a product.
//
// A workgroup takes two tiles of m of one head, two wavefronts per tile: one multiplies into K~, the other into V~
// (four tiles, one wavefront each, when V~ is not wanted).  The staged tiles are shared by its wavefronts.  The
// tiles of the next PD steps are in flight in registers while a step is multiplied; LDS holds two steps.
// Workgroups are numbered so that those of one head run on the same XCD (consecutive workgroup ids go round the
// eight XCDs) and find the head's K and V in that XCD's L2 after the first of them has read them.
//
// The epilogue writes everything the next stage reads: K~ in the element type, its (hi | lo) bf16 pair, the same
// pair as MFMA fragments for the compressed-attention kernel, V~, and V~ either as that kernel's fragments for the
// output product or as the zero-padded transpose a GEMM takes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "csat_kernels.h"

namespace csat {

struct MeasureDirectArgs {
    const bf16_t* Phi; long long ldp;  // [m][ldp], 16-byte aligned rows; columns [ncols, ..) are not read (taken as zero)
    int ncols;                         // a multiple of 8, >= n only if the columns from n on hold zeros
    const bf16_t* K; const bf16_t* V;  // [heads][n][d]
    long long strideX;                 // elements between heads
    int m, n, MT;                      // MT = ceil(m / 32)
    int heads, blocks_per_head;        // grid: 8 * ceil(heads / 8) * blocks_per_head workgroups
    bf16_t* Kc;                        // [heads][m][d]
    bf16_t* KcHL;                      // optional [heads][m][2 d]: hi = bf16(v) | lo = bf16(v - hi)
    uint4* KcPack;                     // optional [heads][MT][2 d / 16][64]: the pair as fragments, zero beyond m
    bf16_t* Vc;                        // [heads][m][d]; V~ is computed only when Vc != nullptr
    bf16_t* VcT; long long ldm;        // optional [heads][d][ldm], columns [m, ldm) written as zero
    uint4* VPack;                      // optional [heads][MT][d / 32][2][64]: V~ as the A fragments of the attention
                                       // kernel's output product (rows 16 s + 4 h .. + 3 and + 8 of a tile per lane half h)
    long long strideA;                 // elements between the heads' own row operands (0: Phi, shared by the heads).  With
                                       // it the kernel is the synthesis C = X V of a head: Phi = the bf16 iterate, m = n_q,
                                       // K = V as the caller holds it, Kc = C
};

// DT = d / 32; KS: rows of K and V per step; PD: steps in flight; WANT_V: V~ too (a.Vc != nullptr)
template <int DT, int KS, int PD, bool WANT_V>
__global__ __launch_bounds__(256) void measure_direct_kernel(MeasureDirectArgs a) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
    constexpr int D = 32 * DT;
    // 64 bytes of padding per staged row: the 4 rows x 32 bytes that the two 16-lane groups of a half wavefront read
    // together then fall into 64 different banks
    constexpr int PITCH = D * 2 + 64;
    constexpr int PR = D / 8;                    // 16-byte pieces per row
    constexpr int PPT = KS * PR / 256;           // pieces per thread and tile
    constexpr int TILE = KS * PITCH;
    // the workgroup's rows of Phi, KS columns per step, row pitch padded by 16 bytes (16 lanes reading 16 bytes of
    // 16 consecutive rows then cover all banks once)
    constexpr int MROWS = WANT_V ? 64 : 128;
    constexpr int PA = KS * 2 + 16, PRA = KS / 8, PPA = MROWS * PRA / 256;
    constexpr int STAGE = 2 * TILE + MROWS * PA;
    static_assert(DT == 2 || DT == 4, "d = 64 or 128");
    __shared__ __attribute__((aligned(16))) char lds[2 * STAGE];      // [stage][K | V | Phi]
    // workgroup id -> (head, block of tiles): XCD x = id % 8 takes heads x, x + 8, ...
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int z = (slot / a.blocks_per_head) * 8 + xcd, mb = slot % a.blocks_per_head;
    if (z >= a.heads) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kh = lane >> 5, li = lane & 31;
    constexpr bool want_v = WANT_V;
    const int mt = want_v ? mb * 2 + (wave >> 1) : mb * 4 + wave;
    const bool for_v = want_v && (wave & 1);              // this wavefront's product
    const bool live = mt < a.MT;
    const int wtile = WANT_V ? wave >> 1 : wave;          // this wavefront's tile within the workgroup's rows of Phi
    const bf16_t* Kz = a.K + (long long)z * a.strideX;
    const bf16_t* Vz = a.V + (long long)z * a.strideX;
    const bf16_t* Az = a.Phi + (long long)z * a.strideA;
    f32x16 acc[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
    // The loop body has no branch: loads behind a branch make the compiler wait for every load in flight at each
    // use.  So every step loads (addresses beyond the data fall back to row 0 / column 0, the staged rows from n on
    // are replaced by zeros, and what Phi contributes there is multiplied by those zeros), wavefronts without a
    // tile multiply like the others and skip the epilogue, and the step count is rounded up to a multiple of PD.
    const int steps = ((a.n + KS - 1) / KS + PD - 1) / PD * PD;
    // (a native vector type: arrays of the HIP uint4 struct end up in scratch memory here)
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    u32x4 gK[PD][PPT], gV[PD][PPT];
    u32x4 gA[PD][PPA];
    auto gload = [&](int s, u32x4 (&k)[PPT], u32x4 (&v)[PPT]) {
#pragma unroll
        for (int q = 0; q < PPT; ++q) {
            const int p = threadIdx.x + 256 * q, r = p / PR, c = p % PR;
            long long row = (long long)s * KS + r;
            row = row < a.n ? row : 0;
            k[q] = *(const u32x4*)(Kz + row * D + c * 8);
            if constexpr (WANT_V) v[q] = *(const u32x4*)(Vz + row * D + c * 8);
        }
    };
    auto lstore = [&](char* stage, int s, const u32x4 (&k)[PPT], const u32x4 (&v)[PPT]) {
#pragma unroll
        for (int q = 0; q < PPT; ++q) {
            const int p = threadIdx.x + 256 * q, r = p / PR, c = p % PR;
            const unsigned keep = (long long)s * KS + r < a.n ? ~0u : 0u;
            *(u32x4*)(stage + r * PITCH + c * 16) = k[q] & keep;
            if constexpr (WANT_V) *(u32x4*)(stage + TILE + r * PITCH + c * 16) = v[q] & keep;
        }
    };
    auto aload = [&](int s, u32x4 (&f)[PPA]) {
#pragma unroll
        for (int q = 0; q < PPA; ++q) {
            const int p = threadIdx.x + 256 * q, r = p / PRA, c = p % PRA;
            long long row = (long long)mb * MROWS + r;
            row = row < a.m ? row : a.m - 1;
            const int col = s * KS + c * 8;
            f[q] = *(const u32x4*)(Az + row * a.ldp + (col + 8 <= a.ncols ? col : 0));
        }
    };
    auto astore = [&](char* stage, const u32x4 (&f)[PPA]) {
#pragma unroll
        for (int q = 0; q < PPA; ++q) {
            const int p = threadIdx.x + 256 * q, r = p / PRA, c = p % PRA;
            *(u32x4*)(stage + 2 * TILE + r * PA + c * 16) = f[q];
        }
    };
    // this lane's corner of the 4 x 16 blocks it helps to read: row 8 kh + e, column 16 jg + 4 q
    const int tr_off = (8 * kh + ((lane & 15) >> 2)) * PITCH + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
    const int fa_off = 2 * TILE + (wtile * 32 + li) * PA + 16 * kh;
    auto product = [&](const char* stage) {
        const char* tile = stage + (for_v ? TILE : 0);
        bf16x8 f[KS / 16];
        s16x4 lo[KS / 16][DT], hi[KS / 16][DT];
#pragma unroll
        for (int u = 0; u < KS / 16; ++u) {
            f[u] = *(const bf16x8*)(stage + fa_off + 32 * u);
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                const char* p = tile + tr_off + 16 * u * PITCH + 64 * t;
                lo[u][t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
                hi[u][t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * PITCH));
            }
        }
#pragma unroll
        for (int u = 0; u < KS / 16; ++u)
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                const s16x8 b = __builtin_shufflevector(lo[u][t], hi[u][t], 0, 1, 2, 3, 4, 5, 6, 7);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[u], __builtin_bit_cast(bf16x8, b), acc[t], 0, 0, 0);
            }
    };
    // register set j holds step s with s % PD == j; a set is free once its tiles are in LDS
#pragma unroll
    for (int j = 0; j < PD; ++j) {
        gload(j, gK[j], gV[j]);
        aload(j, gA[j]);
    }
    lstore(lds, 0, gK[0], gV[0]);
    astore(lds, gA[0]);
    __syncthreads();
    for (int s0 = 0; s0 < steps; s0 += PD) {
#pragma unroll
        for (int j = 0; j < PD; ++j) {
            const int s = s0 + j;
            char* stage = lds + (s & 1) * STAGE;
            char* other = lds + ((s & 1) ^ 1) * STAGE;
            gload(s + PD, gK[j], gV[j]);                 // (beyond the last step: rows >= n, i.e. row 0 again)
            aload(s + PD, gA[j]);
            product(stage);
            lstore(other, s + 1, gK[(j + 1) % PD], gV[(j + 1) % PD]);
            astore(other, gA[(j + 1) % PD]);
            __syncthreads();
        }
    }
    if (!live) return;
    // Epilogue.  The accumulators hold columns (lane = column, 16 rows each); rows of the outputs are contiguous in
    // memory, so a tile goes through this wavefront's piece of the staging LDS (free after the last step's barrier)
    // and leaves as 16-byte pieces of rows.  The transpose of V~ wants four consecutive rows of a column: that is
    // what a lane holds, and it is stored from the registers.
    constexpr int PE = D * 2 + 16;                     // row pitch of the tile in LDS
    char* ep = lds + wave * (32 * PE);
    const long long zm = (long long)z * a.m;
    const int ng = D / 16;
    // which: 0 the value in the element type, 1 what is left of it (the lo half of the pair); rows beyond m as zero
    auto tile_to_lds = [&](int which) {
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rl = 8 * (v >> 2) + 4 * kh + (v & 3);
                const float x = acc[t][v];
                const bf16_t hi = f2bf(x);
                const bf16_t out = which == 0 ? hi : f2bf(x - bf2f(hi));
                *(bf16_t*)(ep + rl * PE + (32 * t + li) * 2) = (long long)mt * 32 + rl < a.m ? out : (bf16_t)0;
            }
    };
    auto rows_out = [&](auto&& store) {            // store(row in tile, piece of the row, 16 bytes)
#pragma unroll
        for (int i = 0; i < 32 * PR / 64; ++i) {
            const int idx = lane + 64 * i, rl = idx / PR, pc = idx % PR;
            store(rl, pc, *(const uint4*)(ep + rl * PE + pc * 16));
        }
    };
    if (!for_v) {
        uint4* pack = a.KcPack ? a.KcPack + ((long long)z * a.MT + mt) * 2 * ng * 64 : nullptr;
        tile_to_lds(0);
        rows_out([&](int rl, int pc, uint4 w) {
            const long long r = (long long)mt * 32 + rl;
            if (r < a.m) {
                *(uint4*)(a.Kc + (zm + r) * D + pc * 8) = w;
                if (a.KcHL) *(uint4*)(a.KcHL + (zm + r) * 2 * D + pc * 8) = w;
            }
            // fragment s = part * ng + pc / 2: lane (rl, pc & 1) holds this piece
            if (pack) pack[(pc >> 1) * 64 + (pc & 1) * 32 + rl] = w;
        });
        if (a.KcHL || pack) {
            tile_to_lds(1);
            rows_out([&](int rl, int pc, uint4 w) {
                const long long r = (long long)mt * 32 + rl;
                if (r < a.m && a.KcHL) *(uint4*)(a.KcHL + (zm + r) * 2 * D + D + pc * 8) = w;
                if (pack) pack[(ng + (pc >> 1)) * 64 + (pc & 1) * 32 + rl] = w;
            });
        }
    } else {
        tile_to_lds(0);
        rows_out([&](int rl, int pc, uint4 w) {
            const long long r = (long long)mt * 32 + rl;
            if (r < a.m) *(uint4*)(a.Vc + (zm + r) * D + pc * 8) = w;
        });
        if (a.VPack) {
            // the accumulator layout is the fragment layout: lane (column, h) holds rows 8 g + 4 h .. + 3 of the tile,
            // a fragment of slab s wants g = 2 s and 2 s + 1
            uint4* vp = a.VPack + ((long long)z * a.MT + mt) * DT * 2 * 64 + lane;
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int sl = 0; sl < 2; ++sl) {
                    float x[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const long long r = (long long)mt * 32 + 8 * (2 * sl + (e >> 2)) + 4 * kh + (e & 3);
                        x[e] = r < a.m ? acc[t][8 * sl + e] : 0.f;
                    }
                    vp[(t * 2 + sl) * 64] = uint4{f2bf_pk(x[0], x[1]), f2bf_pk(x[2], x[3]), f2bf_pk(x[4], x[5]), f2bf_pk(x[6], x[7])};
                }
        }
        if (a.VcT) {
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const long long r0 = (long long)mt * 32 + 8 * g + 4 * kh;        // (< ldm: ldm covers whole tiles)
                    float x[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = r0 + e < a.m ? acc[t][4 * g + e] : 0.f;
                    *(uint2*)(a.VcT + ((long long)z * D + 32 * t + li) * a.ldm + r0) = uint2{f2bf_pk(x[0], x[1]), f2bf_pk(x[2], x[3])};
                }
        }
    }
    // pad columns of the transposed V~ beyond the last tile (ldm is a multiple of 64, the tiles cover a multiple of 32)
    if (for_v && a.VcT && mt == a.MT - 1 && a.ldm > (long long)a.MT * 32) {
        for (int c = lane; c < D; c += 64) {
            uint4* p = (uint4*)(a.VcT + ((long long)z * D + c) * a.ldm + (long long)a.MT * 32);
            const int pieces = (int)((a.ldm - (long long)a.MT * 32) / 8);
            for (int i = 0; i < pieces; ++i) p[i] = uint4{0u, 0u, 0u, 0u};
        }
    }
}

}  // namespace csat
