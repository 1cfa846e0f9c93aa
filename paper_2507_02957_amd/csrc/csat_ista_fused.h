// Fused ISTA decoder for bf16 operands and m <= 512: one launch runs every iteration.
//
// Rows (queries) are independent problems, so a workgroup can carry its own rows through all T
// iterations with no grid-wide synchronisation.  A workgroup is 4 wavefronts (one per SIMD, the
// whole 512-register budget each); every wavefront owns 32 rows and keeps, in registers,
//   rb    the current residual r = y - Phi x as bf16 MFMA operands        (m x 32)
//   racc  the next residual being accumulated in fp32, initialised to y    (m x 32)
// and walks over the n columns in chunks of 32.  Per chunk:
//   U^T[32 cols, 32 rows]  = Phi_chunk^T (32 x m) * r^T (m x 32)            GEMM-U, K = m
//   x  <- eta_theta(x_old + mu U)           (x_old streamed from the fp32 state buffer)
//   racc[m, 32 rows]      -= Phi_chunk (m x 32) * x^T (32 cols x 32 rows)   GEMM-R, K = 32
// Everything is computed transposed (rows of the problem on the MFMA N axis = lanes), so the
// accumulator layout of one product is directly the B-operand layout of the next and no
// activation ever goes through LDS.  The K-slot order inside a 16-wide MFMA slab is then the
// accumulator's row order (4h+{0..3}, 8+4h+{0..3} for lane half h); Phi is packed once per call
// in exactly that order, as ready-to-use A fragments (1 KB per wavefront load, conflict-free),
// in two copies: Phi^T fragments for GEMM-U and Phi fragments for GEMM-R.  Needs at least two
// chunks (n > 32): the state of the next chunk is requested while the current one is computed.  The 4 wavefronts share
// each packed chunk through a double-buffered LDS stage filled by direct global->LDS loads.
#pragma once
#include "csat_kernels.h"
#include <type_traits>

namespace csat {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* glb_ptr_t;

struct IstaFusedArgs {
    const uint4* PhiPack;   // [NCT][4*MT][64] 16-byte fragments: 2*MT of Phi^T (GEMM-U), then 2*MT of Phi (GEMM-R)
    const float* Y;         // [rows, ldy] fp32 measurements, ldy = 32*MT, columns >= m zero
    float* state;           // [row tiles][NCT][4][64] float4: fp32 iterate in accumulator order
    bf16_t* Xb;             // [rows, ldxb] bf16 copy of the final iterate (operand of the synthesis GEMM), or null
    float* Xout;            // [rows, n] final iterate in caller layout, or null
    long long rows;
    int n, nct, ldy, ldxb, iters;
    float mu, theta;
};

// element (lane half h, slot q) of a 16-wide K slab -> index inside the slab
__host__ __device__ inline int slab_slot(int h, int q) { return 8 * (q >> 2) + 4 * h + (q & 3); }

// Packs Phi [m, n] (bf16, row-major) into the fragment order described above; zero beyond m, n.
__global__ void pack_phi_fragments_kernel(const bf16_t* Phi, int m, int n, int MT, int nct, uint4* out) {
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;     // one 16-byte fragment each
    long long total = (long long)nct * 4 * MT * 64;
    if (idx >= total) return;
    int lane = (int)(idx & 63);
    int f = (int)((idx >> 6) % (4 * MT));
    int ct = (int)(idx / (64LL * 4 * MT));
    int li = lane & 31, lh = lane >> 5;
    bf16_t v[8];
    if (f < 2 * MT) {          // Phi^T fragment: row = column j of Phi, K slots = m indices of slab f
        int j = 32 * ct + li;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            int l = 16 * f + slab_slot(lh, q);
            v[q] = (l < m && j < n) ? Phi[(long long)l * n + j] : (bf16_t)0;
        }
    } else {                   // Phi fragment: row = m index, K slots = columns of slab s2 of this chunk
        int g = f - 2 * MT, mt = g >> 1, s2 = g & 1;
        int l = 32 * mt + li;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            int j = 32 * ct + 16 * s2 + slab_slot(lh, q);
            v[q] = (l < m && j < n) ? Phi[(long long)l * n + j] : (bf16_t)0;
        }
    }
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16);
    o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16);
    o.w = v[6] | ((uint32_t)v[7] << 16);
    out[idx] = o;
}

template <int BASE>
__device__ __forceinline__ bf16x8 cvt8(const f32x16& a, float sign) {
    bf16x8 r;
#pragma unroll
    for (int q = 0; q < 8; ++q) r[q] = (__bf16)(sign * a[BASE + q]);
    return r;
}

template <int MT>
__global__ __launch_bounds__(256, 1) void ista_fused_kernel(IstaFusedArgs a) {
    // LDS: 2 stages, each = 4*MT KB of Phi fragments shared by the workgroup + 4 x 4 KB of old
    // iterate, one 4 KB block per wavefront (its own 32 rows x 32 columns, accumulator order)
    extern __shared__ uint4 lds[];
    constexpr int FRAGS = 4 * MT;                  // 1 KB fragments per chunk: [0, 2MT) GEMM-U, [2MT, 4MT) GEMM-R
    constexpr int PHI16 = FRAGS * 64;              // uint4 of Phi fragments per chunk
    constexpr int STAGE = PHI16 + 4 * 256;         // uint4 per stage
    constexpr int G = 4;                           // fragments per software-pipeline step
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lh = lane >> 5;
    const long long rt = (long long)blockIdx.x * 4 + wave;     // 32-row tile of this wavefront
    const long long row = rt * 32 + (lane & 31);
    const bool row_ok = row < a.rows;
    const int nct = a.nct;
    f32x4* st = (f32x4*)a.state + rt * nct * 256 + lane;       // + (ct*4 + g)*64

    // this wavefront's share of a chunk, global -> LDS: Phi fragments, and its own old iterate
    auto stage_chunk = [&](int ct, int buf, bool with_state) {
        const uint4* src = a.PhiPack + (long long)ct * PHI16 + wave * 64 + lane;
        uint4* dst = lds + buf * STAGE + wave * 64;
#pragma unroll
        for (int i = 0; i < MT; ++i)
            __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + i * 256), (lds_ptr_t)(dst + i * 256), 16, 0, 0);
        if (with_state) {
            uint4* sdst = lds + buf * STAGE + PHI16 + wave * 256;
#pragma unroll
            for (int g = 0; g < 4; ++g)
                __builtin_amdgcn_global_load_lds((glb_ptr_t)(st + (ct * 4 + g) * 64), (lds_ptr_t)(sdst + g * 64), 16, 0, 0);
        }
    };

    f32x16 racc[MT];       // minus Phi x, accumulated over the chunks of one iteration
    bf16x8 rb[2 * MT];     // residual r = y - Phi x of the current iterate, as MFMA B operands
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) racc[mt][v] = 0.f;
    // rows past the end read a valid row; their results are never stored
    const float* yrow = a.Y + (row_ok ? row : a.rows - 1) * a.ldy + 4 * lh;

    // Iteration boundary: r = y + racc becomes the bf16 operand of the next GEMM-U and the
    // accumulators restart from zero.  y tiles are fetched one tile ahead so that the burst of
    // loads never needs more than two tiles of registers.
    auto boundary = [&]() {
        f32x4 yb[2][4];
#pragma unroll
        for (int g = 0; g < 4; ++g) yb[0][g] = *(const f32x4*)(yrow + 8 * g);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt + 1 < MT) {
#pragma unroll
                for (int g = 0; g < 4; ++g) yb[(mt + 1) & 1][g] = *(const f32x4*)(yrow + 32 * (mt + 1) + 8 * g);
            }
            f32x16 r;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                r[v] = yb[mt & 1][v >> 2][v & 3] + racc[mt][v];
                racc[mt][v] = 0.f;
            }
            rb[2 * mt] = cvt8<0>(r, 1.f);
            rb[2 * mt + 1] = cvt8<8>(r, 1.f);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One chunk of 32 columns.  Fragments are fetched from LDS G at a time, one step ahead of the
    // MFMAs that consume them; scheduling barriers keep the compiler from hoisting every fetch
    // to the top (which would not fit the register file).
    auto chunk = [&](auto last_tag, int ct, int buf, bool first) {
        constexpr bool kLast = decltype(last_tag)::value;
        constexpr int NF = kLast ? 2 * MT : 4 * MT;
        constexpr int NG = (NF + G - 1) / G;
        const uint4* pl = lds + buf * STAGE + lane;
        const uint4* xs = lds + buf * STAGE + PHI16 + wave * 256 + lane;
        uint4 fr[2][G];
        f32x16 u0, u1, x;
        bf16x8 xb0, xb1;
#pragma unroll
        for (int v = 0; v < 16; ++v) { u0[v] = 0.f; u1[v] = 0.f; }
        auto threshold = [&]() {
            f32x4 xo[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) xo[g] = __builtin_bit_cast(f32x4, xs[g * 64]);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float u = (first ? 0.f : xo[v >> 2][v & 3]) + a.mu * (u0[v] + u1[v]);
                float mag = fabsf(u) - a.theta;
                x[v] = (mag > 0.f) ? copysignf(mag, u) : 0.f;
            }
        };
#pragma unroll
        for (int i = 0; i < G; ++i)
            if (i < NF) fr[0][i] = pl[i * 64];
#pragma unroll
        for (int k = 0; k < NG; ++k) {
#pragma unroll
            for (int i = 0; i < G; ++i)
                if ((k + 1) * G + i < NF) fr[(k + 1) & 1][i] = pl[((k + 1) * G + i) * 64];
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const int f = k * G + i;
                if (f == 2 * MT) {   // all of U is in: threshold, write the state back
                    threshold();
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        f32x4 o = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
                        st[(ct * 4 + g) * 64] = o;
                    }
                    xb0 = cvt8<0>(x, -1.f);
                    xb1 = cvt8<8>(x, -1.f);
                }
                if (f < 2 * MT) {
                    if (f & 1) u1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fr[k & 1][i]), rb[f], u1, 0, 0, 0);
                    else u0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fr[k & 1][i]), rb[f], u0, 0, 0, 0);
                } else if (f < NF) {
                    const int r = f - 2 * MT;
                    racc[r >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fr[k & 1][i]),
                                                                           (r & 1) ? xb1 : xb0, racc[r >> 1], 0, 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (kLast) {
            threshold();
            if (row_ok) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = 32 * ct + 8 * g + 4 * lh;
                    if (a.Xb && col < a.ldxb) {
                        uint2 o;
                        o.x = f2bf(x[4 * g]) | ((uint32_t)f2bf(x[4 * g + 1]) << 16);
                        o.y = f2bf(x[4 * g + 2]) | ((uint32_t)f2bf(x[4 * g + 3]) << 16);
                        *(uint2*)(a.Xb + row * a.ldxb + col) = o;
                    }
                    if (a.Xout) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < a.n) a.Xout[row * (long long)a.n + col + e] = x[4 * g + e];
                    }
                }
            }
        }
    };

    // The chunk being worked on was requested one chunk earlier: wait for it (all wavefronts),
    // then request the next one into the other stage before starting on the arithmetic.
    stage_chunk(0, 0, false);
    int buf = 0;
    for (int t = 0; t + 1 < a.iters; ++t) {
        const bool first = t == 0;
        boundary();
        for (int ct = 0; ct < nct; ++ct) {
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            const bool wrap = ct + 1 == nct;
            stage_chunk(wrap ? 0 : ct + 1, buf ^ 1, wrap || !first);
            chunk(std::false_type{}, ct, buf, first);
            buf ^= 1;
        }
    }
    {   // last iteration: no residual update, outputs instead of state
        const bool first = a.iters == 1;
        boundary();
        for (int ct = 0; ct < nct; ++ct) {
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (ct + 1 < nct) stage_chunk(ct + 1, buf ^ 1, !first);
            chunk(std::true_type{}, ct, buf, first);
            buf ^= 1;
        }
    }
}

}  // namespace csat
