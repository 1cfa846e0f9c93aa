// Compressed attention in one kernel: scores, row softmax and the output product
//     A~ = softmax(Q K~^T / sqrt(d_k)),   Z = A~ V~                      (section 3, eq. for A~ and Z)
// with the softmax taken inside the score tile.
//
// One wavefront owns 32 query rows of one head and everything is computed transposed, as in the fused
// decoder: S^T [m x 32 rows] = K~ [m x d] Q^T [d x 32 rows], so a query row lives in ONE lane pair
// (lanes i and i + 32 hold the even and odd groups of four of its scores, 16 per 32-wide tile of m).  The
// row maximum and the row sum are then reductions over a lane's own registers plus a single exchange with
// the partner lane: no LDS round trip, no second kernel, and the scores never leave the registers before
// they are probabilities.  Up to 16 tiles of m (m <= 512) are held at once; longer rows take two sweeps
// over m in panels of 8 tiles (running maximum and sum first, then the scores again, normalised), which
// costs the cheap product twice (its depth is only d_k) and still writes A~ exactly once.
//
// K~ is the stationary operand.  It is packed once per call as ready MFMA A fragments (1 KB each:
// 32 rows of K~ x one contraction group, lane (l, h) holding its 16 bytes at slot l + 32 h) and a
// workgroup (4 or 8 wavefronts, all on the same head) keeps the head's fragments in LDS: staged once by direct
// global->LDS loads when they fit (then the workgroup works through several rounds of one row tile per
// wavefront), panel by panel otherwise.  Every LDS read is a conflict-free 16 bytes per lane; Q is read once into registers.
//
// The accumulator layout of S^T is the B-operand layout of the output product Z^T [d x rows] =
// V~^T [d x m] P^T [m x rows] up to the order of the contraction index inside a 16-wide slab (lane half
// h holds m = 4h..4h+3 and 8+4h..8+4h+3 of the slab); the A operand, read from the transposed V~, is
// fetched in that same order, so the probabilities go from the softmax into the product as they are.
#pragma once
#include "csat_kernels.h"

namespace csat {

struct AttentionArgs {
    const void* Q;   long long strideQ;            // [BH][n_q][d]
    const uint4* Kf;                               // [BH][mt_total][ns][64] packed fragments of K~ (pack_kc_fragments_kernel)
    int ns, ng;                                    // fragments per tile = kparts * ng; ng = contraction groups of d
    const void* VcT; long long ldv, strideV;       // [BH][d][ldv]: V~^T, columns [m, ldv) zero (only read when Z or ZT is wanted)
    const uint4* Vf;                               // bf16, d = 64 or 128, instead of VcT (kernels with ZM = 2 / 3):
                                                   // [BH][mt_total][d / 32][2][64], V~ as the output product's A fragments
                                                   // (written by the one-kernel measurement)
    int a_tiled;                                   // single-sweep kernels that keep the scores in the accumulator file, n_q a multiple of
                                                   // 32: A is written in accumulator tiles, [tile of 32 rows over all heads][mt][4][64] float4
    int v_lds;                                     // with Vf: first LDS slot (1 KB each) of the head's V~ fragments, staged behind K~'s
    float* A;  long long ldA;                      // [BH*n_q][ldA] probabilities, columns [m, ldA) written as zero; may be null
    void* P;   long long ldP;                      // optional copy of A~ in the element type, zero padded to ldP
    void* Z;                                       // optional [BH][n_q][d] in the element type
    void* ZT;  long long ldT, strideT;             // optional Z^T per head (bf16: hi at [dd][row], lo at [dd][ldT/2 + row]); pre-zeroed
    int n_q, m, d;
    float scale_log2e;                             // log2(e) / sqrt(d_k): exp(s / sqrt(d_k)) = 2^(s * scale_log2e)
    int tiles_per_head;                            // ceil(n_q / 32)
    int rounds;                                    // rounds of one row tile per wavefront (1 unless all of K~ sits in LDS)
    int wg_per_head;                               // ceil(tiles_per_head / (wavefronts per workgroup * rounds))
};

// K~ [BH][m][ld] (row-major, ld = kparts * d: the plain matrix or a bf16 (hi | lo) pair) -> fragments.
// Fragment (tile mt, s = part * ng + g): lane (l, h) gets the 16 bytes of row 32 mt + l, elements
// part * d + (2 g + h) * EPC .. + EPC - 1; zero beyond m and d.  One thread per 16-byte piece.
template <typename T>
__global__ void pack_kc_fragments_kernel(const T* src, long long ld, int m, int d, int kparts, int mt_total, int ng,
                                         uint4* out, long long total) {
    constexpr int EPC = Elem<T>::per_chunk;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int lane = (int)(idx & 63), l = lane & 31, h = lane >> 5;
    const int ns = kparts * ng;
    const int s = (int)((idx >> 6) % ns);
    const int mt = (int)((idx / (64LL * ns)) % mt_total);
    const long long z = idx / (64LL * ns * mt_total);
    const int part = s / ng, g = s % ng;
    const int r = 32 * mt + l, c = (2 * g + h) * EPC;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < m && c < d) v = *(const uint4*)(src + (z * m + r) * ld + part * d + c);
    out[idx] = v;
}

template <typename T> struct AttnVec;
template <> struct AttnVec<bf16_t> {              // four values of the element type
    typedef uint2 type;
    __device__ static __forceinline__ uint2 pack(float a, float b, float c, float d) { return uint2{f2bf_pk(a, b), f2bf_pk(c, d)}; }
};
template <> struct AttnVec<float> {
    typedef f32x4 type;
    __device__ static __forceinline__ f32x4 pack(float a, float b, float c, float d) { return f32x4{a, b, c, d}; }
};

constexpr int kAttnMaxLdsBytes = 144 * 1024;      // fragments of K~ a workgroup keeps in LDS
constexpr int kAttnLdsBytes = 160 * 1024;         // LDS of a CU: K~ and V~ fragments together
constexpr int kAttnPanelTiles = 8;                // tiles of m per panel when K~ is staged panel by panel

// Tiles of m the kernel instance for mt_total tiles holds in registers (`single`: all of them, one sweep).
constexpr int attention_mtp(int mt_total, bool single) {
    return !single ? kAttnPanelTiles : mt_total <= 1 ? 1 : mt_total <= 2 ? 2 : mt_total <= 4 ? 4 : mt_total <= 8 ? 8 : mt_total <= 13 ? 13 : 16;
}
// Wavefronts per workgroup: eight (two per SIMD, 256 registers each, so that one wavefront's softmax arithmetic
// and stores run under the other's products) where the score accumulators leave room for that, else four
// (measured at 13 tiles: eight wavefronts spill and take twice as long).
// With the output product from packed fragments (ZM >= 2) eight tiles already need the 512 registers of a lone wavefront.
constexpr int attention_waves(int MTP, int ZM = 0) { return MTP <= 4 || (MTP <= 8 && ZM < 2) ? 8 : 4; }

// MTP: tiles of m held in registers at once.  SINGLE: all of m fits registers and LDS (one sweep, staged
// once).  ZM: 0 no output product; 1 also the output product (Z and / or its transpose) from the transposed V~; 2 / 3 the
// same from V~ as packed fragments (a.Vf; bf16, d = 64 / 128: four / eight fragments per tile of m; single sweep only, and
// only onto rows of A~ that hold whole tiles: a.A 16-byte aligned with a.ldA a multiple of 4 and >= 32 tiles, as in the
// library's own carving).
template <typename T, int MTP, bool SINGLE, int ZM>
__global__ __launch_bounds__(64 * attention_waves(MTP, ZM), 1) void attention_fused_kernel(AttentionArgs a) {
    constexpr int NW = attention_waves(MTP, ZM);
    constexpr bool kBf16 = sizeof(T) == 2;
    constexpr bool WANT_Z = ZM != 0, VPACK = ZM >= 2;
    static_assert(!VPACK || kBf16, "packed fragments of V~ exist in bf16 only");
    constexpr int EPC = Elem<T>::per_chunk;        // elements per 16-byte chunk
    constexpr int GK = 2 * EPC;                    // contraction depth of one mfma_group (both lane halves)
    constexpr int NGMAX = ZM == 2 ? 64 / GK : 128 / GK;      // d <= 128 (ZM = 2: d = 64)
    constexpr int NZ = ZM == 2 ? 2 : 4;            // tiles of d in the output product
    typedef typename AttnVec<T>::type vec4_t;
    extern __shared__ uint4 lds[];
    const int lane = threadIdx.x & 63, li = lane & 31, lh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int z = blockIdx.x / a.wg_per_head, chunk = blockIdx.x % a.wg_per_head;
    const int d = a.d, m = a.m, ng = a.ng, ns = a.ns;
    const int mt_total = (m + 31) / 32;
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    const uint4* kf = a.Kf + (long long)z * mt_total * ns * 64;

    // fragments [f0, f0 + nf) of this head into LDS slots 0 .. nf - 1, 1 KB per request, shared out over the wavefronts
    // The slots of tiles that do not exist (up to MTP tiles) are zeroed, so that the products below run over all MTP
    // tiles without a test per tile: a test is a branch per MFMA, and an MFMA in a basic block of its own waits out
    // the full latency of its fragment read.  Those tiles' scores are masked like every score beyond m.
    auto stage = [&](int f0, int nf) {
        for (int f = wave; f < nf; f += NW)
            __builtin_amdgcn_global_load_lds((glb_ptr_t)(kf + (long long)(f0 + f) * 64 + lane), (lds_ptr_t)((char*)lds + f * 1024), 16, 0, 0);
        for (int f = nf + wave; f < MTP * ns; f += NW) lds[f * 64 + lane] = zero4;
    };
    if constexpr (SINGLE) {
        stage(0, mt_total * ns);
        if constexpr (VPACK) {
            constexpr int NFS = ZM == 2 ? 4 : 8;
            const uint4* vf = a.Vf + (long long)z * mt_total * NFS * 64;
            for (int f = wave; f < mt_total * NFS; f += NW)
                __builtin_amdgcn_global_load_lds((glb_ptr_t)(vf + (long long)f * 64 + lane), (lds_ptr_t)((char*)lds + (a.v_lds + f) * 1024), 16, 0, 0);
            for (int f = mt_total * NFS + wave; f < MTP * NFS; f += NW) lds[(a.v_lds + f) * 64 + lane] = zero4;
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }

    for (int r = 0; r < a.rounds; ++r) {
        const int rt = (chunk * a.rounds + r) * NW + wave;
        const bool active = rt < a.tiles_per_head;          // wavefront-uniform
        if (SINGLE && !active) continue;                    // no barriers after the staging
        const int row = rt * 32 + li;
        const bool row_ok = active && row < a.n_q;
        const long long grow = (long long)z * a.n_q + (row_ok ? row : a.n_q - 1);      // rows past the end repeat the last one

        // Q^T as B operands: lane (i, h) holds elements (2 g + h) * EPC .. + EPC - 1 of its row for group g
        uint4 qf[NGMAX];
        {
            const T* q = (const T*)a.Q + grow * d;
#pragma unroll
            for (int g = 0; g < NGMAX; ++g) {
                const int c = (2 * g + lh) * EPC;
                qf[g] = (g < ng && c < d) ? *(const uint4*)(q + c) : zero4;
            }
        }

        // raw scores (Q . K~, unscaled) of the panel whose fragments sit in LDS (tiles mt0 .. mt0+MTP-1); -inf beyond m
        auto scores = [&](int mt0, f32x16 (&acc)[MTP]) {
#pragma unroll
            for (int t = 0; t < MTP; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
            const int parts = ns / ng;
            for (int part = 0; part < parts; ++part) {
#pragma unroll
                for (int g = 0; g < NGMAX; ++g) {
                    if (g >= ng) continue;
                    const uint4* fr = lds + (part * ng + g) * 64 + lane;
#pragma unroll
                    for (int t = 0; t < MTP; ++t) mfma_group<T>(fr[t * ns * 64], qf[g], acc[t]);
                }
            }
#pragma unroll
            for (int t = 0; t < MTP; ++t) {
                if (32 * (mt0 + t + 1) <= m) continue;          // only a tile that overhangs m needs the mask (uniform)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int idx = 32 * (mt0 + t) + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (idx >= m) acc[t][v] = -INFINITY;
                }
            }
        };
        auto panel_max = [&](const f32x16 (&acc)[MTP]) {
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < MTP; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc[t][v]);
            return fmaxf(mx, __shfl_xor(mx, 32, 64));        // the partner lane holds the row's other scores
        };

        const int ndt = (d + 31) / 32;
        f32x16 zacc[WANT_Z ? NZ : 1];
        if constexpr (WANT_Z) {
#pragma unroll
            for (int dt = 0; dt < NZ; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) zacc[dt][v] = 0.f;
        }
        float* arow = a.A ? a.A + ((long long)z * a.n_q + row) * a.ldA : nullptr;
        T* prow = a.P ? (T*)a.P + ((long long)z * a.n_q + row) * a.ldP : nullptr;
        const bool a_vec = (a.ldA & 3) == 0 && ((uintptr_t)a.A & 15) == 0;
        // rows of A~ and of its copy that hold whole tiles (the library's own carving): every store is a 16- or 8-byte
        // one at a constant offset from the row's base, no per-store bounds checks
        const bool whole_tiles = (!a.A || (a_vec && a.ldA >= 32 * mt_total)) && (!a.P || a.ldP >= 32 * mt_total);

        // probabilities of a panel: stores and the output product
        auto emit = [&](int mt0, const f32x16 (&acc)[MTP]) {
            if (row_ok && whole_tiles) {
                if (arow) {
                    float* ab = arow + 32 * mt0 + 4 * lh;
#pragma unroll
                    for (int t = 0; t < MTP; ++t)
                        if (mt0 + t < mt_total) {
#pragma unroll
                            for (int g = 0; g < 4; ++g)
                                *(f32x4*)(ab + 32 * t + 8 * g) = f32x4{acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]};
                        }
                }
                if (prow) {
                    T* pb = prow + 32 * mt0 + 4 * lh;
#pragma unroll
                    for (int t = 0; t < MTP; ++t)
                        if (mt0 + t < mt_total) {
#pragma unroll
                            for (int g = 0; g < 4; ++g)
                                *(vec4_t*)(pb + 32 * t + 8 * g) = AttnVec<T>::pack(acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]);
                        }
                }
            }
#pragma unroll
            for (int t = 0; t < MTP; ++t) {
                const int mt = mt0 + t;
                if (mt >= mt_total) continue;
                if (row_ok && !whole_tiles) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int col = 32 * mt + 8 * g + 4 * lh;
                        if (arow) {
                            if (a_vec && col + 4 <= a.ldA) {
                                *(f32x4*)(arow + col) = f32x4{acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]};
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (col + e < a.ldA) arow[col + e] = acc[t][4 * g + e];
                            }
                        }
                        if (prow && col < a.ldP)      // ldP is a multiple of 8: a group of four is inside or outside
                            *(vec4_t*)(prow + col) = AttnVec<T>::pack(acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]);
                    }
                }
                if constexpr (WANT_Z && !VPACK) {
                    const T* vt = (const T*)a.VcT + (long long)z * a.strideV;
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) {
                        if (dt >= ndt) continue;
                        const int dd = 32 * dt + li;
                        const T* vrow = vt + (long long)(dd < d ? dd : d - 1) * a.ldv + 32 * mt;
                        if constexpr (kBf16) {
#pragma unroll
                            for (int s = 0; s < 2; ++s) {      // 16-wide slabs of the tile; slot order 4h..4h+3, 8+4h..8+4h+3
                                const int c0 = 16 * s + 4 * lh, c1 = c0 + 8;
                                uint2 v0 = uint2{0u, 0u}, v1 = uint2{0u, 0u};
                                if (dd < d && 32 * mt + c0 + 4 <= a.ldv) v0 = *(const uint2*)(vrow + c0);
                                if (dd < d && 32 * mt + c1 + 4 <= a.ldv) v1 = *(const uint2*)(vrow + c1);
                                const uint4 vf = make_uint4(v0.x, v0.y, v1.x, v1.y);
                                const uint4 pf = make_uint4(f2bf_pk(acc[t][8 * s], acc[t][8 * s + 1]), f2bf_pk(acc[t][8 * s + 2], acc[t][8 * s + 3]),
                                                            f2bf_pk(acc[t][8 * s + 4], acc[t][8 * s + 5]), f2bf_pk(acc[t][8 * s + 6], acc[t][8 * s + 7]));
                                mfma_group<T>(vf, pf, zacc[dt]);
                            }
                        } else {
#pragma unroll
                            for (int g = 0; g < 4; ++g) {      // 8-wide slabs: lane half h holds m = 8g + 4h .. + 3
                                const int c0 = 8 * g + 4 * lh;
                                uint4 vf = zero4;
                                if (dd < d && 32 * mt + c0 + 4 <= a.ldv) vf = *(const uint4*)(vrow + c0);
                                const f32x4 pv = f32x4{acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]};
                                mfma_group<T>(vf, __builtin_bit_cast(uint4, pv), zacc[dt]);
                            }
                        }
                    }
                }
            }
        };

        if constexpr (SINGLE) {
        bool emitted = false;
        // (without the product: for 9 to 13 tiles, where the other form spills; at 8 and 16 tiles carrying both forms costs more)
        if constexpr (VPACK || (ZM == 0 && MTP == 13)) if (VPACK || whole_tiles) {
            emitted = true;
            // The scores stay in the accumulator registers through the softmax: vector instructions cannot read
            // those, so left to itself the compiler moves all tiles into ordinary registers behind the products
            // (13 tiles: 208 of the 256) and spills.  Here every pass takes one tile at a time through ordinary
            // registers and puts it back (the empty statements pin a tile to the accumulator file), and the last pass
            // - scale, the tile's part of the output product, the tile's stores - consumes it.
            f32x16 acc[MTP];
            scores(0, acc);
#define CSAT_PIN_ACC(x) asm volatile("" : "+a"(x))
            const float sl = a.scale_log2e;
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < MTP; ++t) {
                CSAT_PIN_ACC(acc[t]);
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc[t][v]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float off = -mx * sl;
            float sum = 0.f;
#pragma unroll
            for (int t = 0; t < MTP; ++t) {
                f32x16 e = acc[t];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    e[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(e[v], sl, off));          // 2^(-inf) = 0 beyond m
                    sum += e[v];
                }
                acc[t] = e;
                CSAT_PIN_ACC(acc[t]);
            }
            sum += __shfl_xor(sum, 32, 64);
            const float inv = 1.f / sum;
            constexpr int NF = ZM == 2 ? 4 : 8;
            const uint4* vl = lds + (long long)a.v_lds * 64 + lane;          // (the host stages V~ in LDS for the kernels that use it)
            float* ab = arow ? arow + 4 * lh : nullptr;
            T* pb = prow ? prow + 4 * lh : nullptr;
            float* at = a.A + (((long long)z * a.n_q) / 32 + rt) * (32LL * a.ldA) + lane * 4;       // (a_tiled: ldA = 32 tiles)
#pragma unroll
            for (int t = 0; t < MTP; ++t) {
                f32x16 pr = acc[t];
#pragma unroll
                for (int v = 0; v < 16; ++v) pr[v] *= inv;
                if constexpr (VPACK) {
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const uint4 pf = make_uint4(f2bf_pk(pr[8 * s], pr[8 * s + 1]), f2bf_pk(pr[8 * s + 2], pr[8 * s + 3]),
                                                    f2bf_pk(pr[8 * s + 4], pr[8 * s + 5]), f2bf_pk(pr[8 * s + 6], pr[8 * s + 7]));
#pragma unroll
                        for (int dt = 0; dt < NF / 2; ++dt) mfma_group<T>(vl[(t * NF + dt * 2 + s) * 64], pf, zacc[dt]);
                    }
                }
                if (row_ok && t < mt_total) {
                    if (ab && a.a_tiled) {      // whole 1 KB pieces: what the decoder's wavefront loads back as they are
#pragma unroll
                        for (int g = 0; g < 4; ++g)
                            *(f32x4*)(at + (t * 4 + g) * 256) = f32x4{pr[4 * g], pr[4 * g + 1], pr[4 * g + 2], pr[4 * g + 3]};
                    } else if (ab) {
#pragma unroll
                        for (int g = 0; g < 4; ++g)
                            *(f32x4*)(ab + 32 * t + 8 * g) = f32x4{pr[4 * g], pr[4 * g + 1], pr[4 * g + 2], pr[4 * g + 3]};
                    }
                    if (pb) {
#pragma unroll
                        for (int g = 0; g < 4; ++g)
                            *(vec4_t*)(pb + 32 * t + 8 * g) = AttnVec<T>::pack(pr[4 * g], pr[4 * g + 1], pr[4 * g + 2], pr[4 * g + 3]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#undef CSAT_PIN_ACC
        }
        if constexpr (!VPACK) if (!emitted) {
            f32x16 acc[MTP];
            scores(0, acc);
            // the scale 1/sqrt(d_k) is positive, so the maximum commutes with it: one fused multiply-add per score
            const float sl = a.scale_log2e, off = -panel_max(acc) * sl;
            float sum = 0.f;
#pragma unroll
            for (int t = 0; t < MTP; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    acc[t][v] = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[t][v], sl, off));          // 2^(-inf) = 0 beyond m
                    sum += acc[t][v];
                }
            sum += __shfl_xor(sum, 32, 64);
            const float inv = 1.f / sum;
#pragma unroll
            for (int t = 0; t < MTP; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] *= inv;
            emit(0, acc);
        }
        } else {
            // every wavefront of the workgroup walks the same panels and barriers, whether its row tile exists or not
            const int panels = (mt_total + MTP - 1) / MTP;
            const float sl = a.scale_log2e;
            float run_max = -INFINITY, run_sum = 0.f;          // raw maximum; run_sum: this lane's share, relative to it
            float inv = 0.f;
            for (int sweep = 0; sweep < 2; ++sweep) {
                for (int p = 0; p < panels; ++p) {
                    const int mt0 = p * MTP, nt = mt_total - mt0 < MTP ? mt_total - mt0 : MTP;
                    __syncthreads();                           // the previous panel's fragments have been read
                    stage(mt0 * ns, nt * ns);
                    __builtin_amdgcn_s_waitcnt(0);
                    __syncthreads();
                    f32x16 acc[MTP];
                    scores(mt0, acc);
                    if (sweep == 0) {
                        const float nm = fmaxf(run_max, panel_max(acc));
                        float s = 0.f;
#pragma unroll
                        for (int t = 0; t < MTP; ++t)
#pragma unroll
                            for (int v = 0; v < 16; ++v) s += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[t][v], sl, -nm * sl));
                        run_sum = run_sum * __builtin_amdgcn_exp2f((run_max - nm) * sl) + s;     // first panel: 0 * 2^(-inf) = 0
                        run_max = nm;
                    } else {
#pragma unroll
                        for (int t = 0; t < MTP; ++t)
#pragma unroll
                            for (int v = 0; v < 16; ++v) acc[t][v] = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[t][v], sl, -run_max * sl)) * inv;
                        emit(mt0, acc);
                    }
                }
                if (sweep == 0) {
                    run_sum += __shfl_xor(run_sum, 32, 64);
                    inv = 1.f / run_sum;
                }
            }
        }

        if (row_ok && prow) {      // pad columns of the operand copy beyond the last tile
            for (int col = 32 * mt_total + 4 * lh; col < a.ldP; col += 8) *(vec4_t*)(prow + col) = AttnVec<T>::pack(0.f, 0.f, 0.f, 0.f);
        }
        if (row_ok && arow) {      // and of A~ (leading dimensions beyond the last tile do not occur in the library's own carving)
            for (int col = 32 * mt_total + 4 * lh; col < a.ldA; col += 8)
                for (int e = 0; e < 4; ++e)
                    if (col + e < a.ldA) arow[col + e] = 0.f;
        }
        if constexpr (WANT_Z) {
            if (row_ok) {
#pragma unroll
                for (int dt = 0; dt < NZ; ++dt) {
                    if (dt >= ndt) continue;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int dd0 = 32 * dt + 8 * g + 4 * lh;
                        if (dd0 >= d) continue;            // d is a multiple of 8: a group of four is inside or outside
                        if (a.Z)
                            *(vec4_t*)((T*)a.Z + ((long long)z * a.n_q + row) * d + dd0) =
                                AttnVec<T>::pack(zacc[dt][4 * g], zacc[dt][4 * g + 1], zacc[dt][4 * g + 2], zacc[dt][4 * g + 3]);
                        if (a.ZT) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float v = zacc[dt][4 * g + e];
                                T* t = (T*)a.ZT + (long long)z * a.strideT + (long long)(dd0 + e) * a.ldT + row;
                                if constexpr (kBf16) {
                                    const bf16_t hi = f2bf(v);
                                    t[0] = hi;
                                    t[a.ldT / 2] = f2bf(v - bf2f(hi));
                                } else {
                                    t[0] = v;
                                }
                            }
                        }
                    }
                }
            }
        }
    }
}

}  // namespace csat
