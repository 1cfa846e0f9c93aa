// Fused ISTA decoder for bf16 operands and m <= 512 (up to 16 tiles of 32): one launch runs every iteration.
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
// accumulator's row order (4h+{0..3}, 8+4h+{0..3} for lane half h).
//
// Phi is packed once per call, per chunk, as ready-to-use A fragments of GEMM-R in exactly that
// order (1 KB per wavefront load).  GEMM-U needs the transposed fragments (K along m instead of
// along the chunk's columns); it reads them from the same bytes with the transposing LDS load
// (ds_read_b64_tr_b16: within 16 lanes, lane L receives element L%4 of the 8-byte segments
// addressed by lanes L/4, 4+L/4, 8+L/4, 12+L/4), two loads per fragment.  One copy of Phi halves
// the L2->LDS traffic, which is what bounds the kernel when two copies are staged (a CU gets about
// 32 bytes per clock from L2 when all CUs pull at once).  Inside a fragment the 16-byte slot of lane
// (i, h) is 32h + (i ^ 4h), which keeps both kinds of load free of bank conflicts.
//
// The 4 wavefronts share each packed chunk through a ring of three LDS slots filled by direct
// global->LDS loads: in step c the chunk c is read transposed (GEMM-U), chunk c-1 plainly (GEMM-R)
// and chunk c+1 is in flight.  Needs at least two chunks (n > 32): the state of the next chunk is
// requested while the current one is computed.
#pragma once
#ifndef CSAT_FUSED_G
#define CSAT_FUSED_G 2      // fragments per LDS wait (4: image_text 2 % and the one-chunk schedule on short_video 1.5 % slower; 3, 6: slower at 16 tiles)
#endif
#include "csat_kernels.h"
#include <type_traits>

namespace csat {


struct IstaFusedArgs {
    const uint4* PhiPack;   // [NCT][SETF][64] 16-byte fragments of Phi (A operands of GEMM-R), slots permuted
    const float* Y;         // [rows, ldy] fp32 measurements, ldy = 32*MT, columns >= m zero
    float* state;           // [row tiles][NCT][4][64] float4: fp32 iterate in accumulator order
    uint8_t* mask;          // [row tiles][NCT][64]: bit g of a lane's byte = its float4 g of that tile is non-zero
    bf16_t* Xb;             // [rows, ldxb] bf16 copy of the final iterate (operand of the synthesis GEMM), or null
    float* Xout;            // [rows, n] final iterate in caller layout, or null
    long long rows;
    int n, nct, ldy, ldxb, iters;
    float mu, theta;
    // Work distribution: a unit is one group of 128 rows over one segment of the iterations; the
    // grid is persistent and takes units in order from a counter (see the kernel).
    int groups, segs;       // row groups (ceil(rows / 128)) and segments (1 <= segs <= iters)
    int* sync;              // [2 + groups] zeroed before the launch: next unit, (unused), segments done per group
    uint4* hand;            // [groups][4][2*MT][64] residual operands handed from one segment to the next (segs > 1)
    int* err;               // one word, zero before the launch unless an error is injected: set when a unit gives up
    long long spin_limit;   // polls a unit waits for the preceding segment of its group before it gives up
    int tape;               // two-chunk kernel only, > 0: the group-iterations in `tape` equal shares (see that kernel)
    // Two-chunk kernel only, optional: the synthesis C = X V in the last iteration (d = 64, n_q a multiple of 32, so
    // that the 32 rows of a wavefront lie in one head).  Vf: V as MFMA fragments, [heads][nct][2 slabs][2 tiles of d][64]
    // (pack_v_fragments_kernel); C: [rows][64] in bf16.  With Vf the bf16 copy Xb is not written.
    const uint4* Vf;
    bf16_t* C;
    int n_q;
    // Two-chunk kernel only: Y is laid out in accumulator tiles, [tile of 32 rows][MT][4][64 lanes] float4 (what lane
    // (row, h) holds as elements 4 g .. 4 g + 3 of tile mt), rows a multiple of 32: the attention kernel wrote it so.
    int y_tiled;
    int state_stream;      // one-chunk schedule: the iterate's loads and stores carry the non-temporal hint
};

// element (lane half h, slot q) of a 16-wide K slab -> index inside the slab
__host__ __device__ inline int slab_slot(int h, int q) { return 8 * (q >> 2) + 4 * h + (q & 3); }

// V [heads][n][64] (bf16) -> A fragments of C^T = V^T X^T in the order the decoder holds the new iterate: fragment
// (chunk ct, slab s, tile dt of d), lane (i, h), element q = V[32 ct + 16 s + slab_slot(h, q)][32 dt + i]; zero beyond n.
static __global__ void pack_v_fragments_kernel(const bf16_t* V, int n, int nct, long long total, uint4* out) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;     // one 16-byte piece each
    if (idx >= total) return;
    const int lane = (int)(idx & 63), i = lane & 31, h = lane >> 5;
    const int dt = (int)((idx >> 6) & 1), s = (int)((idx >> 7) & 1);
    const int ct = (int)((idx >> 8) % nct);
    const long long z = idx / (256LL * nct);
    const bf16_t* v = V + z * (long long)n * 64 + 32 * dt + i;
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 8; q += 2) {
        const int k0 = 32 * ct + 16 * s + slab_slot(h, q), k1 = 32 * ct + 16 * s + slab_slot(h, q + 1);
        const uint32_t lo = k0 < n ? v[(long long)k0 * 64] : 0, hi = k1 < n ? v[(long long)k1 * 64] : 0;
        w[q / 2] = lo | (hi << 16);
    }
    out[idx] = uint4{w[0], w[1], w[2], w[3]};
}


// Fragments of one chunk: 2*MT, padded to a multiple of 4 so that each of the 4 wavefronts stages
// an equal, contiguous share.
__host__ __device__ constexpr int ista_fused_set_frags(int MT) { return (2 * MT + 3) / 4 * 4; }

// 16-byte slot of lane (i, h) inside a 1 KB fragment
__host__ __device__ inline int frag_slot(int i, int h) { return 32 * h + (i ^ (4 * h)); }

// Packs Phi [m, n] (bf16, row-major) into the fragment order described above; zero beyond m, n and
// in the pad fragments.  Layout [chunk][fragment][slot] of 16-byte pieces; fragment f = s2*MT + mt
// holds rows 32*mt .. 32*mt+31 of Phi and the 16 columns of slab s2 of the chunk.
static __global__ void pack_phi_fragments_kernel(const bf16_t* Phi, int m, int n, int MT, int nct, uint4* out) {
    const int SETF = ista_fused_set_frags(MT);
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;     // one 16-byte piece each
    long long total = (long long)nct * SETF * 64;
    if (idx >= total) return;
    int slot = (int)(idx & 63);
    int f = (int)((idx >> 6) % SETF);
    int ct = (int)(idx / (64LL * SETF));
    int lh = slot >> 5, li = (slot & 31) ^ (4 * lh);       // inverse of frag_slot
    bf16_t v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = 0;
    if (f < 2 * MT) {
        int s2 = f / MT, mt = f % MT;   // slab-major: consecutive fragments feed different accumulators
        int l = 32 * mt + li;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            int j = 32 * ct + 16 * s2 + slab_slot(lh, q);
            if (l < m && j < n) v[q] = Phi[(long long)l * n + j];
        }
    }
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16);
    o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16);
    o.w = v[6] | ((uint32_t)v[7] << 16);
    out[idx] = o;
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// transposing 8-byte LDS load (see the top of this file), explicit like lds_read16
template <int OFF>
__device__ __forceinline__ void lds_read8_tr(u32x2& dst, uint32_t byte_addr) {
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(byte_addr), "n"(OFF));
}
// at most N LDS reads outstanding (N <= 15, the counter's range)
template <int N>
__device__ __forceinline__ void lds_wait_n() {
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N < 15 ? N : 15));
}
// keeps the consumers of a loaded register behind the preceding wait
__device__ __forceinline__ void lds_pin(u32x4& a) { asm volatile("" : "+v"(a)); }
__device__ __forceinline__ void lds_pin(u32x2& a, u32x2& b) { asm volatile("" : "+v"(a), "+v"(b)); }

template <int BASE>
__device__ __forceinline__ bf16x8 cvt8(const f32x16& a, float sign) {
    bf16x8 r;
#pragma unroll
    for (int q = 0; q < 8; ++q) r[q] = (__bf16)(sign * a[BASE + q]);
    return r;
}

// soft threshold eta_theta(u) = u - clamp(u, -theta, theta): exact zero for |u| <= theta
__device__ __forceinline__ float soft_threshold(float u, float theta) {
    return u - __builtin_amdgcn_fmed3f(u, -theta, theta);
}

// LDS of the fused decoder: three slots of packed Phi chunks plus 2 slots of old iterate
constexpr int ista_fused_state_slots(int) { return 2; }   // 3 (two-step lookahead) measured no faster
constexpr size_t ista_fused_lds_bytes(int MT) {
    return (size_t)3 * ista_fused_set_frags(MT) * 1024 + ista_fused_state_slots(MT) * 16384;
}

// SPARSE: keep the fp32 iterate sparse in memory (per-lane masks); otherwise every lane reads and
// writes all of its state every iteration.
// THIN: for launches with so few rows that every 32-row tile can have a CU of its own.  A workgroup
// then carries one tile: its first wavefront computes (with the CU's LDS bandwidth to itself), the
// other three only stage their share of the packed chunks and keep the barriers.
template <int MT, bool SPARSE, bool THIN = false>
__global__ __launch_bounds__(256, 1) void ista_fused_kernel(IstaFusedArgs a) {
    // LDS (byte offsets): three slots of packed Phi chunks, then two slots of the old iterate
    // (4 x 4 KB, one block per wavefront: its 32 rows x 32 columns, accumulator order)
    extern __shared__ uint4 lds[];
    constexpr int SETF = ista_fused_set_frags(MT), FW = SETF / 4;   // fragments per chunk, per wavefront
    constexpr int HALF = SETF * 1024;              // bytes of one packed chunk
    constexpr int OFF_X = 3 * HALF, XSLOT = 16384;
    // the old iterate comes from HBM, not from L2 like Phi: where LDS has room for a third slot it is
    // requested two steps ahead of its use instead of one
    constexpr int NXS = ista_fused_state_slots(MT), XLA = NXS - 1;
    constexpr int G = CSAT_FUSED_G;                // fragments per software-pipeline group
    // One accumulator chain for GEMM-U, summed in slab order, as on the two-chunk schedule (csat_ista_fused2.h):
    // every variant of the decoder then rounds alike.  (A second chain hides the dependency between consecutive
    // MFMAs but its sum costs more than that: 3.97 against 3.88 ms measured on the two-chunk schedule.)
    constexpr bool TWO_CHAINS = false;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lh = lane >> 5;
    // set per unit of work (see the loop at the end of the kernel)
    long long rt = 0;              // 32-row tile of this wavefront
    long long row = 0;
    bool row_ok = false;
    const int nct = a.nct;
    f32x4* st = nullptr;           // wavefront-uniform; + (ct*4 + g)*64 + lane
    // lane offset re-materialised (opaquely) where addresses are formed, so that per-lane 64-bit
    // addresses are not kept live across the loops
    auto lane_off = [&]() { uint32_t v = lane; asm volatile("" : "+v"(v)); return v; };
    const uint32_t lds0 = (uint32_t)(size_t)(lds_ptr_t)lds;
    const uint32_t lane16 = lds0 + lane * 16;
    // GEMM-R fragments: this lane's slot.  GEMM-U fragments, read transposed: lanes 16G..16G+15 serve
    // column slab G%2 and K half G/2; lane 4e+q of them supplies the segment of Phi row 4*(G/2)+e
    // (+16 per further K slab, +8 for the fragment's upper half) holding the slab's columns 4q..4q+3,
    // i.e. the 8-byte half q/2 of the slot of lane half q%2.
    const uint32_t nat16 = lds0 + frag_slot(lane & 31, lane >> 5) * 16;
    const uint32_t tr8 = lds0 + ((lane >> 4) & 1) * (MT * 1024) + frag_slot(4 * (lane >> 5) + ((lane & 15) >> 2), lane & 1) * 16 +
                         ((lane >> 1) & 1) * 8;

    // The iterate is sparse after the first threshold, so its fp32 state is kept sparse in memory
    // too: a lane reads and writes only those of its four float4 per tile that are non-zero, told by
    // a mask byte per lane and tile.  mT: mask of the chunk thresholded in this step, mD: of the chunk
    // whose old iterate is requested in this step, mL: being loaded for the step after.
    uint32_t mT = 0, mD = 0, mL = 0;
    uint8_t* mk = nullptr;         // wavefront-uniform; + ct*64 + lane

    // Requests of one pipeline step, global -> LDS: this wavefront's quarter of the packed chunk ct_p
    // into ring slot slot_p, and its own old iterate of chunk ct_x.  They all go out at the very
    // start of the step (issuing them between the MFMA groups instead measured 12% slower).
    struct Requests { int ct_p, slot_p, ct_x, slot_x, ct_m; bool want_p, want_x, want_m; };
    // One address per 4 requests: the instruction's immediate offset moves the global and the LDS
    // address together, and both layouts advance 1 KB per fragment.
    auto issue_chunk = [&](int ct, int slot, uint32_t ulane) {
        const uint4* src = a.PhiPack + ((long long)ct * SETF + wave * FW) * 64 + ulane;
        char* dst = (char*)lds + slot * HALF + wave * FW * 1024;
#pragma unroll
        for (int i = 0; i < FW; ++i) {
            const int blk = i / 4;
            switch (i % 4) {
                case 0: __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + blk * 256), (lds_ptr_t)(dst + blk * 4096), 16, 0, 0); break;
                case 1: __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + blk * 256), (lds_ptr_t)(dst + blk * 4096), 16, 1024, 0); break;
                case 2: __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + blk * 256), (lds_ptr_t)(dst + blk * 4096), 16, 2048, 0); break;
                default: __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + blk * 256), (lds_ptr_t)(dst + blk * 4096), 16, 3072, 0); break;
            }
        }
    };
    // THIN: wavefronts 1..3 stage the whole chunk between them, fragment f by wavefront 1 + f % 3
    auto issue_chunk_thin = [&](int ct, int slot, uint32_t ulane) {
        const uint4* src = a.PhiPack + (long long)ct * SETF * 64 + ulane;
        char* dst = (char*)lds + slot * HALF;
#pragma unroll
        for (int i = 0; i < (SETF + 2) / 3; ++i) {
            const int f = wave - 1 + 3 * i;
            if (f < SETF) __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + f * 64), (lds_ptr_t)(dst + f * 1024), 16, 0, 0);
        }
    };
    auto issue_state = [&](const Requests& q, uint32_t ulane) {
        const f32x4* src = st + q.ct_x * 256 + ulane;
        char* dst = (char*)lds + OFF_X + q.slot_x * XSLOT + wave * 4096;
        if (a.state_stream) {
            if (!SPARSE || (mD & 1)) __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 0, 2);
            if (!SPARSE || (mD & 2)) __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 1024, 2);
            if (!SPARSE || (mD & 4)) __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 2048, 2);
            if (!SPARSE || (mD & 8)) __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 3072, 2);
            return;
        }
        if (!SPARSE || (mD & 1)) __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 0, 0);
        if (!SPARSE || (mD & 2)) __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 1024, 0);
        if (!SPARSE || (mD & 4)) __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 2048, 0);
        if (!SPARSE || (mD & 8)) __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 3072, 0);
    };
    auto issue_all = [&](const Requests& q) {
        const uint32_t ulane = lane_off();
        if (!THIN && q.want_p) issue_chunk(q.ct_p, q.slot_p, ulane);      // THIN: the other wavefronts stage
        if (q.want_x) issue_state(q, ulane);
    };

    f32x16 racc[MT];       // minus Phi x, accumulated over the chunks of one iteration
    bf16x8 rb[2 * MT];     // residual r = y - Phi x of the current iterate, as MFMA B operands
    f32x16 u;              // U of the chunk whose threshold step is still pending
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) racc[mt][v] = 0.f;
    const float* yrow = nullptr;   // rows past the end read a valid row; their results are never stored

    // The accumulators of the next residual start from y (load_y, issued in the first step of an
    // iteration, a whole step before GEMM-R touches them: the loads land straight in the accumulator
    // registers while GEMM-U runs) and collect -Phi x over the chunks, so at the iteration boundary
    // they hold r = y - Phi x and only need converting into the bf16 operands of the next GEMM-U.
    auto load_y = [&]() {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 y4 = *(const f32x4*)(yrow + 32 * mt + 8 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) racc[mt][4 * g + e] = y4[e];
            }
    };
    auto boundary = [&]() {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            rb[2 * mt] = cvt8<0>(racc[mt], 1.f);
            rb[2 * mt + 1] = cvt8<8>(racc[mt], 1.f);
        }
    };

    // One pipeline step.  DO_U: GEMM-U of chunk c.  DO_T: threshold of chunk c-1 (its U sits in `u`),
    // interleaved with the GEMM-U MFMAs.  DO_R: GEMM-R of chunk c-1 (needs DO_T).  LAST: final
    // iteration, the threshold writes the outputs instead of the state.
    // pslot: ring slot of chunk c; chunk c-1 sits in the slot before it.
    auto step = [&](auto do_u, auto do_t, auto do_r, auto is_last, int c, bool first, int xslot, int pslot, const Requests& q,
                    auto do_y) {
        constexpr bool DO_U = decltype(do_u)::value, DO_T = decltype(do_t)::value, DO_Y = decltype(do_y)::value;
        constexpr bool DO_R = decltype(do_r)::value, LAST = decltype(is_last)::value;
        constexpr int NU = DO_U ? 2 * MT : 0, NR = DO_R ? 2 * MT : 0, NF = NU + NR;
        constexpr int NG = (NF + G - 1) / G;
        // LDS loads of group k: two (transposing) per GEMM-U fragment, one per GEMM-R fragment
        auto ops = [](int k) constexpr {
            int n = 0;
            for (int i = 0; i < G; ++i) n += (k * G + i < NU) ? 2 : (k * G + i < NF) ? 1 : 0;
            return n;
        };
        constexpr int N0 = ops(0);                                 // LDS loads issued for group 0
        constexpr int NTG = NU / G;                               // groups made of GEMM-U fragments only
        constexpr int EPG = NTG > 0 ? (16 + NTG - 1) / NTG : 16;   // threshold elements per such group
        const uint32_t baseA = tr8 + pslot * HALF;                       // chunk c, read transposed
        const uint32_t baseB = nat16 + (pslot == 0 ? 2 : pslot - 1) * HALF;  // chunk c-1
        const uint32_t baseX = lane16 + OFF_X + xslot * XSLOT + wave * 4096;       // old iterate of chunk c-1

        if constexpr (SPARSE) {
            if (c > 0) { mT = mD; mD = mL; }
            mL = 0;
            if (q.want_m) mL = mk[q.ct_m * 64 + lane_off()];
        }
        issue_all(q);
        if constexpr (DO_Y) load_y();
        u32x4 fr[2][G];        // GEMM-R fragments
        u32x2 ft[2][G][2];     // GEMM-U fragments, lower and upper K half
        u32x4 xs[4];
        f32x16 un, un1, x;
        bf16x8 xb0, xb1;
        if constexpr (DO_T) {
            lds_read16<0>(xs[0], baseX);
            lds_read16<1024>(xs[1], baseX);
            lds_read16<2048>(xs[2], baseX);
            lds_read16<3072>(xs[3], baseX);
        }
        auto fetch = [&](auto kc, auto ic) {      // fragment number kc*G+ic of this step
            constexpr int k = decltype(kc)::value, i = decltype(ic)::value, f = k * G + i;
            if constexpr (f < NU) {        // K slab f of m: row tile f/2, rows 16*(f%2) .. +15
                lds_read8_tr<(f >> 1) * 1024 + (f & 1) * 256>(ft[k & 1][i][0], baseA);
                lds_read8_tr<(f >> 1) * 1024 + (f & 1) * 256 + 128>(ft[k & 1][i][1], baseA);
            } else if constexpr (f < NF) lds_read16<(f - NU) * 1024>(fr[k & 1][i], baseB);
        };
        auto threshold = [&](int v) {
            const bool have = SPARSE ? ((mT >> (v >> 2)) & 1) != 0 : !first;
            float uu = (have ? __builtin_bit_cast(f32x4, xs[v >> 2])[v & 3] : 0.f) + a.mu * u[v];
            float xv = soft_threshold(uu, a.theta);
            // keeps the arithmetic where it is written, between the MFMAs of its group: the value is first
            // used behind the branches of the write-out, and the compiler would otherwise sink it there
            asm volatile("" : "+v"(xv));
            x[v] = xv;
        };
        auto finish_t = [&]() {                   // all 16 elements thresholded
            if constexpr (!LAST) {
                const uint32_t ulane = lane_off();
                uint32_t nz = 0;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 o = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
                    if (!SPARSE || o[0] != 0.f || o[1] != 0.f || o[2] != 0.f || o[3] != 0.f) {
                        if (a.state_stream) __builtin_nontemporal_store(o, st + ((c - 1) * 4 + g) * 64 + ulane);
                        else st[((c - 1) * 4 + g) * 64 + ulane] = o;
                        nz |= 1u << g;
                    }
                }
                if constexpr (SPARSE) mk[(c - 1) * 64 + ulane] = (uint8_t)nz;
                xb0 = cvt8<0>(x, -1.f);
                xb1 = cvt8<8>(x, -1.f);
            } else if (row_ok) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = 32 * (c - 1) + 8 * g + 4 * lh;
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
        };
#pragma unroll
        for (int v = 0; v < 16; ++v) { un[v] = 0.f; un1[v] = 0.f; }

        auto fetch_group = [&](auto self, auto kc, auto ic) {     // all G fragments of group kc
            constexpr int i = decltype(ic)::value;
            if constexpr (i < G) {
                fetch(kc, ic);
                self(self, kc, std::integral_constant<int, i + 1>{});
            }
        };
        if constexpr (NG > 0) fetch_group(fetch_group, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        if constexpr (DO_T && NTG == 0) {          // nothing to hide the threshold behind
            lds_wait_n<N0>();
            lds_pin(xs[0]); lds_pin(xs[1]); lds_pin(xs[2]); lds_pin(xs[3]);
#pragma unroll
            for (int v = 0; v < 16; ++v) threshold(v);
            finish_t();
        }
        auto group = [&](auto kc) {
            constexpr int k = decltype(kc)::value;
            constexpr int NEXT = (k + 1 < NG) ? ops(k + 1) : 0;   // loads issued now
            if constexpr (k + 1 < NG) fetch_group(fetch_group, std::integral_constant<int, k + 1>{}, std::integral_constant<int, 0>{});
            if constexpr (DO_T && NTG > 0 && k == 0) {
                lds_wait_n<NEXT + N0>();
                lds_pin(xs[0]); lds_pin(xs[1]); lds_pin(xs[2]); lds_pin(xs[3]);
            }
            lds_wait_n<NEXT>();
#pragma unroll
            for (int i = 0; i < G; ++i) {
                if (k * G + i < NU) lds_pin(ft[k & 1][i][0], ft[k & 1][i][1]);
                else if (k * G + i < NF) lds_pin(fr[k & 1][i]);
            }
            if constexpr (DO_T && NTG > 0 && k == NTG) finish_t();
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const int f = k * G + i;
                if (f < NU) {
                    // two accumulator chains: an MFMA never waits for the one issued just before it
                    const u32x4 fa = __builtin_shufflevector(ft[k & 1][i][0], ft[k & 1][i][1], 0, 1, 2, 3);
                    if (TWO_CHAINS && (f & 1)) un1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa), rb[f], un1, 0, 0, 0);
                    else un = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa), rb[f], un, 0, 0, 0);
                } else if (f < NF) {
                    const int r = f - NU;          // fragment r: column slab r / MT, accumulator tile r % MT
                    racc[r % MT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fr[k & 1][i]),
                                                                           (r >= MT) ? xb1 : xb0, racc[r % MT], 0, 0, 0);
                }
            }
            if constexpr (DO_T && NTG > 0 && k < NTG) {
#pragma unroll
                for (int e = 0; e < EPG; ++e)
                    if (k * EPG + e < 16) threshold(k * EPG + e);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        // NG <= 4*MT/G = 16 groups
        auto run = [&](auto self, auto kc) {
            constexpr int k = decltype(kc)::value;
            if constexpr (k < NG) {
                group(kc);
                self(self, std::integral_constant<int, k + 1>{});
            }
        };
        run(run, std::integral_constant<int, 0>{});
        if constexpr (DO_T && LAST && NTG > 0) {
            if constexpr (NTG >= NG) finish_t();   // no trailing group ran it
        }
        if constexpr (DO_U) {
#pragma unroll
            for (int v = 0; v < 16; ++v) u[v] = TWO_CHAINS ? un[v] + un1[v] : un[v];
        }
    };

    using T_ = std::true_type;
    using F_ = std::false_type;
    // Requests are issued one step ahead of their use: during step c the packed chunk c+1 (read by
    // steps c+1 and c+2; after the last chunk of an iteration, chunk 0 for the next iteration) and
    // the old iterate of chunk c (used by step c+1).  Each step starts by waiting for what the
    // previous step requested, for every wavefront; the slot being filled in step c was last read
    // in step c-1.
    // A step that requested old-iterate blocks issued them last, as exactly 4 loads: leaving 4
    // operations outstanding still guarantees (loads return in order) that every fragment request,
    // and every old-iterate request of earlier steps, has landed.
    auto sync = [&](bool state_in_flight) {
        if (XLA == 2 && state_in_flight) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };
    int ps = 0;            // ring slot of the chunk whose GEMM-U runs in the coming step
    // In step c also: old iterate of chunk c+XLA-1 (thresholded in step c+XLA), which for the last
    // XLA-1 steps of an iteration is a chunk of the next iteration.  Old-iterate slots rotate with a
    // counter that runs on across iterations: kb = (iteration * nct) mod NXS.
    bool inflight = false;
    int kb = 0;
    // last: nothing is requested for the iteration after this one (final iteration of a segment)
    auto requests = [&](int c, bool first, bool last) {
        const int cx = c + XLA - 1;
        const bool wx = cx < nct ? !first : (!last && cx - nct < XLA - 1);
        // mask of the chunk whose old iterate the next step requests
        const int cm = cx + 1;
        const bool wm = cm < nct ? !first : (!last && cm - nct < XLA);
        return Requests{c + 1 < nct ? c + 1 : 0, ps == 2 ? 0 : ps + 1, cx < nct ? cx : cx - nct, (kb + cx) % NXS,
                        cm < nct ? cm : cm - nct, c < nct && (c + 1 < nct || !last), wx, wm && c < nct};
    };
    auto rslot = [&](int c) { return (kb + c - 1 + NXS) % NXS; };
    auto advance = [&]() { ps = ps == 2 ? 0 : ps + 1; };

    // Work distribution.  The rows of a group stay with one workgroup for a whole segment of the
    // iterations, not for all of them: with G groups on P CUs a launch of whole-length groups takes
    // ceil(G / P) rounds, while units of 1/S of the length take ceil(G S / P) / S (600 groups on 256
    // CUs: 3 against 2.4).  Units are numbered segment-major and handed out in order by an atomic
    // counter; a unit (segment k > 0) waits for segment k-1 of the same group, which was handed out
    // earlier and never waits for a later unit, so every wait ends.  The residual operands rb are
    // what one segment hands to the next (the iterate itself lives in memory already).
    __shared__ int s_unit, s_err;
    const int total = a.groups * a.segs;
    if constexpr (THIN) {
        // Wavefronts 1..3 own no rows: they walk the same schedule of units, steps and barriers as the
        // first wavefront and only issue their share of the packed chunks.
        if (wave != 0) {
            for (;;) {
                __syncthreads();                       // the first wavefront has published the unit
                const int unit = s_unit;
                if (unit >= total) break;
                const int seg = unit / a.groups;
                const int t0 = (int)((long long)seg * a.iters / a.segs), t1 = (int)((long long)(seg + 1) * a.iters / a.segs);
                if (seg > 0) {
                    __syncthreads();                   // end of its wait for the previous segment
                    if (s_err) break;
                }
                ps = 0;
                kb = 0;
                issue_chunk_thin(0, 0, lane_off());
                const int tn = t1 < a.iters ? t1 : a.iters - 1;
                for (int t = t0; t < tn; ++t) {
                    for (int c = 0; c <= nct; ++c) {
                        sync(false);
                        const Requests q = requests(c, t == 0, t + 1 == t1);
                        if (q.want_p) issue_chunk_thin(q.ct_p, q.slot_p, lane_off());
                        if (c < nct) advance();
                    }
                    kb = (kb + nct) % NXS;
                }
                if (t1 == a.iters) {
                    for (int c = 0; c < nct; ++c) {
                        sync(false);
                        const Requests q = requests(c, a.iters == 1, true);
                        if (q.want_p) issue_chunk_thin(q.ct_p, q.slot_p, lane_off());
                        advance();
                    }
                    sync(false);
                } else {
                    __syncthreads();                   // the hand-over's barrier
                }
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();
            }
            return;
        }
    }
    for (;;) {
        if (threadIdx.x == 0) {
            s_unit = atomicAdd(a.sync, 1);
            s_err = 0;
        }
        __syncthreads();
        const int unit = s_unit;
        if (unit >= total) break;
        const int seg = unit / a.groups, grp = unit - seg * a.groups;
        const int t0 = (int)((long long)seg * a.iters / a.segs), t1 = (int)((long long)(seg + 1) * a.iters / a.segs);
        rt = THIN ? (long long)grp : (long long)grp * 4 + wave;
        row = rt * 32 + (lane & 31);
        row_ok = row < a.rows;
        st = (f32x4*)a.state + rt * nct * 256;
        mk = a.mask + rt * nct * 64;
        yrow = a.Y + (row_ok ? row : a.rows - 1) * a.ldy + 4 * lh;
        if (seg > 0) {
            if (threadIdx.x == 0) {     // bounded wait: a limit that is never reached unless the launch is broken
                long long spins = 0;
                for (;;) {
                    // some unit gave up already (its rows stay unfinished, so the call has failed): stop as well
                    if (__hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { s_err = 1; break; }
                    if (__hip_atomic_load(a.sync + 2 + grp, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) >= seg) break;
                    if (++spins > a.spin_limit) {
                        __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        s_err = 1;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(64);
                }
            }
            __syncthreads();
            if (s_err) break;
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        if (seg == 0) {            // x = 0: r = y
            load_y();
            boundary();
        } else {                   // residual operands left by the previous segment
            const uint4* hp = a.hand + ((long long)rt * 2 * MT) * 64 + lane_off();
#pragma unroll
            for (int f = 0; f < 2 * MT; ++f) rb[f] = __builtin_bit_cast(bf16x8, hp[f * 64]);
        }
        ps = 0;
        kb = 0;
        inflight = false;
        if constexpr (SPARSE) {      // the mask pipeline restarts: chunk 0's mask is needed by the first step
            mT = 0;
            mL = 0;
            mD = t0 > 0 ? mk[lane_off()] : 0;
        }
        issue_all(Requests{0, 0, 0, 0, 0, true, false, false});
        const int tn = t1 < a.iters ? t1 : a.iters - 1;       // normal iterations of this unit: [t0, tn)
        for (int t = t0; t < tn; ++t) {
            const bool first = t == 0;
            const bool seg_last = t + 1 == t1;
            {
                sync(inflight);
                const Requests q = requests(0, first, seg_last);
                step(T_{}, F_{}, F_{}, F_{}, 0, first, 0, ps, q, T_{});
                inflight = q.want_x;
                advance();
            }
            for (int c = 1; c < nct; ++c) {
                sync(inflight);
                const Requests q = requests(c, first, seg_last);
                step(T_{}, T_{}, T_{}, F_{}, c, first, rslot(c), ps, q, F_{});
                inflight = q.want_x;
                advance();
            }
            {
                sync(inflight);
                const Requests q = requests(nct, first, seg_last);
                step(F_{}, T_{}, T_{}, F_{}, nct, first, rslot(nct), ps, q, F_{});
                inflight = q.want_x;
            }
            kb = (kb + nct) % NXS;
            boundary();            // residual operands of the next iteration
        }
        if (t1 == a.iters) {   // last iteration: no residual update, outputs instead of state
            const bool first = a.iters == 1;
            {
                sync(inflight);
                const Requests q = requests(0, first, true);
                step(T_{}, F_{}, F_{}, T_{}, 0, first, 0, ps, q, F_{});
                inflight = q.want_x;
                advance();
            }
            for (int c = 1; c < nct; ++c) {
                sync(inflight);
                const Requests q = requests(c, first, true);
                step(T_{}, T_{}, F_{}, T_{}, c, first, rslot(c), ps, q, F_{});
                inflight = q.want_x;
                advance();
            }
            sync(inflight);
            step(F_{}, T_{}, F_{}, T_{}, nct, first, rslot(nct), ps, Requests{0, 0, 0, 0, 0, false, false, false}, F_{});
        } else {               // hand the residual operands to the next segment
            uint4* hp = a.hand + ((long long)rt * 2 * MT) * 64 + lane_off();
#pragma unroll
            for (int f = 0; f < 2 * MT; ++f) hp[f * 64] = __builtin_bit_cast(uint4, rb[f]);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __syncthreads();
            if (threadIdx.x == 0) __hip_atomic_store(a.sync + 2 + grp, seg + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        // nothing of this unit may still be in flight towards LDS when the next one starts staging
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }
}

}  // namespace csat
