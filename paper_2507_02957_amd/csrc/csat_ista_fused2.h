// Fused ISTA decoder, second schedule: the same arithmetic, registers and memory layouts as
// ista_fused_kernel (csat_ista_fused.h: rows on the MFMA N axis, residual operands rb and residual
// accumulators racc in registers, one packed copy of Phi per 32-column chunk read plainly by GEMM-R and
// transposed by GEMM-U), walked in steps of TWO chunks (a, b) with one workgroup barrier per step:
//
//     phase 1   U_a = Phi_a^T r                                   (GEMM-U of chunk a; requests for the next step)
//     phase 2   U_b = Phi_b^T r        with  x_a = eta(x_a + mu U_a)  between its MFMAs
//     phase 3   racc -= Phi_a x_a      with  x_b = eta(x_b + mu U_b)  between its MFMAs, state of a written out
//     phase 4   racc -= Phi_b x_b      state of b written out
//
// Both products of a chunk run in the same step, so only the step's own pair of chunks and the pair in flight
// are in LDS (a ring of two slots of two chunks), and everything that happens once per step - the barrier, the
// wait for the staged data, the staging requests, the ramp of the fragment pipeline - is paid once per 64
// columns instead of once per 32.  The old iterate of a step's two chunks sits in a block of LDS private to the
// wavefront; a half of the block is refilled for the next step as soon as its values are in registers (three
// phases before it is read again), so no second block is needed.
//
// With one wavefront per SIMD the kernel is bound by what that wavefront can issue: an MFMA keeps the matrix pipe
// for 32 cycles, the 1 KB fragment read it needs takes about half of that in issue time, and what is left holds
// about three more instructions.  So all other work of a step (staging requests, the threshold arithmetic a
// stage of four independent instructions at a time, stores, refills) is cut into slots, one behind each MFMA,
// and kept lean: global addresses are a scalar base plus a 32-bit lane offset, a lane without an old iterate
// reads a block of zeros instead of selecting per element, accumulator elements are read where they are used.
//
// n is handled in whole pairs: the chunk count is rounded up to even, the packed Phi holds a zero chunk there,
// whose iterate stays zero and is never stored beyond the real columns.
#pragma once
#include "csat_ista_fused.h"

namespace csat {

#ifndef CSAT_FUSED2_PIN
#define CSAT_FUSED2_PIN 1                    // (measured 2 % faster with the registers pinned behind each wait than without)
#endif
// In LDS the fragments of column slab 1 of a chunk sit this many bytes further than in the packed chunk.  The
// transposing reads of GEMM-U take slab 0 with lanes 0-15 and slab 1 with lanes 16-31 of each half wavefront; a whole
// number of KB between the two sends both to the same 32 of the 64 banks (counted as bank-conflict cycles for a third
// of the LDS activity), 128 bytes more sends them to different halves (none counted).
#ifndef CSAT_FUSED2_SLAB_SHIFT
#define CSAT_FUSED2_SLAB_SHIFT 128
#endif
// LDS: two ring slots of two packed chunks, the old-iterate blocks (8 KB per wavefront), and 4 KB of zeros that a
// lane reads instead of its block when it has no old iterate (so the threshold arithmetic needs no select)
constexpr int ista_fused2_chunk_bytes(int MT) { return ista_fused_set_frags(MT) * 1024 + CSAT_FUSED2_SLAB_SHIFT; }
constexpr size_t ista_fused2_lds_bytes(int MT) { return (size_t)4 * ista_fused2_chunk_bytes(MT) + 4 * 8192 + 4096; }

#ifndef CSAT_FUSED2_REQUESTS_IN_PHASE
#define CSAT_FUSED2_REQUESTS_IN_PHASE 4      // staging requests behind the MFMAs of this many phases (0: before the step)
#endif
#ifndef CSAT_FUSED2_G
#define CSAT_FUSED2_G 3                      // fragments per pipeline group (2: 0.7 % slower on short_video, 1 and 4: 1-7 %)
#endif
#ifndef CSAT_FUSED2_LOOKAHEAD
#define CSAT_FUSED2_LOOKAHEAD 2              // items whose fragment reads are in flight ahead of the one being multiplied
#endif

// LDS reads of the fragments of group k of phase p (phases 0, 1: two transposing reads per fragment)
constexpr int fused2_frag_loads(int p, int k, int G, int NF) {
    int n = 0;
    for (int i = 0; i < G; ++i) n += (k * G + i < NF) ? (p < 2 ? 2 : 1) : 0;
    return n;
}
// LDS reads issued for pipeline item q = p * NG + k (none beyond the step's NP phases): its fragments, preceded by
// the four old-iterate reads when it opens phase 1 or 2
constexpr int fused2_item_loads(int q, int G, int NF, int NG, int NP) {
    if (q >= NP * NG) return 0;
    const int p = q / NG, k = q % NG;
    return fused2_frag_loads(p, k, G, NF) + ((k == 0 && (p == 1 || p == 2)) ? 4 : 0);
}
constexpr int fused2_ahead_loads(int q, int LA, int G, int NF, int NG, int NP) {
    int n = 0;
    for (int j = 1; j <= LA; ++j) n += fused2_item_loads(q + j, G, NF, NG, NP);
    return n;
}

template <int MT, bool SPARSE>
__global__ __launch_bounds__(256, 1) void ista_fused2_kernel(IstaFusedArgs a) {
    extern __shared__ uint4 lds[];
    constexpr int SETF = ista_fused_set_frags(MT), FW = SETF / 4;   // fragments per chunk, per wavefront
    constexpr int HALF = ista_fused2_chunk_bytes(MT);   // bytes of one packed chunk in LDS
    constexpr int SHIFT = CSAT_FUSED2_SLAB_SHIFT;
    constexpr int PAIR = 2 * HALF;                 // bytes of a ring slot
    constexpr int OFF_X = 2 * PAIR;                // old-iterate blocks
    constexpr int OFF_Z = OFF_X + 4 * 8192;        // zeros
    constexpr int G = CSAT_FUSED2_G;               // fragments per software-pipeline group
    constexpr int NF = 2 * MT;                     // fragments (= MFMAs) of one product of one chunk
    constexpr int NG = (NF + G - 1) / G;
    // items the LDS reads run ahead of the MFMAs (one for the thinnest instantiations: the threshold arithmetic needs
    // slots before the old-iterate registers are reloaded, see step)
    constexpr int LA = (NG - CSAT_FUSED2_LOOKAHEAD) * G > 2 ? CSAT_FUSED2_LOOKAHEAD : 1, NB = LA + 1;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lh = lane >> 5;
    long long rt = 0, row = 0;
    bool row_ok = false;
    const int nct = a.nct;                         // even
    const int S = nct / 2;                         // steps per iteration
    f32x4* st = nullptr;                           // wavefront-uniform; + (ct*4 + g)*64 + lane
    uint8_t* mk = nullptr;                         // wavefront-uniform; + ct*64 + lane
    auto lane_off = [&]() { uint32_t v = lane; asm volatile("" : "+v"(v)); return v; };
    // Global addresses are a wavefront-uniform base plus a 32-bit per-lane byte offset: the loads and stores take
    // the base from scalar registers, and the vector unit does no address arithmetic between the MFMAs.
    const uint32_t lane16b = lane * 16;
    auto at16 = [&](const void* base) { return (const char*)base + lane16b; };
    const uint32_t lds0 = (uint32_t)(size_t)(lds_ptr_t)lds;
    const uint32_t lane16 = lds0 + lane * 16;
    const uint32_t nat16 = lds0 + frag_slot(lane & 31, lane >> 5) * 16;
    const uint32_t tr8 = lds0 + ((lane >> 4) & 1) * (MT * 1024 + SHIFT) + frag_slot(4 * (lane >> 5) + ((lane & 15) >> 2), lane & 1) * 16 +
                         ((lane >> 1) & 1) * 8;
    const uint32_t xblock = lane16 + OFF_X + wave * 8192;        // this wavefront's old-iterate block (a: +0, b: +4096)
    const uint32_t zblock = lane16 + OFF_Z;
    lds[OFF_Z / 16 + threadIdx.x] = uint4{0u, 0u, 0u, 0u};        // (the barrier of the unit loop orders this before any read)

    f32x16 racc[MT];
    bf16x8 rb[2 * MT];
    f32x16 xA, xB;         // new iterate of chunks a and b
    f32x16 cacc[2];        // C^T of this wavefront's rows (two tiles of d), last iteration with a.Vf
    const uint4* vfz = nullptr;      // this wavefront's head in a.Vf (wavefront-uniform)
    uint32_t bitsA = 0, bitsB = 0;      // OR of their bit patterns
    bf16x8 xbA0, xbA1, xbB0, xbB1;      // -x of chunks a and b as GEMM-R operands (column slabs 0 and 1)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) racc[mt][v] = 0.f;
    const float* yrow = nullptr;
    const float* ytile = nullptr;      // a.y_tiled: this wavefront's tile of y (wavefront-uniform)

    auto load_y = [&]() {
        if (a.y_tiled) {         // whole 1 KB pieces: a uniform base that advances by 4 KB per tile of m, plus 0 .. 3 KB
            // (the base is made opaque: fifty-two addresses computed ahead and kept across the iterations would spill)
            const float* yp = ytile;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                asm volatile("" : "+s"(yp));
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 y4 = *(const f32x4*)at16(yp + g * 256);
#pragma unroll
                    for (int e = 0; e < 4; ++e) racc[mt][4 * g + e] = y4[e];
                }
                yp += 1024;
            }
        } else {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 y4 = *(const f32x4*)(yrow + 32 * mt + 8 * g);
#pragma unroll
                    for (int e = 0; e < 4; ++e) racc[mt][4 * g + e] = y4[e];
                }
        }
    };
    auto boundary = [&]() {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            rb[2 * mt] = cvt8<0>(racc[mt], 1.f);
            rb[2 * mt + 1] = cvt8<8>(racc[mt], 1.f);
        }
    };

    // this wavefront's share (2 FW fragments) of the packed chunk pair `pair` into ring slot `slot`: request i of it
    auto issue_pair_one = [&](auto ic, int pair, int slot, uint32_t ulane) {
        constexpr int i = decltype(ic)::value;
        (void)ulane;
        const uint4* src = (const uint4*)at16(a.PhiPack + ((long long)pair * 2 * SETF + wave * 2 * FW) * 64);
        // flat fragment F of the pair goes to F KB plus one shift per slab 1 reached (of chunk a, of chunk b)
        const int F = wave * 2 * FW + i;
        char* dst = (char*)lds + slot * PAIR + wave * 2 * FW * 1024 + (SHIFT ? SHIFT * ((F >= MT) + (F >= SETF + MT)) : 0);
        constexpr int blk = i / 4;
        if constexpr (i % 4 == 0) __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + blk * 256), (lds_ptr_t)(dst + blk * 4096), 16, 0, 0);
        else if constexpr (i % 4 == 1) __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + blk * 256), (lds_ptr_t)(dst + blk * 4096), 16, 1024, 0);
        else if constexpr (i % 4 == 2) __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + blk * 256), (lds_ptr_t)(dst + blk * 4096), 16, 2048, 0);
        else __builtin_amdgcn_global_load_lds((glb_ptr_t)(src + blk * 256), (lds_ptr_t)(dst + blk * 4096), 16, 3072, 0);
    };
    auto issue_pair_range = [&](auto self, auto lo, auto hi, int pair, int slot, uint32_t ulane) {
        constexpr int l = decltype(lo)::value, h = decltype(hi)::value;
        if constexpr (l < h && l < 2 * FW) {
            issue_pair_one(lo, pair, slot, ulane);
            self(self, std::integral_constant<int, l + 1>{}, hi, pair, slot, ulane);
        }
    };
    auto issue_pair_all = [&](int pair, int slot) {
        issue_pair_range(issue_pair_range, std::integral_constant<int, 0>{}, std::integral_constant<int, 2 * FW>{}, pair, slot, 0u);
    };
    // State: the layout of the one-chunk schedule ([row tile][chunk][4][lane] float4, 1 KB contiguous per request),
    // but the mask [row tile][chunk][lane] is one flag per lane and tile: non-zero when any of the lane's 16 values is.
    // A lane with a zero tile neither writes nor reads it (SPARSE), and a tile costs one test, not one per float4.
    // Old iterate of chunk ct into half `sub` of this wavefront's block (only the lanes the mask names, if SPARSE).
    auto issue_state = [&](int ct, int sub, uint32_t m) {
        const f32x4* src = (const f32x4*)at16(st + ct * 256);
        char* dst = (char*)lds + OFF_X + wave * 8192 + sub * 4096;
        if (!SPARSE || m != 0) {
            __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 0, 0);
            __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 1024, 0);
            __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 2048, 0);
            __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)dst, 16, 3072, 0);
        }
    };

    // Non-zero masks (SPARSE) of the old iterate: of this step's chunks a and b, of the next step's (they tell which
    // pieces of the old iterate to request) and of the step's after that, fetched two steps ahead so that the value
    // has arrived by the barrier before it is used: a mask waited for in the middle of a step would wait for
    // every request and store issued since.
    uint32_t mA = 0, mB = 0, mNA = 0, mNB = 0, mFA = 0, mFB = 0;

    // What one step is told about the steps after it: the pair staged for the next step (a valid pair even when
    // nothing follows: the request is then harmless), whether the next step reads an old iterate, and the pair whose
    // masks are fetched now for the step after next (-1: none).
    struct Next { int pair, slot; bool want_x; int pair2; };

    // x = eta(old + mu u) for a tile, old from the four float4 in xs, u from the accumulator tile un.
    // With a single wavefront on the SIMD nothing hides the latency of a dependent vector instruction (in a loop of
    // MFMAs and dependent fmas each one waits about twice its issue time), so the arithmetic is cut into stages of four
    // INDEPENDENT instructions: stage 0 reads four accumulator elements (left to the compiler, all 16 come out in one
    // burst right behind the last MFMA of the product, which stalls on it), stage 1 adds mu u to the old values (the
    // only stage that needs them), stage 2 clamps, stage 3 subtracts and collects the bit patterns in `bits` (any
    // set bit: the tile is not all +0).  Stage st of quad q is stage-group 4 q + st; the groups go behind different
    // MFMAs, in order.  The MFMA that wrote un must have left the pipe before stage 0: callers start no earlier than
    // behind the second MFMA issued after it.
    float tq[4];
    auto threshold_stage = [&](f32x16& x, int g, const u32x4 (&xs)[4], const f32x16& un, uint32_t& bits) {
        const int q = g >> 2, st = g & 3;
        if (st == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float uv;
                asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(uv) : "a"(un[4 * q + e]));
                x[4 * q + e] = uv;
            }
        } else if (st == 1) {
            const f32x4 old = __builtin_bit_cast(f32x4, xs[q]);
            float t0 = old[0] + a.mu * x[4 * q], t1 = old[1] + a.mu * x[4 * q + 1];
            float t2 = old[2] + a.mu * x[4 * q + 2], t3 = old[3] + a.mu * x[4 * q + 3];
            asm volatile("" : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3));      // keeps the arithmetic where it is written
            x[4 * q] = t0; x[4 * q + 1] = t1; x[4 * q + 2] = t2; x[4 * q + 3] = t3;
        } else if (st == 2) {
#pragma unroll
            for (int e = 0; e < 4; ++e) tq[e] = __builtin_amdgcn_fmed3f(x[4 * q + e], -a.theta, a.theta);
            asm volatile("" : "+v"(tq[0]), "+v"(tq[1]), "+v"(tq[2]), "+v"(tq[3]));
        } else {      // eta_theta(u) = u - clamp(u, -theta, theta): exact zero for |u| <= theta
            float t0 = x[4 * q] - tq[0], t1 = x[4 * q + 1] - tq[1], t2 = x[4 * q + 2] - tq[2], t3 = x[4 * q + 3] - tq[3];
            asm volatile("" : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3));
            bits |= (__builtin_bit_cast(uint32_t, t0) | __builtin_bit_cast(uint32_t, t1)) |
                    (__builtin_bit_cast(uint32_t, t2) | __builtin_bit_cast(uint32_t, t3));
            x[4 * q] = t0; x[4 * q + 1] = t1; x[4 * q + 2] = t2; x[4 * q + 3] = t3;
        }
    };
    // state (or, in the last iteration, the outputs) of chunk ct from x
    // (`half`: the state goes out in two parts, float4 0-1 and 2-3 with the flag, so that neither holds up the
    // MFMA it is issued behind for long; the outputs of the last iteration go out in one part, half 0)
    auto write_out = [&](auto is_last, int ct, const f32x16& x, uint32_t bits, int half) {
        constexpr bool LAST = decltype(is_last)::value;
        if constexpr (!LAST) {
            if (!SPARSE || bits != 0) {      // (a -0 sets a bit and only costs a store)
                f32x4* dst = (f32x4*)at16(st + ct * 256);
#pragma unroll
                for (int g = 2 * half; g < 2 * half + 2; ++g) dst[g * 64] = f32x4{x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
            }
            if constexpr (SPARSE) { if (half == 1) (mk + ct * 64)[lane] = (uint8_t)(bits != 0); }
        } else if (half == 0 && row_ok) {
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
    };

    auto make_xb = [&](const f32x16& x, bf16x8& b0, bf16x8& b1) {
        b0 = cvt8<0>(x, -1.f);
        b1 = cvt8<8>(x, -1.f);
    };

    // One step: the chunk pair (ca, ca + 1) in ring slot `slot`.  LAST: final iteration (no residual update,
    // outputs instead of state).  DO_Y: first step of an iteration (racc restarts from y).
    //
    // The four products are ONE pipeline of 4 * NG items of up to G fragments, across the phase boundaries too, so
    // the LDS latency is exposed once per step.  A wavefront issues in order and an MFMA is accepted only when the
    // one before it has left the pipe, so whatever is issued after the last MFMA of an item beyond the eight or so
    // instructions that fit under it delays the next MFMA.  Everything else a step has to do is therefore cut into
    // slots, one behind EACH MFMA: the LDS read of one fragment of the item LA items ahead, a staging request, one
    // or two elements of the threshold arithmetic; scheduling barriers keep the compiler from regrouping them.
    auto step = [&](auto is_last, auto do_y, int ca, int slot, bool first, const Next& nx) {
        constexpr bool LAST = decltype(is_last)::value, DO_Y = decltype(do_y)::value;
        constexpr int NP = LAST ? 2 : 4;               // phases with MFMAs
        constexpr int NI = NP * NG;                    // items
        constexpr int PS = NG * G;                     // slots of a phase
        // Threshold arithmetic of a phase: from slot LEAD on (the slots before it hold what opens the phase) and
        // done before the old-iterate registers are reloaded for the next phase, in slot 0 of item NG - LA.
        static_assert(NG > LA && MT >= 3, "group count");
        constexpr int LEAD1 = 1, LEAD2 = 2, TEND = (NG - LA) * G;
        static_assert(TEND > LEAD2, "no slot for the threshold arithmetic");
        // stage-group g of the threshold arithmetic goes behind slot LEAD + g (TEND - LEAD) / 16
        constexpr int RP = CSAT_FUSED2_REQUESTS_IN_PHASE < NP ? CSAT_FUSED2_REQUESTS_IN_PHASE : NP;
        const uint32_t baseU = tr8 + slot * PAIR, baseR = nat16 + slot * PAIR;
        const int cb = ca + 1;
        // U of a and of b each in one accumulator chain of its own (a second chain per product measured slower: its
        // sum costs more than the dependent MFMAs; separate accumulators let U_a be read while U_b accumulates)
        f32x16 unA, unB;
        u32x4 xs[4];
        u32x4 fr[NB][G];
        u32x2 ft[NB][G][2];
        // old iterate of a (sub 0) or b (sub 1): from this wavefront's block, or zeros for a lane that has none
        auto read_xs = [&](int sub) {
            const uint32_t m = sub ? mB : mA;
            const uint32_t b = (SPARSE ? m != 0 : !first) ? xblock + sub * 4096 : zblock;
            lds_read16<0>(xs[0], b);
            lds_read16<1024>(xs[1], b);
            lds_read16<2048>(xs[2], b);
            lds_read16<3072>(xs[3], b);
        };
        auto pin_xs = [&]() { lds_pin(xs[0]); lds_pin(xs[1]); lds_pin(xs[2]); lds_pin(xs[3]); };
        // item = (phase p, group k): phases 0, 1 are GEMM-U of a, b (transposed fragments), 2, 3 GEMM-R of a, b
        auto fetch = [&](auto pc, auto kc, auto ic) {
            constexpr int p = decltype(pc)::value, k = decltype(kc)::value, i = decltype(ic)::value, f = k * G + i;
            constexpr int par = (p * NG + k) % NB;
            if constexpr (f < NF) {
                if constexpr (p < 2) {      // K slab f of m: row tile f/2, rows 16*(f%2) .. +15
                    lds_read8_tr<(p & 1) * HALF + (f >> 1) * 1024 + (f & 1) * 256>(ft[par][i][0], baseU);
                    lds_read8_tr<(p & 1) * HALF + (f >> 1) * 1024 + (f & 1) * 256 + 128>(ft[par][i][1], baseU);
                } else {
                    lds_read16<(p & 1) * HALF + f * 1024 + (f >= MT ? SHIFT : 0)>(fr[par][i], baseR);
                }
            }
        };
        // all reads of item q at once (the first LA items of a step, which have no MFMAs to go behind)
        auto fetch_item = [&](auto self, auto pc, auto kc, auto ic) {
            constexpr int i = decltype(ic)::value;
            if constexpr (i < G) {
                fetch(pc, kc, ic);
                self(self, pc, kc, std::integral_constant<int, i + 1>{});
            }
        };
        // what goes behind MFMA i of item (p, k)
        auto slot_work = [&](auto pc, auto kc, auto ic) {
            constexpr int p = decltype(pc)::value, k = decltype(kc)::value, i = decltype(ic)::value;
            constexpr int q = p * NG + k, j = k * G + i;
            // fragment i of the item LA items ahead, preceded by the old-iterate reads when that item opens phase 1 or 2
            constexpr int q2 = q + LA;
            if constexpr (q2 < NI) {
                constexpr int p2 = q2 / NG, k2 = q2 % NG;
                if constexpr (i == 0 && k2 == 0 && (p2 == 1 || p2 == 2)) read_xs(p2 - 1);
                fetch(std::integral_constant<int, p2>{}, std::integral_constant<int, k2>{}, ic);
            }
            // staging requests of the next pair, spread evenly over the slots of the first RP phases
            if constexpr (p < RP) {
                constexpr int TOT = RP * PS, jj = p * PS + j;
                issue_pair_range(issue_pair_range, std::integral_constant<int, jj * 2 * FW / TOT>{},
                                 std::integral_constant<int, (jj + 1) * 2 * FW / TOT>{}, nx.pair, nx.slot, 0u);
            }
            if constexpr (p == 1) {              // threshold of a; its half of the old-iterate block refilled
                // (the old iterate of a is in registers since the wait of item (1, 0))
                if constexpr (j == 0) {
                    if (nx.want_x) issue_state(2 * nx.pair, 0, mNA);
                    bitsA = 0;
                }
#pragma unroll
                for (int g = 0; g < 16; ++g)
                    if (LEAD1 + g * (TEND - LEAD1) / 16 == j) threshold_stage(xA, g, xs, unA, bitsA);
                if constexpr (j == PS - 1 && !LAST) make_xb(xA, xbA0, xbA1);
            } else if constexpr (p == 2) {       // a written out, b's half of the block refilled; threshold of b
                if constexpr (j == 0) {
                    write_out(is_last, ca, xA, bitsA, 0);
                    bitsB = 0;
                }
                if constexpr (j == 1) {
                    write_out(is_last, ca, xA, bitsA, 1);
                    if (nx.want_x) issue_state(2 * nx.pair + 1, 1, mNB);
                }
#pragma unroll
                for (int g = 0; g < 16; ++g)
                    if (LEAD2 + g * (TEND - LEAD2) / 16 == j) threshold_stage(xB, g, xs, unB, bitsB);
                if constexpr (j == PS - 1) make_xb(xB, xbB0, xbB1);
            } else if constexpr (p == 3) {       // b written out
                if constexpr (j == 0) write_out(is_last, cb, xB, bitsB, 0);
                if constexpr (j == 1) write_out(is_last, cb, xB, bitsB, 1);
            }
        };
        // MFMA i of item (p, k) and its slot, then the next one
        auto mfma_slot = [&](auto self, auto pc, auto kc, auto ic) {
            constexpr int p = decltype(pc)::value, k = decltype(kc)::value, i = decltype(ic)::value;
            constexpr int par = (p * NG + k) % NB, f = k * G + i;
            if constexpr (i < G) {
                if constexpr (f < NF) {
                    if constexpr (p < 2) {
                        const u32x4 fa = __builtin_shufflevector(ft[par][i][0], ft[par][i][1], 0, 1, 2, 3);
                        if constexpr (p == 0) unA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa), rb[f], unA, 0, 0, 0);
                        else unB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa), rb[f], unB, 0, 0, 0);
                    } else {      // fragment f: column slab f / MT, accumulator tile f % MT
                        racc[f % MT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, fr[par][i]), p == 2 ? ((f >= MT) ? xbA1 : xbA0) : ((f >= MT) ? xbB1 : xbB0),
                            racc[f % MT], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                slot_work(pc, kc, ic);
                __builtin_amdgcn_sched_barrier(0);
                self(self, pc, kc, std::integral_constant<int, i + 1>{});
            }
        };
        // item q = p * NG + k.  On entry the reads of items q .. q + LA - 1 are in flight, in that order; those of
        // item q + LA go out behind this item's MFMAs.
        auto item = [&](auto self, auto pc, auto kc) {
            constexpr int p = decltype(pc)::value, k = decltype(kc)::value;
            constexpr int q = p * NG + k;
            constexpr int par = q % NB;
            lds_wait_n<fused2_ahead_loads(q, LA - 1, G, NF, NG, NP)>();
#if CSAT_FUSED2_PIN
#pragma unroll
            for (int i = 0; i < G; ++i) {
                if (k * G + i < NF) {
                    if constexpr (p < 2) lds_pin(ft[par][i][0], ft[par][i][1]);
                    else lds_pin(fr[par][i]);
                }
            }
            if constexpr (k == 0 && (p == 1 || p == 2)) pin_xs();      // (read before this item's fragments: landed too)
#endif
            // (the consumers of the registers just waited for stay behind the wait: nothing crosses the barrier below)
            __builtin_amdgcn_sched_barrier(0);
            mfma_slot(mfma_slot, pc, kc, std::integral_constant<int, 0>{});
            if constexpr (q + 1 < NI) self(self, std::integral_constant<int, (q + 1) / NG>{}, std::integral_constant<int, (q + 1) % NG>{});
        };

        if constexpr (SPARSE) {      // masks of the step after next (see the declaration of the masks)
            mFA = 0;
            mFB = 0;
            if (nx.pair2 >= 0) {
                const uint32_t ul = lane_off();
                mFA = mk[(2 * nx.pair2) * 64 + ul];
                mFB = mk[(2 * nx.pair2 + 1) * 64 + ul];
            }
        }
        if (!CSAT_FUSED2_REQUESTS_IN_PHASE) issue_pair_all(nx.pair, nx.slot);
        if constexpr (DO_Y) load_y();
#pragma unroll
        for (int v = 0; v < 16; ++v) { unA[v] = 0.f; unB[v] = 0.f; }
        static_assert(LA >= 1 && LA <= 4 && LA < NG, "lookahead");       // (the first LA items lie in phase 0)
        fetch_item(fetch_item, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        if constexpr (LA > 1) fetch_item(fetch_item, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{});
        if constexpr (LA > 2) fetch_item(fetch_item, std::integral_constant<int, 0>{}, std::integral_constant<int, 2>{}, std::integral_constant<int, 0>{});
        if constexpr (LA > 3) fetch_item(fetch_item, std::integral_constant<int, 0>{}, std::integral_constant<int, 3>{}, std::integral_constant<int, 0>{});
        item(item, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        // the synthesis in the last iteration: the fragments of V for this step's two chunks, requested here, used at
        // the end of the step
        u32x4 vf[8];
        if constexpr (LAST) {
            if (vfz) {
#pragma unroll
                for (int i = 0; i < 8; ++i) vf[i] = *(const u32x4*)at16(vfz + (ca * 4 + i) * 64);   // chunks ca, ca + 1
            }
        }
        auto synthesize = [&](const f32x16& x, int sub) {
            const bf16x8 b0 = cvt8<0>(x, 1.f), b1 = cvt8<8>(x, 1.f);
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                cacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[4 * sub + dt]), b0, cacc[dt], 0, 0, 0);
                cacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[4 * sub + 2 + dt]), b1, cacc[dt], 0, 0, 0);
            }
        };
        if constexpr (LAST) {        // no residual update: a is written out, b thresholded on its own
            write_out(is_last, ca, xA, bitsA, 0);
            if (vfz) synthesize(xA, 0);
            read_xs(1);
            lds_wait_n<0>();
            pin_xs();
            asm volatile("s_nop 15");         // (the last MFMA into unB is long done; the compiler cannot see the reads below)
#pragma unroll
            for (int g = 0; g < 16; ++g) threshold_stage(xB, g, xs, unB, bitsB);
            write_out(is_last, cb, xB, bitsB, 0);
            if (vfz) synthesize(xB, 1);
            if (nx.want_x) issue_state(2 * nx.pair + 1, 1, mNB);
        }
        if constexpr (SPARSE) { mA = mNA; mB = mNB; mNA = mFA; mNB = mFB; }
    };

    using T_ = std::true_type;
    using F_ = std::false_type;
    auto sync = [&]() {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };

    // Work distribution.  The work of a launch is groups x iterations group-iterations, and the iterations of a group
    // run one after the other; a persistent grid of one workgroup per CU finishes soonest when every workgroup gets the
    // same number of group-iterations.  a.tape > 0 (the default): the group-iterations, laid out group by group, are
    // cut into a.tape equal shares (a.tape <= groups, so a share is at least one group's iterations and holds the end
    // of one group, whole groups, and the beginning of one more).  A workgroup takes a share from an atomic counter
    // and runs, in this order: the BEGINNING piece of the share's last group (iterations 0 .. c - 1: nothing to wait
    // for), the whole groups, and last the END piece of the share's first group (iterations c' .. T - 1), whose
    // beginning the holder of the share before ran first thing.  So every group is cut at most once, a hand-over is
    // waited for a whole share's time after it was produced, and the launch takes ceil(groups x T / shares)
    // iterations: short_video (600 groups, 256 CUs, T = 20) 47 iteration times against 50 for two equal segments per
    // group and 60 for whole groups.  (Shares weighted by cost - a group's last iteration has no residual
    // update - measured no better.)  Shares are handed out in order, so the producer of a hand-over has always
    // started when its consumer waits (no deadlock if the workgroups are not all resident); the wait is bounded as
    // before.  a.tape == 0: as in ista_fused_kernel (units of one group over one of a.segs equal segments of the
    // iterations, in segment-major order).
    // sync[2 + group] counts the iterations of the group that have been published.
    __shared__ int s_unit, s_err;
    const int total = a.tape > 0 ? a.tape : a.groups * a.segs;
    bool failed = false;
    for (;;) {
        if (threadIdx.x == 0) {
            s_unit = atomicAdd(a.sync, 1);
            s_err = 0;
        }
        __syncthreads();
        const int unit = __builtin_amdgcn_readfirstlane(s_unit);      // (uniform: the addresses below stay in scalar registers)
        if (unit >= total) break;
        // pieces of this unit: (group, first iteration, one past the last) in execution order
        int np = 1, g_first = 0, g_last = 0, lo_first = 0, hi_last = a.iters;
        bool end_first = false, start_last = false;
        if (a.tape > 0) {
            const long long tot = (long long)a.groups * a.iters;
            const long long b0 = tot * unit / a.tape, b1 = tot * (unit + 1) / a.tape;
            g_first = (int)(b0 / a.iters);
            g_last = (int)((b1 - 1) / a.iters);
            lo_first = (int)(b0 - (long long)g_first * a.iters);
            hi_last = (int)(b1 - (long long)g_last * a.iters);
            np = g_last - g_first + 1;
            end_first = np > 1 && hi_last < a.iters;       // the last group's beginning piece goes first
            start_last = np > 1 && lo_first > 0;           // the first group's end piece goes last
        }
        for (int pi = 0; pi < np; ++pi) {
        int grp, t0, t1;
        if (a.tape > 0) {
            // position pi -> group: [last group if end_first] [groups in between, ascending] [first group if start_last]
            int gi;
            if (end_first && pi == 0) gi = g_last;
            else if (start_last && pi == np - 1) gi = g_first;
            else gi = g_first + pi - (end_first ? 1 : 0) + (start_last ? 1 : 0);
            grp = gi;
            t0 = gi == g_first ? lo_first : 0;
            t1 = gi == g_last ? hi_last : a.iters;
        } else {
            const int seg = unit / a.groups;
            grp = unit - seg * a.groups;
            t0 = (int)((long long)seg * a.iters / a.segs);
            t1 = (int)((long long)(seg + 1) * a.iters / a.segs);
        }
        rt = (long long)grp * 4 + wave;
        row = rt * 32 + (lane & 31);
        row_ok = row < a.rows;
        st = (f32x4*)a.state + rt * nct * 256;
        mk = a.mask + rt * nct * 64;
        yrow = a.Y + (row_ok ? row : a.rows - 1) * a.ldy + 4 * lh;
        if (a.y_tiled) {           // (tiles beyond the last repeat it; nothing of theirs is stored)
            const long long tile = rt * 32 < a.rows ? rt : a.rows / 32 - 1;
            ytile = a.Y + tile * (long long)a.ldy * 32;
        }
        if (a.Vf) {     // (rows beyond the last repeat the last head; nothing of theirs is stored)
            const long long r0 = rt * 32 < a.rows ? rt * 32 : a.rows - 1;
            vfz = a.Vf + (r0 / a.n_q) * ((long long)nct * 4 * 64);
        }
        if (t0 > 0) {
            if (threadIdx.x == 0) {
                long long spins = 0;
                for (;;) {
                    if (__hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { s_err = 1; break; }
                    if (__hip_atomic_load(a.sync + 2 + grp, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) >= t0) break;
                    if (++spins > a.spin_limit) {
                        __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        s_err = 1;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(64);
                }
            }
            __syncthreads();
            if (s_err) { failed = true; break; }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        if (t0 == 0) {             // x = 0: r = y
            load_y();
            boundary();
        } else {                   // residual operands left by the previous segment
            const uint4* hp = a.hand + ((long long)rt * 2 * MT) * 64 + lane_off();
#pragma unroll
            for (int f = 0; f < 2 * MT; ++f) rb[f] = __builtin_bit_cast(bf16x8, hp[f * 64]);
        }
        // the first pair and, from the second iteration on, its old iterate and the masks of the first two steps
        int slot = 0;
        issue_pair_all(0, 0);
        mA = mB = mNA = mNB = 0;
        if (t0 > 0) {
            if constexpr (SPARSE) {
                const uint32_t ul = lane_off();
                mA = mk[ul];
                mB = mk[64 + ul];
                mNA = mk[128 + ul];
                mNB = mk[192 + ul];
            }
            issue_state(0, 0, mA);
            issue_state(1, 1, mB);
        }
        const int tn = t1 < a.iters ? t1 : a.iters - 1;       // normal iterations of this unit: [t0, tn)
        // S >= 3 (the host sends shorter rows to the one-chunk schedule): the pair whose masks step s fetches was
        // written at least one step before, also across the iteration boundary.
        auto next_of = [&](int s, bool first, bool more) {
            const bool wrap = s + 1 == S;
            const int s2 = s + 2;
            const int pair2 = s2 < S ? (first ? -1 : s2) : (more ? s2 - S : -1);
            return Next{wrap ? 0 : s + 1, slot ^ 1, wrap ? more : !first, pair2};
        };
        for (int t = t0; t < tn; ++t) {
            const bool first = t == 0;
            const bool more = t + 1 < t1;                      // another iteration of this unit follows
            {
                sync();
                step(F_{}, T_{}, 0, slot, first, next_of(0, first, more));
                slot ^= 1;
            }
            for (int s = 1; s < S; ++s) {
                sync();
                step(F_{}, F_{}, 2 * s, slot, first, next_of(s, first, more));
                slot ^= 1;
            }
            boundary();            // residual operands of the next iteration
        }
        if (t1 == a.iters) {   // last iteration: no residual update, outputs instead of state
            const bool first = a.iters == 1;
#pragma unroll
            for (int v = 0; v < 16; ++v) { cacc[0][v] = 0.f; cacc[1][v] = 0.f; }
            for (int s = 0; s < S; ++s) {
                sync();
                step(T_{}, F_{}, 2 * s, slot, first, next_of(s, first, false));
                slot ^= 1;
            }
            if (a.Vf && row_ok) {      // C^T tile: lane (row, h), register v <-> d = 32 dt + 8 (v / 4) + 4 h + v % 4
                bf16_t* crow = a.C + row * 64 + 4 * lh;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        *(uint2*)(crow + 32 * dt + 8 * g) = uint2{f2bf_pk(cacc[dt][4 * g], cacc[dt][4 * g + 1]),
                                                                  f2bf_pk(cacc[dt][4 * g + 2], cacc[dt][4 * g + 3])};
            }
        } else {               // hand the residual operands to the next segment
            uint4* hp = a.hand + ((long long)rt * 2 * MT) * 64 + lane_off();
#pragma unroll
            for (int f = 0; f < 2 * MT; ++f) hp[f * 64] = __builtin_bit_cast(uint4, rb[f]);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __syncthreads();
            if (threadIdx.x == 0) __hip_atomic_store(a.sync + 2 + grp, t1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        // nothing of this piece may still be in flight towards LDS when the next one starts staging
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        }
        if (failed) break;
    }
}

}  // namespace csat
