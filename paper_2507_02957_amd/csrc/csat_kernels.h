// Device kernels of the CSAT forward pass for gfx950 (CDNA4, 64-wide wavefronts, MFMA).
//
// One tiled "NT" GEMM core  C[M,N] = sum_k A[M,k] * Bt[N,k]  (both operands K-contiguous) feeds
// every dense contraction of the path; what differs between stages is the epilogue functor
// that consumes the fp32 accumulators.  bf16 operands use the 32x32x16 MFMA (fp32 accumulate),
// float operands the 32x32x2 MFMA.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace csat {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

typedef uint16_t bf16_t;   // storage type of a bfloat16 element

typedef __bf16 hwbf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// two floats -> packed bf16 (a in the low half), round to nearest even: one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t f2bf_pk(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, hwbf16x2));
}
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* glb_ptr_t;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// LDS fragment reads are issued as inline assembly with their own wait counts: the compiler
// cannot tell that the direct global->LDS loads of the *next* chunk write a different stage than
// the one being read, and would otherwise wait for them before every LDS read.
template <int OFF>
__device__ __forceinline__ void lds_read16(u32x4& dst, uint32_t byte_addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(byte_addr), "n"(OFF));
}
// Waits until at most N LDS reads are outstanding (they return in order); naming the fragments
// as in/out operands keeps their consumers behind the wait.
template <int N>
__device__ __forceinline__ void lds_wait(u32x4& a, u32x4& b, u32x4& c, u32x4& d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int per_chunk = 4;   // elements per 16-byte chunk
    __device__ static __forceinline__ float load(const float* p) { return *p; }
    __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int per_chunk = 8;
    __device__ static __forceinline__ float load(const bf16_t* p) { return bf2f(*p); }
    __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f2bf(v); }
};

// ----------------------------------------------------------------------------------------
// GEMM core.  256 threads = 4 wavefronts arranged WM x WN; each wavefront owns TM x TN
// MFMA tiles of 32x32.  The K loop advances 128 bytes of K per operand row per step
// (64 bf16 or 32 float): global -> registers (prefetch of the next step) -> LDS -> MFMA.
// LDS rows are padded by one 16-byte chunk so the 16-byte fragment reads of 32 consecutive
// rows fall in distinct banks.
//
// Operand contract: row pointers are 16-byte aligned (ld multiple of the chunk size), and
// elements in columns [K, roundup(K, chunk)) are zero.  Rows >= M (or >= N for Bt) and
// chunks at k >= K are zero-filled by the loader, never read.
// ----------------------------------------------------------------------------------------
constexpr int kRowChunks = 8;               // 16-byte chunks of K per tile row (128 bytes)
constexpr int kLdsRowChunks = kRowChunks + 1;

struct GemmArgs {
    const void* A;  long long lda;  long long strideA;   // strides in elements, per batch index z
    const void* Bt; long long ldb;  long long strideB;
    int M, N, K;
    int a_kwrap;   // > 0: A has only this many 16-byte chunks of K per row and is re-read cyclically
                   // (A' = [A | A | ...]); used to contract Q against a [hi | lo] split operand
    int raster = 0;   // large-tile kernel only: how the 1-D grid walks the tiles (see csat_gemm_big.h)
};
constexpr int kRasterStreamA = 64;   // flag in GemmArgs::raster: the A rows are loaded with the non-temporal hint

template <typename T>
__device__ __forceinline__ void mfma_group(const uint4& a, const uint4& b, f32x16& acc);

template <>
__device__ __forceinline__ void mfma_group<bf16_t>(const uint4& a, const uint4& b, f32x16& acc) {
    bf16x8 av = __builtin_bit_cast(bf16x8, a);
    bf16x8 bv = __builtin_bit_cast(bf16x8, b);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mfma_group<float>(const uint4& a, const uint4& b, f32x16& acc) {
    f32x4 av = __builtin_bit_cast(f32x4, a);
    f32x4 bv = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s], bv[s], acc, 0, 0, 0);
}

template <typename T, int BM, int BN, int WM, int WN, typename Epi>
__global__ __launch_bounds__(256) void gemm_nt_kernel(GemmArgs g, Epi epi) {
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    static_assert(TM >= 1 && TN >= 1, "tile too small for the wavefront grid");
    constexpr int EPC = Elem<T>::per_chunk;
    constexpr int A_CHUNKS = BM * kRowChunks / 256, B_CHUNKS = BN * kRowChunks / 256;

    __shared__ uint4 sA[BM * kLdsRowChunks];
    __shared__ uint4 sB[BN * kLdsRowChunks];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lh = lane >> 5;
    const int z = blockIdx.z;
    const long long row0 = (long long)blockIdx.x * BM, col0 = (long long)blockIdx.y * BN;

    const T* A = (const T*)g.A + (long long)z * g.strideA;
    const T* Bt = (const T*)g.Bt + (long long)z * g.strideB;
    const int kchunks = (g.K + EPC - 1) / EPC;           // valid 16-byte chunks per row
    const int ksteps = (kchunks + kRowChunks - 1) / kRowChunks;

    uint4 ra[A_CHUNKS], rb[B_CHUNKS];
    auto load_global = [&](int ks) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            int id = tid + 256 * i, r = id / kRowChunks, c = id % kRowChunks;
            int kc = ks * kRowChunks + c;
            long long gr = row0 + r;
            int kca = g.a_kwrap > 0 ? kc % g.a_kwrap : kc;
            ra[i] = (gr < g.M && kc < kchunks)
                        ? *(const uint4*)(A + gr * g.lda + (long long)kca * EPC) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            int id = tid + 256 * i, r = id / kRowChunks, c = id % kRowChunks;
            int kc = ks * kRowChunks + c;
            long long gr = col0 + r;
            rb[i] = (gr < g.N && kc < kchunks)
                        ? *(const uint4*)(Bt + gr * g.ldb + (long long)kc * EPC) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            int id = tid + 256 * i;
            sA[(id / kRowChunks) * kLdsRowChunks + (id % kRowChunks)] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            int id = tid + 256 * i;
            sB[(id / kRowChunks) * kLdsRowChunks + (id % kRowChunks)] = rb[i];
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    load_global(0);
    store_lds();
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        if (ks + 1 < ksteps) load_global(ks + 1);
#pragma unroll
        for (int gk = 0; gk < kRowChunks / 2; ++gk) {
            uint4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = sA[((wm * TM + i) * 32 + li) * kLdsRowChunks + 2 * gk + lh];
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = sB[((wn * TN + j) * 32 + li) * kLdsRowChunks + 2 * gk + lh];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mfma_group<T>(fa[i], fb[j], acc[i][j]);
        }
        __syncthreads();
        if (ks + 1 < ksteps) {
            store_lds();
            __syncthreads();
        }
    }

    // accumulator layout of the 32x32 MFMA: lane (li, lh), register v holds
    // row 8*(v/4) + 4*lh + (v%4), column li of the tile
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            long long c = col0 + (wn * TN + j) * 32 + li;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                long long r = row0 + (wm * TM + i) * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
                epi(z, r, c, acc[i][j][v]);
            }
        }
}

// ----------------------------------------------------------------------------------------
// Epilogues.  Each sees (batch z, row r, column c, fp32 accumulator) and does its own bounds
// checks: the tile grid may overhang M and N.
// ----------------------------------------------------------------------------------------

// out[z][r][c] = alpha * acc, optionally also outT[z][c][r] (a transposed copy whose pad
// columns [M, ldT) were zeroed beforehand).
template <typename TO>
struct EpiStore {
    TO* out; long long ld, stride;
    TO* outT; long long ldT, strideT;
    float alpha; int M, N;
    __device__ __forceinline__ void operator()(int z, long long r, long long c, float v) const {
        if (r >= M || c >= N) return;
        v *= alpha;
        if (out) Elem<TO>::store(out + z * stride + r * ld + c, v);
        if (outT) Elem<TO>::store(outT + z * strideT + c * ldT + r, v);
    }
};

// C[r][c] = v, written with the non-temporal hint: for a large result that is read once by the next kernel and
// should not push that kernel's other inputs out of the caches (matching pursuit's correlations).
struct EpiStoreStream {
    float* out; long long ld;
    int M, N;
    __device__ __forceinline__ void operator()(int, long long r, long long c, float v) const {
        if (r < M && c < N) __builtin_nontemporal_store(v, out + r * ld + c);
    }
};

// Compressed keys for the score contraction: next to the element-type copy Kc[z][r][c], writes
// the bf16 pair (hi, lo) with hi = bf16(v), lo = bf16(v - hi) as KcHL[z][r][0..N) | [N..2N), so
// that scores against [Q | Q] see K~ to ~16 mantissa bits (the decoder amplifies score error).
struct EpiMeasureSplit {
    bf16_t* Kc; bf16_t* KcHL; int M, N;
    __device__ __forceinline__ void operator()(int z, long long r, long long c, float v) const {
        if (r >= M || c >= N) return;
        bf16_t hi = f2bf(v);
        Kc[((long long)z * M + r) * N + c] = hi;
        long long o = ((long long)z * M + r) * 2 * N + c;
        KcHL[o] = hi;
        KcHL[o + N] = f2bf(v - bf2f(hi));
    }
};

// Output of the compressed block for the column-wise decode: next to the element-type copy
// out[z][r][c] (optional) writes the transposed value as a bf16 pair, outT[z][c][r] = hi and
// outT[z][c][ldT/2 + r] = lo (rows of outT have ldT = 2 * padded n elements, pads zeroed beforehand),
// so that the measurement Phi Z sees Z to ~16 mantissa bits.
struct EpiStoreSplitT {
    bf16_t* out; long long ld, stride;
    bf16_t* outT; long long ldT, strideT;
    int M, N;
    __device__ __forceinline__ void operator()(int z, long long r, long long c, float v) const {
        if (r >= M || c >= N) return;
        const bf16_t hi = f2bf(v);
        if (out) out[z * stride + r * ld + c] = hi;
        bf16_t* t = outT + z * strideT + c * ldT + r;
        t[0] = hi;
        t[ldT / 2] = f2bf(v - bf2f(hi));
    }
};

// ISTA residual: R[r][c] = Y[r][c] - acc  (acc = (Phi x)[c]); pad columns [N, ldR) get zero.
template <typename TO>
struct EpiResidual {
    const float* Y; long long ldY;
    TO* R; long long ldR;
    long long M; int N;
    __device__ __forceinline__ void operator()(int, long long r, long long c, float v) const {
        if (r >= M || c >= ldR) return;
        float out = (c < N) ? Y[r * ldY + c] - v : 0.f;
        Elem<TO>::store(R + r * ldR + c, out);
    }
};

// ISTA update: u = x + mu * acc (acc = (Phi^T r)[c]); x <- sign(u) max(|u| - theta, 0).
// Writes the fp32 state Xs (ld = ldS, pad columns zero), an optional bf16 operand copy Xb
// (same ld) and an optional caller-layout copy Xo (ld = N).  `first` marks x^0 = 0: the old
// state is not read.
struct EpiIstaUpdate {
    float* Xs; bf16_t* Xb; long long ldS;
    float* Xo;
    float mu, theta;
    long long M; int N; int first;
    __device__ __forceinline__ void operator()(int, long long r, long long c, float v) const {
        if (r >= M || c >= ldS) return;
        float x = 0.f;
        if (c < N) {
            float u = mu * v;
            if (!first) u += Xs[r * ldS + c];
            float a = fabsf(u) - theta;
            x = (a > 0.f) ? copysignf(a, u) : 0.f;
            if (Xo) Xo[r * (long long)N + c] = x;
        }
        Xs[r * ldS + c] = x;
        if (Xb) Xb[r * ldS + c] = f2bf(x);
    }
};

// One layer of the unrolled decoder alpha <- eta_theta(S alpha + B y), with S applied as I + D:
// u = x_old + acc + W  (acc = (D x)[c], W = (B y)[c]), x <- eta_theta(u).  The fp32 iterate is read
// from Xold and written to Xnew (same leading dimension ldS, pad columns zero; the two may be the same
// buffer when the GEMM's operand is a separate bf16 copy), Xb is the bf16 operand copy for the next
// layer, Xo an optional caller-layout copy (ld = N).
struct EpiListaUpdate {
    const float* Xold; float* Xnew; long long ldS;
    const float* W;
    bf16_t* Xb;
    float* Xo;
    float theta;
    long long M; int N;
    __device__ __forceinline__ void operator()(int, long long r, long long c, float v) const {
        if (r >= M || c >= ldS) return;
        float x = 0.f;
        if (c < N) {
            const float u = Xold[r * ldS + c] + v + W[r * ldS + c];
            x = u - __builtin_amdgcn_fmed3f(u, -theta, theta);
            if (Xo) Xo[r * (long long)N + c] = x;
        }
        Xnew[r * ldS + c] = x;
        if (Xb) Xb[r * ldS + c] = f2bf(x);
    }
};

// Tile-level epilogues of the large-tile kernel.  A wavefront owns 64 rows x 128 columns as 2 x 4
// MFMA tiles (lane (li, lh), accumulator register v <-> row 8*(v/4) + 4*lh + (v%4), column li) and
// calls, in this order:
//   Pre begin(r0w, c0w, lane)                      before the main loop (early loads)
//   half(i, r0, c0w, lane, acc[4], stage, pre)     i = 0, 1: rows r0 .. r0+31 of the block
//     (or, for an epilogue with kWhole, one call whole(r0w, c0w, lane, acc[2][4], stage, pre) instead)
//   flush(r0w, c0w, lane, stage)                   after both halves
// `stage` is kStageBytes of LDS private to the wavefront, used to turn accumulator order into
// row-contiguous 16-byte accesses.

constexpr uint32_t kBufferFlags = 0x00027000;      // raw 32-bit buffer descriptor word 3 (gfx9 family)
// Cache policy of the accesses to the fp32 iterate (buffer instruction aux bit 1 = nt): it is touched once per
// iteration and is larger than any cache, so it must not evict what the next kernel reads (operands in L2,
// the bf16 copy of the iterate in the Infinity Cache).  Update GEMM -10 %, residual GEMM up to -25 % measured.
constexpr int kStreamAux = 2;
constexpr int kOutOfRange = 0x7fffffff;            // byte offset beyond any descriptor: loads give 0, stores are dropped

// r = y - Phi x for the large-tile kernel.  Y rows must be 16-byte aligned (ldY % 4 == 0).
struct EpiResidualTiled {
    static constexpr bool kTile = true;
    static constexpr int kPitch = 528;               // 128 floats + 16 bytes
    static constexpr int kStageBytes = 32 * kPitch;
    struct Pre {};
    const float* Y; long long ldY;
    bf16_t* R; long long ldR;
    long long M; int N;
    __device__ __forceinline__ Pre begin(long long, long long, int) const { return {}; }
    __device__ __forceinline__ void half(int, long long r0, long long c0w, int lane, const f32x16 (&acc)[4], char* stage,
                                         const Pre&) const {
        const int li = lane & 31, lh = lane >> 5;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                *(float*)(stage + (8 * (v / 4) + 4 * lh + (v % 4)) * kPitch + (j * 32 + li) * 4) = acc[j][v];
        // 16 bytes (4 columns) per lane: one instruction covers 2 rows x 512 bytes of the stage
        const long long c = c0w + li * 4;
        f32x4 y[16];
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const long long r = r0 + p * 2 + lh;
            y[p] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (r < M && c < N) y[p] = *(const f32x4*)(Y + r * ldY + c);     // pads of Y rows are zero or beyond N
        }
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const long long r = r0 + p * 2 + lh;
            const f32x4 a = *(const f32x4*)(stage + (p * 2 + lh) * kPitch + li * 16);
            if (r < M && c < ldR) {
                uint16_t o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (c + e < N) ? f2bf(y[p][e] - a[e]) : (uint16_t)0;
                *(uint2*)(R + r * ldR + c) = uint2{(uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16)};
            }
        }
    }
    __device__ __forceinline__ void flush(long long, long long, int, const char*) const {}
};

// The ISTA update for the large-tile kernel.  The fp32 state is kept in accumulator order
// ([row tile][column tile][4][lane] float4), so that a lane reads and writes its 16 values of a tile
// as four 16-byte accesses and a wavefront moves 1 KB per instruction.  The iterate is sparse: a
// per-lane mask byte per tile says which of the four float4 are non-zero, and only those are read
// and written.  The accesses go through a buffer descriptor over the 4 tiles of a half, an absent
// float4 being an out-of-range offset, so the 16 loads of a half are issued back to back without
// branches; the mask bytes are fetched before the main loop.  The bf16 operand copy is staged in
// LDS and written row-wise by flush().
struct EpiIstaUpdateTiled {
    static constexpr bool kTile = true;
    static constexpr int kPitch = 272;               // 128 bf16 + 16 bytes
    static constexpr int kStageBytes = 64 * kPitch;
    struct Pre { uint32_t have[2]; };                // byte j of have[i]: mask of tile (i, j)
    f32x4* Xs; long long tiles_n;      // column tiles per row tile (ldS / 32)
    uint8_t* Mask;                     // [row tile][column tile][lane]: bit g = float4 g of that lane is non-zero
    bf16_t* Xb; long long ldS;
    float* Xo;
    float mu, theta;
    long long M; int N; int first;
    __device__ __forceinline__ int live_tiles(long long r0, long long c0w) const {
        if (r0 >= M || c0w >= ldS) return 0;
        const long long left = (ldS - c0w) >> 5;
        return left < 4 ? (int)left : 4;
    }
    __device__ __forceinline__ Pre begin(long long r0w, long long c0w, int lane) const {
        Pre pre{{0u, 0u}};
        if (first) return pre;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int nl = live_tiles(r0w + i * 32, c0w);
            const long long t = ((r0w >> 5) + i) * tiles_n + (c0w >> 5);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j < nl) pre.have[i] |= (uint32_t)Mask[(t + j) * 64 + lane] << (8 * j);
        }
        return pre;
    }
    static constexpr bool kWhole = true;      // the kernel calls whole() instead of half(0), half(1)
    // All 2 x 4 tiles of the wavefront's block, in four batches of two tiles (batch b: row half b/2,
    // tiles 2*(b%2), 2*(b%2)+1).  The old-state loads of batch b+2 are issued before batch b+1 is
    // worked on, so from the second batch on their latency hides behind arithmetic and stores.
    __device__ __forceinline__ void whole(long long r0w, long long c0w, int lane, const f32x16 (&acc)[2][4], char* stage,
                                          const Pre& pre) const {
        // interior blocks (the common case) need no per-element bounds handling
        if (r0w + 64 <= M && c0w + 128 <= N && !Xo) run<false>(r0w, c0w, lane, acc, stage, pre);
        else run<true>(r0w, c0w, lane, acc, stage, pre);
    }
    template <bool EDGE>
    __device__ __forceinline__ void run(long long r0w, long long c0w, int lane, const f32x16 (&acc)[2][4], char* stage,
                                        const Pre& pre) const {
        const int li = lane & 31, lh = lane >> 5;
        const int nl[2] = {live_tiles(r0w, c0w), live_tiles(r0w + 32, c0w)};
        const long long t[2] = {(r0w >> 5) * tiles_n + (c0w >> 5), ((r0w >> 5) + 1) * tiles_n + (c0w >> 5)};
        __amdgpu_buffer_rsrc_t rs[2] = {
            __builtin_amdgcn_make_buffer_rsrc((void*)(Xs + t[0] * 256), 0, nl[0] * 4096, kBufferFlags),
            __builtin_amdgcn_make_buffer_rsrc((void*)(Xs + t[1] * 256), 0, nl[1] * 4096, kBufferFlags)};
        auto issue = [&](auto bc, u32x4 (&xo)[2][4]) {
            constexpr int b = decltype(bc)::value, i = b >> 1, j0 = (b & 1) * 2;
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int j = j0 + jj;
                    const int off = ((pre.have[i] >> (8 * j + g)) & 1) ? j * 4096 + g * 1024 + lane * 16 : kOutOfRange;
                    xo[jj][g] = __builtin_amdgcn_raw_buffer_load_b128(rs[i], off, 0, kStreamAux);
                }
        };
        auto work = [&](auto bc, const u32x4 (&xo)[2][4]) {
            constexpr int b = decltype(bc)::value, i = b >> 1, j0 = (b & 1) * 2;
            const long long r0 = r0w + 32 * i;
            char* sw = stage + (i * 32 + 4 * lh) * kPitch + li * 2;      // this lane's first staged element of the half
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int j = j0 + jj;
                const long long c = c0w + j * 32 + li;
                uint32_t nz = 0;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 old = __builtin_bit_cast(f32x4, xo[jj][g]);
                    f32x4 xn;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float u = old[e] + mu * acc[i][j][4 * g + e];
                        float x = u - __builtin_amdgcn_fmed3f(u, -theta, theta);
                        if constexpr (EDGE) {
                            const long long r = r0 + 8 * g + 4 * lh + e;
                            if (!(c < N && r < M)) x = 0.f;
                            if (Xo && c < N && r < M) Xo[r * (long long)N + c] = x;
                        }
                        xn[e] = x;
                    }
#pragma unroll
                    for (int e = 0; e < 4; e += 2) {
                        const uint32_t pk = f2bf_pk(xn[e], xn[e + 1]);
                        *(bf16_t*)(sw + (8 * g + e) * kPitch + j * 64) = (bf16_t)pk;
                        *(bf16_t*)(sw + (8 * g + e + 1) * kPitch + j * 64) = (bf16_t)(pk >> 16);
                    }
                    const u32x4 xb = __builtin_bit_cast(u32x4, xn);
                    const bool any = ((xb[0] | xb[1]) | (xb[2] | xb[3])) != 0u;    // a thresholded zero is +0
                    __builtin_amdgcn_raw_buffer_store_b128(xb, rs[i], any ? j * 4096 + g * 1024 + lane * 16 : kOutOfRange, 0, kStreamAux);
                    nz |= any ? 1u << g : 0u;
                }
                if (j < nl[i]) Mask[(t[i] + j) * 64 + lane] = (uint8_t)nz;
            }
        };
        using B0 = std::integral_constant<int, 0>;
        using B1 = std::integral_constant<int, 1>;
        using B2 = std::integral_constant<int, 2>;
        using B3 = std::integral_constant<int, 3>;
        u32x4 xa[2][4], xb2[2][4];
        issue(B0{}, xa);
        issue(B1{}, xb2);
        work(B0{}, xa);
        issue(B2{}, xa);
        work(B1{}, xb2);
        issue(B3{}, xb2);
        work(B2{}, xa);
        work(B3{}, xb2);
    }
    // The wavefront's staged 64 rows x 128 columns of bf16, written 16 bytes per lane:
    // one instruction covers 4 rows x 256 contiguous bytes.
    __device__ __forceinline__ void flush(long long r0, long long c0, int lane, const char* stage) const {
        const int chunk = lane & 15, rsub = lane >> 4;
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = p * 4 + rsub;
            const long long r = r0 + row, c = c0 + chunk * 8;
            if (r < M && c < ldS)
                *(uint4*)(Xb + r * ldS + c) = *(const uint4*)(stage + row * kPitch + chunk * 16);
        }
    }
};

// One layer of the unrolled decoder on the large-tile kernel: u = alpha + (S - I) alpha + B y.  The
// accumulators start from W = B y (stored in accumulator order by EpiStoreAccTiled, loaded before the
// main loop), so the epilogue is the ISTA one with mu = 1 and this layer's threshold.
struct EpiListaUpdateTiled : EpiIstaUpdateTiled {
    static constexpr bool kAccInit = true;
    const f32x4* W;
    __device__ __forceinline__ void init(long long r0w, long long c0w, int lane, f32x16 (&acc)[2][4]) const {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int nl = live_tiles(r0w + i * 32, c0w);
            const long long t = ((r0w >> 5) + i) * tiles_n + (c0w >> 5);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j < nl) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const f32x4 w = __builtin_nontemporal_load(W + (t + j) * 256 + g * 64 + lane);
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[i][j][4 * g + e] = w[e];
                    }
                }
        }
    }
};

// Stores the accumulators as they are, in accumulator order: tile (row tile, column tile) of 32 x 32 is
// 256 float4, [g][lane] = rows 8g + 4*lh .. +3 of column li.  Same tiling as the sparse iterate.
struct EpiStoreAccTiled {
    static constexpr bool kTile = true;
    static constexpr bool kWhole = true;
    static constexpr int kStageBytes = 0;
    struct Pre {};
    f32x4* W; long long tiles_n; long long ldS;
    long long M;
    __device__ __forceinline__ Pre begin(long long, long long, int) const { return {}; }
    __device__ __forceinline__ void whole(long long r0w, long long c0w, int lane, const f32x16 (&acc)[2][4], char*,
                                          const Pre&) const {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (r0w + i * 32 >= M || c0w >= ldS) continue;
            const long long left = (ldS - c0w) >> 5;
            const int nl = left < 4 ? (int)left : 4;
            const long long t = ((r0w >> 5) + i) * tiles_n + (c0w >> 5);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j < nl) {
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        W[(t + j) * 256 + g * 64 + lane] =
                            f32x4{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                }
        }
    }
    __device__ __forceinline__ void flush(long long, long long, int, const char*) const {}
};

template <typename E, typename = void> struct has_acc_init : std::false_type {};
template <typename E> struct has_acc_init<E, std::enable_if_t<E::kAccInit>> : std::true_type {};
template <typename E, typename = void> struct has_whole_epilogue : std::false_type {};
template <typename E> struct has_whole_epilogue<E, std::enable_if_t<E::kWhole>> : std::true_type {};
template <typename E, typename = void> struct has_tile_epilogue : std::false_type {};
template <typename E> struct has_tile_epilogue<E, std::enable_if_t<E::kTile>> : std::true_type {};

// ----------------------------------------------------------------------------------------
// Layout helpers (HBM-bound, off the dominant path).
// ----------------------------------------------------------------------------------------

// dst[r][0..ld) = convert(src[r][0..cols)) with zero fill up to ld.  One thread per element.
template <typename TI, typename TO>
__global__ void pack_rows_kernel(const TI* src, long long lds_, TO* dst, long long ldd, long long rows, int cols) {
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = rows * ldd;
    if (idx >= total) return;
    long long r = idx / ldd;
    int c = (int)(idx % ldd);
    float v = (c < cols) ? Elem<TI>::load(src + r * lds_ + c) : 0.f;
    Elem<TO>::store(dst + idx, v);
}

// dst[z][c][r] = src[z][r][c] for r < R, c < Cc; dst rows have ld = ldd >= R, zero filled.
// 32x32 tiles through LDS so both sides are coalesced.
template <typename T>
__global__ void transpose_pack_kernel(const T* src, long long strideS, T* dst, long long ldd, long long strideD,
                                      int R, int Cc) {
    __shared__ T tile[32][33];
    const int z = blockIdx.z;
    const int r0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    const T* s = src + (long long)z * strideS;
    T* d = dst + (long long)z * strideD;
    for (int i = threadIdx.y; i < 32; i += blockDim.y) {
        int r = r0 + i, c = c0 + threadIdx.x;
        tile[i][threadIdx.x] = (r < R && c < Cc) ? s[(long long)r * Cc + c] : (T)0;
    }
    __syncthreads();
    for (int i = threadIdx.y; i < 32; i += blockDim.y) {
        int c = c0 + i, r = r0 + threadIdx.x;
        if (c < Cc && r < ldd) d[(long long)c * ldd + r] = tile[threadIdx.x][i];
    }
}

// D[c][k] = S[c][k] - (c == k) for c, k < n, rows of D padded to ldd with zeros (operand layout).
template <typename T>
__global__ void sub_identity_pack_kernel(const T* S, int n, T* D, long long ldd) {
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)n * ldd) return;
    const long long c = idx / ldd, kcol = idx % ldd;
    float v = 0.f;
    if (kcol < n) v = Elem<T>::load(S + c * n + kcol) - (c == kcol ? 1.f : 0.f);
    Elem<T>::store(D + idx, v);
}

// dst[z][c][r] = (TO) src[z][r][c] for r < R, c < Cc (both contiguous), 32x32 tiles through LDS.
template <typename TO>
__global__ void transpose_cast_kernel(const float* src, TO* dst, int R, int Cc) {
    __shared__ float tile[32][33];
    const int z = blockIdx.z;
    const int r0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    const float* s = src + (long long)z * R * Cc;
    TO* d = dst + (long long)z * R * Cc;
    for (int i = threadIdx.y; i < 32; i += blockDim.y) {
        int r = r0 + i, c = c0 + threadIdx.x;
        tile[i][threadIdx.x] = (r < R && c < Cc) ? s[(long long)r * Cc + c] : 0.f;
    }
    __syncthreads();
    for (int i = threadIdx.y; i < 32; i += blockDim.y) {
        int c = c0 + i, r = r0 + threadIdx.x;
        if (c < Cc && r < R) Elem<TO>::store(d + (long long)c * R + r, tile[threadIdx.x][i]);
    }
}

// r = y - sum_s P[s] for a residual product that was split along K into S partial products
// P[s] [rows, ldR] (float): R [rows, ldR] in bf16 with zero pads.  One thread per element; the sum
// runs in a fixed order, so the result does not depend on how the partial launches were scheduled.
static __global__ void residual_reduce_kernel(const float* Y, long long ldY, const float* P, int S, long long strideP,
                                       bf16_t* R, long long ldR, long long rows, int m) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * ldR) return;
    const long long r = idx / ldR;
    const int c = (int)(idx % ldR);
    float v = 0.f;
    if (c < m) {
        float acc = 0.f;
        for (int s = 0; s < S; ++s) acc += P[s * strideP + idx];
        v = Y[r * ldY + c] - acc;
    }
    R[idx] = f2bf(v);
}

// zero `words` 4-byte words (a fill kernel rather than a memset node, so callers may capture it)
static __global__ void fill_zero_kernel(uint32_t* p, long long words) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0u;
}

// *p = value (one word; a kernel rather than a memset node, so callers may capture it)
// *p = value, and zero[0 .. words) = 0 (the fused decoder's counters, cleared in the same launch as its status word)
static __global__ void set_word_kernel(int* p, int value, uint32_t* zero, long long words) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = value;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride) zero[i] = 0u;
}

// When *err != 0, overwrites a[0..na) with the fp32 quiet NaN and b[0..nb) with pairs of the bf16 quiet NaN;
// otherwise does nothing.  Runs behind a decoder that may have given up, so that a failed call cannot be
// mistaken for a result.
static __global__ void poison_on_error_kernel(const int* err, uint32_t* a, long long na, uint32_t* b, long long nb) {
    if (*err == 0) return;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < na; i += stride) a[i] = 0x7fc00000u;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < nb; i += stride) b[i] = 0x7fc07fc0u;
}

// Row softmax in place over S [rows, m] (float), one wavefront per row: wavefront max and sum
// by cross-lane shuffles.  Also writes an operand copy P [rows, ldp] in TO with zero pads.
// Rows of S have leading dimension lds_ >= m; columns [m, lds_) are set to zero.
template <typename TO, int kHeld>      // kHeld scores per lane are kept in registers: rows up to 64*kHeld are read once
__global__ __launch_bounds__(256) void softmax_rows_kernel(float* S, long long lds_, long long rows, int m, TO* P,
                                                           long long ldp) {
    const int lane = threadIdx.x & 63;
    long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    float* s = S + r * lds_;
    if (m <= 64 * kHeld) {
        float v[kHeld];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < kHeld; ++i) {
            const int c = lane + 64 * i;
            v[i] = c < m ? s[c] : -INFINITY;
            mx = fmaxf(mx, v[i]);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < kHeld; ++i) {
            v[i] = lane + 64 * i < m ? expf(v[i] - mx) : 0.f;
            sum += v[i];
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        const float inv = 1.f / sum;
#pragma unroll
        for (int i = 0; i < kHeld; ++i) {
            const int c = lane + 64 * i;
            const float p = v[i] * inv;        // 0 beyond m
            if (c < lds_) s[c] = p;
            if (P && c < ldp) Elem<TO>::store(P + r * ldp + c, p);
        }
        for (int c = 64 * kHeld + lane; c < lds_; c += 64) s[c] = 0.f;
        if (P)
            for (int c = 64 * kHeld + lane; c < ldp; c += 64) Elem<TO>::store(P + r * ldp + c, 0.f);
        return;
    }
    float mx = -INFINITY;
    for (int c = lane; c < m; c += 64) mx = fmaxf(mx, s[c]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float sum = 0.f;
    for (int c = lane; c < m; c += 64) sum += expf(s[c] - mx);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    const float inv = 1.f / sum;
    for (int c = lane; c < m; c += 64) s[c] = expf(s[c] - mx) * inv;
    for (int c = m + lane; c < lds_; c += 64) s[c] = 0.f;
    if (P)
        for (int c = lane; c < ldp; c += 64) Elem<TO>::store(P + r * ldp + c, c < m ? s[c] : 0.f);
}

}  // namespace csat
