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

__device__ __forceinline__ bf16_t f2bf(float f) {
    // round to nearest even; NaN stays NaN
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
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
};

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

// The same update for the large-tile kernel, one 32x32 MFMA tile at a time: the fp32 state is kept
// in accumulator order ([row tile][column tile][4][lane] float4), so that a lane reads and writes
// its 16 values as four 16-byte accesses and a wavefront moves 1 KB per instruction.
struct EpiIstaUpdateTiled {
    static constexpr bool kTile = true;
    static constexpr int kPitch = 272;      // bytes per staged row: 128 bf16 + 16 (keeps 16-byte reads off one bank)
    f32x4* Xs; long long tiles_n;      // column tiles per row tile (ldS / 32)
    uint8_t* Mask;                     // [row tile][column tile][lane]: bit g = float4 g of that lane is non-zero
    bf16_t* Xb; long long ldS;
    float* Xo;
    float mu, theta;
    long long M; int N; int first;
    // One 32x32 MFMA tile (i, j) of the wavefront's 64x128 block.  The bf16 copy is staged in LDS
    // (`stage`, this wavefront's own 64 x kPitch bytes) so that flush() can write it out row-wise.
    __device__ __forceinline__ void tile(int, long long r0, long long c0, int lane, const f32x16& acc, char* stage,
                                         int i, int j) const {
        const int li = lane & 31, lh = lane >> 5;
        const long long c = c0 + li;
        const bool live = c0 < ldS && r0 < M;
        const long long t = (r0 >> 5) * tiles_n + (c0 >> 5);
        f32x4* s = Xs + t * 256 + lane;
        // the iterate is sparse: only the non-zero float4 of a lane are read and written
        const uint32_t have = (first || !live) ? 0u : Mask[t * 64 + lane];
        uint32_t nz = 0;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 xo = {0.f, 0.f, 0.f, 0.f};
            if ((have >> g) & 1) xo = s[g * 64];
            f32x4 xn;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const long long r = r0 + 8 * g + 4 * lh + e;
                float u = xo[e] + mu * acc[4 * g + e];
                float x = (c < N && r < M) ? u - __builtin_amdgcn_fmed3f(u, -theta, theta) : 0.f;
                xn[e] = x;
                *(bf16_t*)(stage + (i * 32 + 8 * g + 4 * lh + e) * kPitch + (j * 32 + li) * 2) = f2bf(x);
                if (Xo && c < N && r < M) Xo[r * (long long)N + c] = x;
            }
            if (live && (xn[0] != 0.f || xn[1] != 0.f || xn[2] != 0.f || xn[3] != 0.f)) {
                s[g * 64] = xn;
                nz |= 1u << g;
            }
        }
        if (live) Mask[t * 64 + lane] = (uint8_t)nz;
    }
    // The wavefront's staged 64 rows x 128 columns of bf16, written 16 bytes per lane:
    // one instruction covers 4 rows x 256 contiguous bytes.
    __device__ __forceinline__ void flush(long long r0, long long c0, int lane, const char* stage) const {
        const int chunk = lane & 15, rsub = lane >> 4;
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = p * 4 + rsub;
            const long long r = r0 + row, c = c0 + chunk * 8;
            if (r < M && c < ldS) *(uint4*)(Xb + r * ldS + c) = *(const uint4*)(stage + row * kPitch + chunk * 16);
        }
    }
};

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

// zero `words` 4-byte words (a fill kernel rather than a memset node, so callers may capture it)
__global__ void fill_zero_kernel(uint32_t* p, long long words) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0u;
}

// Row softmax in place over S [rows, m] (float), one wavefront per row: wavefront max and sum
// by cross-lane shuffles.  Also writes an operand copy P [rows, ldp] in TO with zero pads.
// Rows of S have leading dimension lds_ >= m; columns [m, lds_) are set to zero.
template <typename TO>
__global__ __launch_bounds__(256) void softmax_rows_kernel(float* S, long long lds_, long long rows, int m, TO* P,
                                                           long long ldp) {
    const int lane = threadIdx.x & 63;
    long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    float* s = S + r * lds_;
    float mx = -INFINITY;
    for (int c = lane; c < m; c += 64) mx = fmaxf(mx, s[c]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float sum = 0.f;
    for (int c = lane; c < m; c += 64) sum += expf(s[c] - mx);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    const float inv = 1.f / sum;
    for (int c = lane; c < ldp; c += 64) {
        float p = 0.f;
        if (c < m) {
            p = expf(s[c] - mx) * inv;
            s[c] = p;
        }
        if (P) Elem<TO>::store(P + r * ldp + c, p);
    }
    for (int c = m + lane; c < lds_; c += 64) s[c] = 0.f;
}

}  // namespace csat
