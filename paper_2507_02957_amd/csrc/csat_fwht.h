// ISTA decoder for a structured measurement matrix.  Section 3's sentence on measurement ensembles names
// structured Hadamard matrices next to random Gaussian and Rademacher ones and gives no construction; the one
// used here (row subsampling, random column signs, 1/sqrt(m) scale) is this library's own:
// Phi = m rows of the Walsh-Hadamard matrix H_N (N = the power of two >= n,
// natural ordering), columns flipped by signs s, first n columns, scaled by c = 1/sqrt(m):
//     Phi x   = c * (H_N (s . x, zero padded))[rows]
//     Phi^T r = c * s . (H_N (r scattered to `rows`, zero elsewhere))[0..n)
// so both products of an iteration are one fast Walsh-Hadamard transform of length N (N log2 N
// additions) instead of 2 m n multiply-adds, and a row's whole decode runs out of LDS: nothing of
// the iterate touches memory between the first and the last iteration.
//
// One workgroup (256 to 1024 threads) per row.  The transform runs in place on an LDS array in passes
// of up to four butterfly stages: a thread loads the 16 elements whose indices differ in the pass's
// bits, does the butterflies in registers and stores them back (about log2 N / 4 LDS round trips
// instead of log2 N).  Index i lives at word i + i/32 so that the strided accesses of the later
// passes spread over the banks.
#pragma once
#include "csat_kernels.h"

namespace csat {

struct HadamardArgs {
    const float* Y; long long ldy;   // [rows, m] measurements
    const int* rows_of_h;            // [m] rows of H_N, ascending
    const signed char* signs;        // [N] +-1
    float* X;                        // [rows, n] final iterate in caller layout, or null
    void* Xop; long long ldx;        // [rows, ldx] final iterate as GEMM operand (element type T, pads zero), or null
    long long rows;
    int n, m, N, logN, iters;
    float mu, theta, scale;          // scale: 1/sqrt(m) as the element type holds it
};

constexpr int kFwhtMaxN = 16384;
__host__ __device__ inline int fwht_pad(int i) { return i + (i >> 5); }
inline size_t ista_hadamard_lds_bytes(int N, int m) { return (size_t)(N + fwht_pad(N) + 1 + 2 * m) * 4; }

// One pass of K butterfly stages on bits [b0, b0+K) of the index: a thread takes the 2^K elements of a
// group into registers, transforms them and stores them back.
template <int NT, int K, bool SYNC = true>
__device__ __forceinline__ void fwht_pass(float* W, int logN, int b0, int tid) {
    constexpr int E = 1 << K;
    const int groups = 1 << (logN - K);
#pragma unroll 1
    for (int g = tid; g < groups; g += NT) {
        const int lo = g & ((1 << b0) - 1), hi = g >> b0;
        const int base = (hi << (b0 + K)) | lo;
        float v[E];
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = W[fwht_pad(base + (e << b0))];
#pragma unroll
        for (int s = 0; s < K; ++s)
#pragma unroll
            for (int e = 0; e < E; ++e)
                if (!(e & (1 << s))) {
                    const float p = v[e], q = v[e | (1 << s)];
                    v[e] = p + q;
                    v[e | (1 << s)] = p - q;
                }
#pragma unroll
        for (int e = 0; e < E; ++e) W[fwht_pad(base + (e << b0))] = v[e];
    }
    if (SYNC) __syncthreads();
}

// In-place transform of W[fwht_pad(0..N-1)], N = 2^logN, by the whole workgroup of NT threads, in
// balanced passes of at most 4 stages, and no more than leaves every thread a group.
// `top` < logN: only the stages of index bits [0, top) (the caller does the others).
template <int NT>
__device__ __forceinline__ void fwht_lds(float* W, int logN, int tid, int top = -1) {
    int kmax = logN - (31 - __builtin_clz(NT));
    kmax = kmax < 1 ? 1 : (kmax > 4 ? 4 : kmax);
    if (top < 0) top = logN;
    for (int b0 = 0; b0 < top;) {
        const int left = top - b0;
        const int passes = (left + kmax - 1) / kmax;
        const int k = (left + passes - 1) / passes;
        switch (k) {
            case 1: fwht_pass<NT, 1>(W, logN, b0, tid); break;
            case 2: fwht_pass<NT, 2>(W, logN, b0, tid); break;
            case 3: fwht_pass<NT, 3>(W, logN, b0, tid); break;
            default: fwht_pass<NT, 4>(W, logN, b0, tid); break;
        }
        b0 += k;
    }
}

// The same transform on `cols` buffers `stride` words apart, one barrier per pass for all of them.
template <int NT>
__device__ __forceinline__ void fwht_lds_multi(float* W, int stride, int cols, int logN, int tid) {
    int kmax = logN - (31 - __builtin_clz(NT));
    kmax = kmax < 1 ? 1 : (kmax > 4 ? 4 : kmax);
    for (int b0 = 0; b0 < logN;) {
        const int left = logN - b0;
        const int passes = (left + kmax - 1) / kmax;
        const int k = (left + passes - 1) / passes;
        for (int q = 0; q < cols; ++q) {
            float* Wq = W + q * stride;
            switch (k) {
                case 1: fwht_pass<NT, 1, false>(Wq, logN, b0, tid); break;
                case 2: fwht_pass<NT, 2, false>(Wq, logN, b0, tid); break;
                case 3: fwht_pass<NT, 3, false>(Wq, logN, b0, tid); break;
                default: fwht_pass<NT, 4, false>(Wq, logN, b0, tid); break;
            }
        }
        __syncthreads();
        b0 += k;
    }
}

// NT threads per row: 256 up to N = 2048, more for longer transforms (more wavefronts to hide LDS latency)
template <typename T, int NT>
__global__ __launch_bounds__(NT) void ista_hadamard_kernel(HadamardArgs a) {
    extern __shared__ float hl[];
    float* Xl = hl;                               // [N]      the iterate
    float* Wl = Xl + a.N;                         // [pad(N)+1] transform buffer
    float* Yl = Wl + fwht_pad(a.N) + 1;           // [m]      measurements of this row
    float* Rl = Yl + a.m;                         // [m]      residual
    const int tid = threadIdx.x;
    const float cs = a.mu * a.scale;
    // a row index outside H_N would leave the transform buffer: clamp (the result is then wrong, not a fault)
    auto hrow = [&](int l) { const int v = a.rows_of_h[l]; return v < 0 ? 0 : (v >= a.N ? a.N - 1 : v); };
    for (long long r = blockIdx.x; r < a.rows; r += gridDim.x) {
        for (int l = tid; l < a.m; l += NT) Yl[l] = a.Y[r * a.ldy + l];
        for (int i = tid; i < a.N; i += NT) Xl[i] = 0.f;
        __syncthreads();
        for (int t = 0; t < a.iters; ++t) {
            if (t > 0) {      // r = y - Phi x
                for (int i = tid; i < a.N; i += NT) Wl[fwht_pad(i)] = i < a.n ? (float)a.signs[i] * Xl[i] : 0.f;
                __syncthreads();
                fwht_lds<NT>(Wl, a.logN, tid);
                for (int l = tid; l < a.m; l += NT) Rl[l] = Yl[l] - a.scale * Wl[fwht_pad(hrow(l))];
            } else {
                for (int l = tid; l < a.m; l += NT) Rl[l] = Yl[l];
            }
            __syncthreads();
            for (int i = tid; i < a.N; i += NT) Wl[fwht_pad(i)] = 0.f;      // Phi^T r: the residual scattered to its rows of H
            __syncthreads();
            for (int l = tid; l < a.m; l += NT) Wl[fwht_pad(hrow(l))] = Rl[l];
            __syncthreads();
            fwht_lds<NT>(Wl, a.logN, tid);
            for (int i = tid; i < a.n; i += NT) {
                const float u = Xl[i] + cs * (float)a.signs[i] * Wl[fwht_pad(i)];
                Xl[i] = u - __builtin_amdgcn_fmed3f(u, -a.theta, a.theta);
            }
            __syncthreads();
        }
        if (a.X)
            for (int i = tid; i < a.n; i += NT) a.X[r * (long long)a.n + i] = Xl[i];
        if (a.Xop)
            for (int i = tid; i < a.ldx; i += NT) Elem<T>::store((T*)a.Xop + r * a.ldx + i, i < a.n ? Xl[i] : 0.f);
        __syncthreads();
    }
}

// All RB butterfly stages over 2^RB values held in registers.
template <int RB>
__device__ __forceinline__ void fwht_regs(float (&v)[1 << RB]) {
#pragma unroll
    for (int s = 0; s < RB; ++s)
#pragma unroll
        for (int q = 0; q < (1 << RB); ++q)
            if (!(q & (1 << s))) {
                const float a = v[q], b = v[q | (1 << s)];
                v[q] = a + b;
                v[q | (1 << s)] = a - b;
            }
}

// The same passes with the transform length and the bit range known at compile time (the register-resident
// kernel): element e of a group sits at a constant distance from the group's first element, because for a
// group base whose bits [B0, B0+K) are zero, fwht_pad(base + d) = fwht_pad(base) + d + d/32 for d = e << B0
// (the low bits of base never carry into bit 5 of d) -- so one address per group, the rest are immediates.
template <int NT, int LOGN, int B0, int K>
__device__ __forceinline__ void fwht_pass_static(float* W, int tid) {
    constexpr int E = 1 << K, GROUPS = 1 << (LOGN - K);
#pragma unroll 1
    for (int g = tid; g < GROUPS; g += NT) {
        const int lo = g & ((1 << B0) - 1), hi = g >> B0;
        float* Wb = W + fwht_pad((hi << (B0 + K)) | lo);
        float v[E];
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = Wb[(e << B0) + ((e << B0) >> 5)];
        fwht_regs<K>(v);
#pragma unroll
        for (int e = 0; e < E; ++e) Wb[(e << B0) + ((e << B0) >> 5)] = v[e];
    }
    __syncthreads();
}
// stages of index bits [B0, TOP) in balanced passes of at most four, and no more than leaves every thread a group
template <int NT, int LOGN, int TOP, int B0 = 0>
__device__ __forceinline__ void fwht_lds_static(float* W, int tid) {
    if constexpr (B0 < TOP) {
        constexpr int LOGNT = NT == 64 ? 6 : NT == 128 ? 7 : NT == 256 ? 8 : NT == 512 ? 9 : 10;
        constexpr int KM = LOGN - LOGNT < 1 ? 1 : (LOGN - LOGNT > 4 ? 4 : LOGN - LOGNT);
        constexpr int LEFT = TOP - B0, PASSES = (LEFT + KM - 1) / KM, K = (LEFT + PASSES - 1) / PASSES;
        fwht_pass_static<NT, LOGN, B0, K>(W, tid);
        fwht_lds_static<NT, LOGN, TOP, B0 + K>(W, tid);
    }
}

// inv[i] = l where rows_of_h[l] == i, else -1 (N entries).  Two launches: fill, then scatter.
static __global__ void hadamard_inverse_fill_kernel(int* inv, int N) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) inv[i] = -1;
}
static __global__ void hadamard_inverse_scatter_kernel(const int* rows_of_h, int m, int N, int* inv) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= m) return;
    const int v = rows_of_h[l];
    inv[v < 0 ? 0 : (v >= N ? N - 1 : v)] = l;
}

// The same decoder for long transforms (N = NT * VPT >= 4096).  The iterate, the column signs and the
// inverse of the row selection live in registers (thread tid owns indices tid + NT*j), so LDS holds only
// the transform buffer: two workgroups fit a CU at N = 16384 and fill each other's barrier waits, the
// zero-fill-then-scatter of the residual becomes one gather through the inverse map, and the iterate
// makes no LDS round trip.
template <typename T, int NT, int VPT>
__global__ __launch_bounds__(NT, 4) void ista_hadamard_reg_kernel(HadamardArgs a, const int* __restrict__ inv) {
    extern __shared__ float hl[];
    float* Wl = hl;                               // [pad(N)+1] transform buffer
    float* Yl = Wl + fwht_pad(a.N) + 1;           // [m]      measurements of this row
    float* Rl = Yl + a.m;                         // [m]      residual
    const int tid = threadIdx.x;
    const float cs = a.mu * a.scale;
    auto hrow = [&](int l) { const int v = a.rows_of_h[l]; return v < 0 ? 0 : (v >= a.N ? a.N - 1 : v); };
    // index tid + NT*j sits at word fwht_pad(tid) + j * (NT + NT/32): one base, constant offsets
    float* Wt = Wl + fwht_pad(tid);
    constexpr int WS = NT + NT / 32;
    // The values a thread owns differ in the top log2 VPT bits of the index, so the stages of (up to four
    // of) those bits are butterflies among its own registers: on the way into LDS for the first transform
    // of an iteration (its result is read at the selected rows, from LDS), on the way out for the second
    // (its result meets the iterate in registers).  LDS passes cover the bits below.
    constexpr int LOGV = VPT == 2 ? 1 : VPT == 4 ? 2 : VPT == 8 ? 3 : VPT == 16 ? 4 : 5;
    constexpr int RB = LOGV < 4 ? LOGV : 4, G = VPT >> RB;
    constexpr int LOGN = LOGV + (NT == 64 ? 6 : NT == 128 ? 7 : NT == 256 ? 8 : 9), TOP = LOGN - RB;
    // residual entry that lands on index tid + NT*j, 16 bits each (m <= 16384), 0xffff = none
    uint32_t src[VPT / 2];
    uint32_t neg = 0;                             // bit j: the column sign of index tid + NT*j is -1
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int i = tid + NT * j;
        const uint32_t v = (uint32_t)inv[i] & 0xffffu;
        src[j / 2] = (j & 1) ? (src[j / 2] | (v << 16)) : v;
        neg |= (a.signs[i] < 0 ? 1u : 0u) << j;
    }
    for (long long r = blockIdx.x; r < a.rows; r += gridDim.x) {
        float x[VPT];
#pragma unroll
        for (int j = 0; j < VPT; ++j) x[j] = 0.f;
        for (int l = tid; l < a.m; l += NT) Yl[l] = a.Y[r * a.ldy + l];
        __syncthreads();
        for (int t = 0; t < a.iters; ++t) {
            if (t > 0) {      // r = y - Phi x   (x is zero beyond n)
#pragma unroll
                for (int p = 0; p < G; ++p) {
                    float v[1 << RB];
#pragma unroll
                    for (int q = 0; q < (1 << RB); ++q) v[q] = ((neg >> (p + G * q)) & 1) ? -x[p + G * q] : x[p + G * q];
                    fwht_regs<RB>(v);
#pragma unroll
                    for (int q = 0; q < (1 << RB); ++q) Wt[(p + G * q) * WS] = v[q];
                }
                __syncthreads();
                fwht_lds_static<NT, LOGN, TOP>(Wl, tid);
                for (int l = tid; l < a.m; l += NT) Rl[l] = Yl[l] - a.scale * Wl[fwht_pad(hrow(l))];
            } else {
                for (int l = tid; l < a.m; l += NT) Rl[l] = Yl[l];
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < VPT; ++j) {      // Phi^T r: the residual gathered to its rows of H
                const uint32_t l = (src[j / 2] >> (16 * (j & 1))) & 0xffffu;
                Wt[j * WS] = l != 0xffffu ? Rl[l] : 0.f;
                if (j % 8 == 7) asm volatile("" ::: "memory");      // eight gathers in flight, not VPT: registers
            }
            __syncthreads();
            fwht_lds_static<NT, LOGN, TOP>(Wl, tid);
#pragma unroll
            for (int p = 0; p < G; ++p) {
                float v[1 << RB];
#pragma unroll
                for (int q = 0; q < (1 << RB); ++q) v[q] = Wt[(p + G * q) * WS];
                fwht_regs<RB>(v);
#pragma unroll
                for (int q = 0; q < (1 << RB); ++q) {
                    const int j = p + G * q;
                    if (tid + NT * j < a.n) {
                        const float u = x[j] + cs * (((neg >> j) & 1) ? -v[q] : v[q]);
                        x[j] = u - __builtin_amdgcn_fmed3f(u, -a.theta, a.theta);
                    }
                }
            }
            __syncthreads();
        }
        float* xo = a.X ? a.X + r * (long long)a.n + tid : nullptr;
        T* xp = a.Xop ? (T*)a.Xop + r * a.ldx + tid : nullptr;
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            const int i = tid + NT * j;
            if (xo && i < a.n) xo[NT * j] = x[j];
            if (xp && i < a.ldx) Elem<T>::store(xp + NT * j, x[j]);
            asm volatile("" ::: "memory");      // one address pair at a time (registers)
        }
    }
}

// Measurement with the structured matrix (section 3, K~ = Phi K): for every head and feature column c,
// K~[:, c] = scale * (H_N (s . K[:, c], zero padded))[rows] -- one transform of length N per column instead of
// an m x n product, and no stored Phi at all.  A workgroup takes one head and a group of CB = 16 / sizeof(T)
// columns (one 16-byte load per token), transforms them `held` at a time (as many as fit LDS) and writes the m
// selected entries of each.
//   In [BH, n, d] -> Out [BH, m, d], both element type T; grid (ceil(d / CB), BH).
//   OutHL (bf16 mode, optional): [BH, m, 2d], the value as a (hi | lo) bf16 pair for the score contraction.
template <typename T, int NT>
__global__ __launch_bounds__(NT) void measure_hadamard_kernel(const T* __restrict__ In, T* __restrict__ Out,
                                                              const int* __restrict__ rows_of_h,
                                                              const signed char* __restrict__ signs, int n, int d, int m,
                                                              int N, int logN, float scale, int held,
                                                              bf16_t* __restrict__ OutHL) {
    constexpr int CB = 16 / (int)sizeof(T);
    extern __shared__ float hm[];
    const int tid = threadIdx.x;
    const int c0 = blockIdx.x * CB;
    const long long bh = blockIdx.y;
    const T* in = In + bh * (long long)n * d;
    T* out = Out + bh * (long long)m * d;
    const int stride = fwht_pad(N) + 1;            // words per column buffer
    const bool vec = d % CB == 0 && c0 + CB <= d;      // a token's CB columns are one aligned 16-byte piece
    for (int cb = 0; cb < CB && c0 + cb < d; cb += held) {
        const int cols = min(held, min(CB - cb, d - c0 - cb));
        for (int j = tid; j < N; j += NT) {
            const float sg = j < n ? (float)signs[j] : 0.f;
            if (j < n && vec) {
                const uint4 raw = *(const uint4*)(in + (long long)j * d + c0);
                const T* e = (const T*)&raw;
#pragma unroll
                for (int q = 0; q < CB; ++q)       // static indices into the loaded piece
                    if (q >= cb && q < cb + cols) hm[(q - cb) * stride + fwht_pad(j)] = sg * Elem<T>::load(e + q);
            } else {
                for (int q = 0; q < cols; ++q)
                    hm[q * stride + fwht_pad(j)] = j < n ? sg * Elem<T>::load(in + (long long)j * d + c0 + cb + q) : 0.f;
            }
        }
        __syncthreads();
        fwht_lds_multi<NT>(hm, stride, cols, logN, tid);
        for (int l = tid; l < m; l += NT) {
            const int v = rows_of_h[l];
            const int hr = fwht_pad(v < 0 ? 0 : (v >= N ? N - 1 : v));
            for (int q = 0; q < cols; ++q) {
                const float v = scale * hm[q * stride + hr];
                Elem<T>::store(out + (long long)l * d + c0 + cb + q, v);
                if constexpr (sizeof(T) == 2) {
                    if (OutHL) {
                        bf16_t* hl = OutHL + (bh * m + l) * 2 * d + c0 + cb + q;
                        const bf16_t hi = f2bf(v);
                        hl[0] = hi;
                        hl[d] = f2bf(v - bf2f(hi));
                    }
                }
            }
        }
        __syncthreads();
    }
}

// Measurement of the compressed output's feature columns for the column-wise reading, Y = Phi Z by transforms:
// row r = (head, column) of ZT holds that column along the tokens (element type T; in bf16 mode as a hi | lo
// pair, lo_off elements apart, which carries Z to ~16 mantissa bits); Yt [rows, ldy] (float, pads zeroed) receives
// its m measurements.  One workgroup per row.
template <typename T, int NT>
__global__ __launch_bounds__(NT) void measure_columns_hadamard_kernel(const T* __restrict__ ZT, long long ldzt, long long lo_off,
                                                                      const int* __restrict__ rows_of_h,
                                                                      const signed char* __restrict__ signs,
                                                                      float* __restrict__ Yt, long long ldy, long long rows,
                                                                      int n, int m, int N, int logN, float scale) {
    extern __shared__ float hc[];
    const int tid = threadIdx.x;
    for (long long r = blockIdx.x; r < rows; r += gridDim.x) {
        const T* z = ZT + r * ldzt;
        for (int j = tid; j < N; j += NT) {
            float v = 0.f;
            if (j < n) {
                v = Elem<T>::load(z + j);
                if (lo_off) v += Elem<T>::load(z + lo_off + j);
                v *= (float)signs[j];
            }
            hc[fwht_pad(j)] = v;
        }
        __syncthreads();
        fwht_lds<NT>(hc, logN, tid);
        for (int l = tid; l < ldy; l += NT) {
            float y = 0.f;
            if (l < m) {
                const int h = rows_of_h[l];
                y = scale * hc[fwht_pad(h < 0 ? 0 : (h >= N ? N - 1 : h))];
            }
            Yt[r * ldy + l] = y;
        }
        __syncthreads();
    }
}

}  // namespace csat
