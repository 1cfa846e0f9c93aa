// Orthogonal matching pursuit, the greedy decoder the paper names next to ISTA (introduction and
// limitations sections; it gives no details, so this is the standard algorithm).  Per row: k times
// pick the column of Phi most correlated with the residual (largest |phi_j^T r|, lowest index on a
// tie, never a column twice), refit the picked coefficients by least squares, update the residual.
//
// The correlations of all rows are one GEMM per pick (R Phi, the decoder's update product).  The
// least-squares refit is kept as an incrementally built QR factorisation per row (modified
// Gram-Schmidt): with the picked columns Phi_S = Q T (Q orthonormal, T upper triangular), the
// residual update is r <- r - (q^T r) q for the new q only, and the coefficients follow once at the
// end from T x = Q^T y.  One wavefront per row, lanes strided over m, fp32 throughout.
#pragma once
#include "csat_kernels.h"

namespace csat {

constexpr int kOmpMaxPicks = 32;     // registers of the finishing kernel hold one coefficient per pick
constexpr int kOmpMaxM = 1024;       // 16 values of an m-vector per lane

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// picks[r][it] = argmax_c |Cm[r][c]| over the columns not picked before (lowest index on a tie)
static __global__ __launch_bounds__(256) void omp_pick_kernel(const float* Cm, long long ldc, long long rows, int n, int* picks,
                                                       int k, int it) {
    const int lane = threadIdx.x & 63;
    const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const float* c = Cm + r * ldc;
    int* pk = picks + r * k;
    float best = -1.f;
    int bi = 0x7fffffff;
    const int mine = lane < it ? pk[lane] : -1;    // earlier picks, one per lane (it <= 32)
    // four columns per lane and step (rows of Cm are 16-byte aligned: ldc is a multiple of 4)
    for (int j4 = lane * 4; j4 < n; j4 += 256) {
        const f32x4 cv = __builtin_nontemporal_load((const f32x4*)(c + j4));      // read once: keep it out of the caches' way
        float a[4] = {fabsf(cv[0]), fabsf(cv[1]), fabsf(cv[2]), fabsf(cv[3])};
        for (int s = 0; s < it; ++s) {            // uniform trip count: only the picks made so far
            const int d = __builtin_amdgcn_readlane(mine, s) - j4;
#pragma unroll
            for (int e = 0; e < 4; ++e) a[e] = d == e ? -2.f : a[e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j4 + e < n && a[e] > best) { best = a[e]; bi = j4 + e; }    // ascending index per lane: the first maximum stays
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
    }
    if (lane == 0) pk[it] = bi < n ? bi : 0;      // only reachable when every correlation is NaN
}

// Adds the picked column to the row's factorisation and updates its residual.
//   PhiT [n, ldp]   columns of Phi as rows (element type T)
//   Qb [rows, k, mq]  orthonormal vectors, Tri [rows, k, k] the triangular factor (column `it` written here),
//   Z [rows, k]  q^T y,  Rf [rows, mq] fp32 residual (in/out),  Rop [rows, ldr] operand copy of it (pads zero)
// MQ: values of an m-vector per lane, ceil(m / 64) rounded up to 4, 8 or 16.
template <typename T, int MQ>
__global__ __launch_bounds__(256) void omp_update_kernel(const T* PhiT, long long ldp, int m, const int* picks, int k, int it,
                                                         float* Qb, float* Tri, float* Z, float* Rf, int mq, T* Rop,
                                                         long long ldr, long long rows) {
    const int lane = threadIdx.x & 63;
    const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int j = picks[r * k + it];
    const T* col = PhiT + (long long)j * ldp;
    float* qrow = Qb + r * (long long)k * mq;
    float v[MQ];
#pragma unroll
    for (int i = 0; i < MQ; ++i) {
        const int l = lane + 64 * i;
        v[i] = l < m ? Elem<T>::load(col + l) : 0.f;
    }
    for (int s = 0; s < it; ++s) {
        const float* q = qrow + (long long)s * mq;
        float qv[MQ];
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < MQ; ++i) {
            const int l = lane + 64 * i;
            qv[i] = l < mq ? q[l] : 0.f;
            dot += qv[i] * v[i];
        }
        dot = wave_sum(dot);
        if (lane == 0) Tri[(r * k + s) * k + it] = dot;
#pragma unroll
        for (int i = 0; i < MQ; ++i) v[i] -= dot * qv[i];
    }
    float nn = 0.f;
#pragma unroll
    for (int i = 0; i < MQ; ++i) nn += v[i] * v[i];
    const float nrm = sqrtf(wave_sum(nn));
    const float inv = nrm > 0.f ? 1.f / nrm : 0.f;       // a column inside the span of the earlier picks adds nothing
    if (lane == 0) Tri[(r * k + it) * k + it] = nrm;
    float* res = Rf + r * mq;
    float zt = 0.f;
    float rv[MQ];
#pragma unroll
    for (int i = 0; i < MQ; ++i) {
        const int l = lane + 64 * i;
        v[i] *= inv;
        if (l < mq) qrow[(long long)it * mq + l] = v[i];
        rv[i] = l < mq ? res[l] : 0.f;
        zt += v[i] * rv[i];
    }
    zt = wave_sum(zt);
    if (lane == 0) Z[r * k + it] = zt;
#pragma unroll
    for (int i = 0; i < MQ; ++i) {
        const int l = lane + 64 * i;
        const float x = rv[i] - zt * v[i];
        if (l < mq) res[l] = x;
        if (l < ldr) Elem<T>::store(Rop + r * ldr + l, l < m ? x : 0.f);
    }
    for (int l = lane + 64 * MQ; l < ldr; l += 64) Elem<T>::store(Rop + r * ldr + l, 0.f);    // operand pads beyond the lanes' share
}

// Coefficients from T x = z by back substitution, scattered into X (zeroed beforehand); optional
// copy of the picks and C[r,:] = sum_s x_s V[head(r), pick_s, :].
template <typename T>
__global__ __launch_bounds__(256) void omp_finish_kernel(const float* Tri, const float* Z, const int* picks, int k, long long rows,
                                                         int n_q, int n, int d, float* X, int* picks_out, const T* V, T* C) {
    const int lane = threadIdx.x & 63;
    const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const float* tri = Tri + r * (long long)k * k;
    const int* pk = picks + r * k;
    float x[kOmpMaxPicks];
#pragma unroll
    for (int s = 0; s < kOmpMaxPicks; ++s) x[s] = 0.f;
    // every lane runs the same k^2/2 operations (k <= 32): no communication needed
#pragma unroll
    for (int s = kOmpMaxPicks - 1; s >= 0; --s) {
        if (s < k) {
            float acc = Z[r * k + s];
#pragma unroll
            for (int t = 0; t < kOmpMaxPicks; ++t)
                if (t > s && t < k) acc -= tri[s * k + t] * x[t];
            const float dg = tri[s * k + s];
            x[s] = dg > 0.f ? acc / dg : 0.f;
        }
    }
#pragma unroll
    for (int s = 0; s < kOmpMaxPicks; ++s) {
        if (s < k && lane == 0) {
            if (X) X[r * (long long)n + pk[s]] = x[s];
            if (picks_out) picks_out[r * k + s] = pk[s];
        }
    }
    if (C) {
        const T* v = V + (r / n_q) * (long long)n * d;
        for (int c = lane; c < d; c += 64) {
            float acc = 0.f;
#pragma unroll
            for (int s = 0; s < kOmpMaxPicks; ++s)
                if (s < k) acc += x[s] * Elem<T>::load(v + (long long)pk[s] * d + c);
            Elem<T>::store(C + r * (long long)d + c, acc);
        }
    }
}

}  // namespace csat
