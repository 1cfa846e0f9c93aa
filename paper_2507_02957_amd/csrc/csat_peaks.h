// Reference kernels that measure what this chip delivers for the two roofs the decoder is priced
// against: a streaming copy (HBM) and a register-resident bf16 MFMA loop (matrix cores); and what one
// wavefront per SIMD can issue next to its MFMAs.  None is on the product path; the benchmark launches them
// to quote "achievable" next to the published peaks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "csat_kernels.h"

namespace csat {

// dst[i] = src[i] for n 16-byte words; grid-stride, four coalesced b128 loads in flight per lane, streaming
// (non-temporal) accesses since nothing is reused
static __global__ __launch_bounds__(256) void peak_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                        long long n) {
    typedef __attribute__((ext_vector_type(4))) unsigned int u4;
    const u4* s = (const u4*)src;
    u4* d = (u4*)dst;
    const long long stride = (long long)gridDim.x * 256;
    long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        u4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = __builtin_nontemporal_load(s + i + k * stride);
#pragma unroll
        for (int k = 0; k < 4; ++k) __builtin_nontemporal_store(v[k], d + i + k * stride);
    }
    for (; i < n; i += stride) d[i] = s[i];
}

constexpr int kPeakMfmaPerIter = 16;                                   // MFMAs per wavefront and loop iteration
constexpr double kPeakMfmaFlopsEach = 2.0 * 32 * 32 * 16;             // one v_mfma_f32_32x32x16_bf16

// Every wavefront issues iters * 16 MFMAs on four independent accumulator tiles, operands held in
// registers: no LDS, no memory traffic inside the loop.  The sums are stored once so nothing is elided.
static __global__ __launch_bounds__(256) void peak_mfma_kernel(float* __restrict__ out, int iters) {
    typedef __attribute__((ext_vector_type(8))) __bf16 frag_t;
    typedef __attribute__((ext_vector_type(16))) float acc_t;
    frag_t a, b;
    // operands with all mantissa bits in play, as real data has: the sustained clock depends on what the
    // multipliers toggle (a loop over zeros runs at a higher clock than any real product)
    unsigned h = (threadIdx.x + 1u) * 2654435761u;
    for (int i = 0; i < 8; ++i) {
        h = h * 1664525u + 1013904223u;
        a[i] = (__bf16)((float)(int)(h >> 8 & 0xffff) * (1.f / 32768.f) - 1.f);
        h = h * 1664525u + 1013904223u;
        b[i] = (__bf16)((float)(int)(h >> 8 & 0xffff) * (1.f / 32768.f) - 1.f);
    }
    acc_t acc[4];
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kPeakMfmaPerIter; ++k)
            acc[k & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k & 3], 0, 0, 0);
    }
    float t = 0.f;
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) t += acc[j][v];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

// What ONE wavefront per SIMD (the fused decoder's occupancy: its registers leave room for no second one) can
// issue next to its MFMAs: a loop of { MFMA; KV independent fp32 fmas; KL 16-byte LDS reads per lane }, four
// accumulator tiles, operands as above.  With a single wavefront nothing else can fill the issue slots, so the
// time per MFMA shows how many other instructions fit under one before they delay the next.
constexpr size_t kPeakIssueLdsBytes = 96 * 1024;       // (more than half of the LDS: one workgroup per CU)
template <int KV, int KL>
static __global__ __launch_bounds__(256, 1) void peak_issue_kernel(float* __restrict__ out, int iters) {
    typedef __attribute__((ext_vector_type(8))) __bf16 frag_t;
    typedef __attribute__((ext_vector_type(16))) float acc_t;
    typedef __attribute__((ext_vector_type(4))) unsigned int u4;
    extern __shared__ uint4 peak_lds[];
    for (int i = threadIdx.x; i < 4096; i += 256) peak_lds[i] = uint4{(unsigned)i, 1u, 2u, 3u};
    __syncthreads();
    const int lane = threadIdx.x & 63;
    frag_t a, b;
    unsigned h = (threadIdx.x + 1u) * 2654435761u;
    for (int i = 0; i < 8; ++i) {
        h = h * 1664525u + 1013904223u;
        a[i] = (__bf16)((float)(int)(h >> 8 & 0xffff) * (1.f / 32768.f) - 1.f);
        h = h * 1664525u + 1013904223u;
        b[i] = (__bf16)((float)(int)(h >> 8 & 0xffff) * (1.f / 32768.f) - 1.f);
    }
    acc_t acc[4];
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    float v[KV > 0 ? KV : 1];
    for (int k = 0; k < (KV > 0 ? KV : 1); ++k) v[k] = 1e-3f * (lane + k);
    u4 r[2] = {};
    const unsigned laddr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)peak_lds + lane * 16;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j & 3], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < KV; ++k) {
                v[k] = __builtin_fmaf(v[k], 1.0001f, 0.5f);
                asm volatile("" : "+v"(v[k]));
            }
#pragma unroll
            for (int k = 0; k < KL; ++k)
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r[k & 1]) : "v"(laddr), "n"(1024 * (k + 1)));
            __builtin_amdgcn_sched_barrier(0);
        }
        if (KL) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    float t = 0.f;
    for (int j = 0; j < 4; ++j)
        for (int e = 0; e < 16; ++e) t += acc[j][e];
    for (int k = 0; k < KV; ++k) t += v[k];
    t += (float)r[0][0] + (float)r[1][0];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

}  // namespace csat
