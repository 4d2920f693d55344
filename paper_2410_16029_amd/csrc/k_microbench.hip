// Micro-benchmarks behind ng_microbench: what this GPU sustains on a plain stream and on a bare MFMA
// loop, measured beside the step so that its roofline fractions can be read against a measured
// ceiling as well as the nominal one.  Not part of the optimizer path.
#include "ng_internal.h"

namespace ng {

#define NG_AS1 __attribute__((address_space(1)))

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

// Both streaming kernels give every workgroup contiguous chunks of kChunk 16-byte vectors (64 KB),
// grid-stride over the chunks, four vectors in flight per lane, nontemporal accesses (the step's
// streaming kernels move the history and the moments the same way).  Measured against workgroups that
// interleave single vectors: copy 5.3-5.7 instead of 4.6 TB/s, read 7.0 instead of 6.0 TB/s.
constexpr int kChunk = 4096;

__global__ __launch_bounds__(256) void k_mb_copy(const NG_AS1 u32x4_t* __restrict__ src,
                                                 NG_AS1 u32x4_t* __restrict__ dst, long long n16) {
    for (long long c0 = (long long)blockIdx.x * kChunk; c0 < n16; c0 += (long long)gridDim.x * kChunk) {
        const long long c1 = c0 + kChunk < n16 ? c0 + kChunk : n16;
        long long i = c0 + threadIdx.x;
        for (; i + 3 * 256 < c1; i += 4 * 256) {
            u32x4_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
            for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * 256);
        }
        for (; i < c1; i += 256) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
    }
}

// read-only pass: every lane folds what it reads into one word, stored only if it is a value that a
// buffer of finite floats cannot produce (keeps the loads alive without a store stream)
__global__ __launch_bounds__(256) void k_mb_read(const NG_AS1 u32x4_t* __restrict__ src, long long n16,
                                                 unsigned int* sink) {
    unsigned int acc = 0;
    for (long long c0 = (long long)blockIdx.x * kChunk; c0 < n16; c0 += (long long)gridDim.x * kChunk) {
        const long long c1 = c0 + kChunk < n16 ? c0 + kChunk : n16;
        long long i = c0 + threadIdx.x;
        for (; i + 3 * 256 < c1; i += 4 * 256) {
            u32x4_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        }
        for (; i < c1; i += 256) {
            const u32x4_t v = __builtin_nontemporal_load(src + i);
            acc ^= v.x ^ v.y ^ v.z ^ v.w;
        }
    }
    if (acc == 0x7fc12345u) *sink = acc;
}

// NACC independent 32x32x16 bf16 MFMA accumulators per wavefront, operands in registers, no memory
// traffic: the rate the matrix cores sustain at the clock the chip settles on under that load.
// RANDOM: the operands are pseudo-random values of magnitude 1..2 with random signs and mantissas, two
// sets in alternation (every MFMA sees operands that differ from the previous one's): the switching
// activity of real data, which is what sets the clock.  Otherwise small integers that never change.
template <int NACC, bool RANDOM>
__global__ __launch_bounds__(256) void k_mb_mfma_bf16(int iters, float* sink) {
    floatx16 acc[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    bf16x8_t a[2], b[2];
    unsigned int h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (RANDOM) {
                h = h * 1664525u + 1013904223u;
                const unsigned short ua = (unsigned short)(((h >> 16) & 0x807fu) | 0x3f80u);   // +-1.mmmmmmm
                h = h * 1664525u + 1013904223u;
                const unsigned short ub = (unsigned short)(((h >> 16) & 0x807fu) | 0x3f80u);
                a[q][e] = __builtin_bit_cast(__bf16, ua);
                b[q][e] = __builtin_bit_cast(__bf16, ub);
            } else {
                a[q][e] = (__bf16)(float)((threadIdx.x + e) & 3);
                b[q][e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
            }
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NACC; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j & 1], b[(j >> 1) & 1], acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NACC; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    if (s == -1.2345e-30f) *sink = s;   // never true in practice; keeps the accumulators alive
}

hipError_t launch_mb_copy(const void* src, void* dst, size_t bytes, hipStream_t stream) {
    const long long n16 = (long long)(bytes / 16);
    hipLaunchKernelGGL(k_mb_copy, dim3(256 * 16), dim3(256), 0, stream, (const NG_AS1 u32x4_t*)src,
                       (NG_AS1 u32x4_t*)dst, n16);
    return hipGetLastError();
}

hipError_t launch_mb_read(const void* src, size_t bytes, void* sink, hipStream_t stream) {
    const long long n16 = (long long)(bytes / 16);
    hipLaunchKernelGGL(k_mb_read, dim3(256 * 16), dim3(256), 0, stream, (const NG_AS1 u32x4_t*)src, n16,
                       (unsigned int*)sink);
    return hipGetLastError();
}

// flops of one launch are returned through *flops
hipError_t launch_mb_mfma(int iters, int waves_per_simd, bool random_operands, void* sink, double* flops,
                          hipStream_t stream) {
    // 256 compute units x 4 SIMDs; a workgroup of 4 wavefronts puts one on each SIMD of a unit
    const int groups = 256 * waves_per_simd * 4;   // four workgroups deep per unit and wave slot: keeps every unit busy to the end
    constexpr int kAcc = 8;
    if (random_operands)
        hipLaunchKernelGGL((k_mb_mfma_bf16<kAcc, true>), dim3(groups), dim3(256), 0, stream, iters, (float*)sink);
    else
        hipLaunchKernelGGL((k_mb_mfma_bf16<kAcc, false>), dim3(groups), dim3(256), 0, stream, iters, (float*)sink);
    *flops = (double)groups * 4.0 * iters * kAcc * 2.0 * 32 * 32 * 16;
    return hipGetLastError();
}

}  // namespace ng
