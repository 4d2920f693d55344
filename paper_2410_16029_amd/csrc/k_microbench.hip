// Micro-benchmarks behind ng_microbench: what this GPU sustains on a plain stream and on a bare MFMA
// loop, measured beside the step so that its roofline fractions can be read against a measured
// ceiling as well as the nominal one.  Not part of the optimizer path.
#include "ng_internal.h"

namespace ng {

#define NG_AS1 __attribute__((address_space(1)))

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

// dst[i] = src[i], 16 bytes per lane, four loads in flight per lane; nontemporal both ways
// (the step's streaming kernels move the history and the moments the same way)
__global__ __launch_bounds__(256) void k_mb_copy(const NG_AS1 u32x4_t* __restrict__ src,
                                                 NG_AS1 u32x4_t* __restrict__ dst, long long n16) {
    const long long stride = (long long)gridDim.x * 256;
    long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        u32x4_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
    for (; i < n16; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// read-only pass: every lane folds what it reads into one word, stored only if it is a value that a
// buffer of finite floats cannot produce (keeps the loads alive without a store stream)
__global__ __launch_bounds__(256) void k_mb_read(const NG_AS1 u32x4_t* __restrict__ src, long long n16,
                                                 unsigned int* sink) {
    const long long stride = (long long)gridDim.x * 256;
    long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    unsigned int acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        u32x4_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n16; i += stride) {
        const u32x4_t v = __builtin_nontemporal_load(src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x7fc12345u) *sink = acc;
}

// NACC independent 32x32x16 bf16 MFMA accumulators per wavefront, operands in registers, no memory
// traffic: the rate the matrix cores sustain at the clock the chip settles on under that load.
template <int NACC>
__global__ __launch_bounds__(256) void k_mb_mfma_bf16(int iters, float* sink) {
    floatx16 acc[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    bf16x8_t a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
        b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NACC; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    if (s == -1.f) *sink = s;   // sums of non-negative products: never true
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
hipError_t launch_mb_mfma(int iters, int waves_per_simd, void* sink, double* flops, hipStream_t stream) {
    // 256 compute units x 4 SIMDs; a workgroup of 4 wavefronts puts one on each SIMD of a unit
    const int groups = 256 * waves_per_simd * 4;   // four workgroups deep per unit and wave slot: keeps every unit busy to the end
    constexpr int kAcc = 8;
    hipLaunchKernelGGL(k_mb_mfma_bf16<kAcc>, dim3(groups), dim3(256), 0, stream, iters, (float*)sink);
    *flops = (double)groups * 4.0 * iters * kAcc * 2.0 * 32 * 32 * 16;
    return hipGetLastError();
}

}  // namespace ng
