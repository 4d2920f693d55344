// HBM-bound phases of the Natural GaLore step (paper Sec. 2.4 and the Adam
// equations of Sec. 2.2), plus small utility kernels.
//
//   k_gram_row        y_j = <R, H_j>_F for all s ring slots (the new row of the s x s Gram matrix)
//   k_solve           (lambda I + K/s) w = e_head by Cholesky in fp64, one wavefront per matrix
//   k_transform_adam  g~ = sum_j w_j H_j, Adam moments, update direction N
//
// The transform is evaluated as H_mat (lambda I + K/s)^{-1} e_head.  This equals
// the section's g/lambda - U z/lambda^2 (push U through the inverse: the current
// gradient is slot `head` of the stack) but has no cancellation, which the printed
// form has at about log10(||R||^2 / (s lambda)) digits.
#include "ng_internal.h"

namespace ng {

// Pointers read out of the per-matrix table are cast to the global address space so that the
// streaming kernels use global_load / global_store instead of flat accesses.
#define NG_AS1 __attribute__((address_space(1)))
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

// ------------------------------------------------------------------ helpers
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two floats -> two bf16 (round to nearest even) in one v_cvt_pk_bf16_f32; a in the low half
__device__ __forceinline__ unsigned int pack_bf16x2(float a, float b) {
    const f32x2_t f = {a, b};
    bf16x2_t hv = __builtin_convertvector(f, bf16x2_t);
    return *reinterpret_cast<unsigned int*>(&hv);
}
__device__ __forceinline__ unsigned short f32_to_bf16_rne(float x) { return (unsigned short)(pack_bf16x2(x, 0.f) & 0xffffu); }

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// ------------------------------------------------------------------ per-step table upload
__global__ void k_upload_dyn(MatDyn* table, DynChunk chunk, int first, int n, const MatDev* mats) {
    int i = threadIdx.x;
    if (i >= n) return;
    table[first + i] = chunk.e[i];
    if (mats == nullptr) return;
    // the zero-padded copy of the last gradient row's final partial 8-column chunk (bf16 projection)
    const MatDev& md = mats[first + i];
    const int nf = md.n & 7;
    if (md.side == NG_SIDE_RIGHT || nf == 0 || md.tail8_off < 0 || chunk.e[i].g == nullptr) return;
    const bf16_t* last = (const bf16_t*)chunk.e[i].g + (long long)(md.m - 1) * md.ld_g + (md.n - nf);
    bf16_t* tail8 = step_scratch<bf16_t>(table, md.tail8_off);
    for (int x = 0; x < 8; ++x) tail8[x] = x < nf ? last[x] : (bf16_t)0;
}

hipError_t launch_upload_dyn(MatDyn* table, const DynChunk& chunk, int first, int n, const MatDev* mats,
                             hipStream_t stream) {
    hipLaunchKernelGGL(k_upload_dyn, dim3(1), dim3(128), 0, stream, table, chunk, first, n, mats);
    return hipGetLastError();
}

// ------------------------------------------------------------------ zero fill
__global__ void k_fill_zero(uint4* p16, size_t n16, unsigned int* tail, int ntail) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    uint4 z = make_uint4(0, 0, 0, 0);
    for (; i < n16; i += stride) p16[i] = z;
    if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0u;
}

hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t stream) {
    if (bytes == 0) return hipSuccess;
    size_t n16 = bytes / 16;
    int ntail = (int)((bytes % 16) / 4);
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)blocks), dim3(256), 0, stream, (uint4*)ptr, n16,
                       (unsigned int*)((char*)ptr + n16 * 16), ntail);
    return hipGetLastError();
}

// History ring and Gram block (K, weights) of every matrix in one launch.  h_elem_bytes: 4 or 2; both
// buffers are whole multiples of 256 bytes (the sizes the library reports for them).
__global__ __launch_bounds__(256) void k_clear_history(const MatDev* __restrict__ mats, int s, int h_elem_bytes,
                                                       unsigned long long k_bytes) {
    const MatDev& md = mats[blockIdx.y];
    const unsigned long long hb =
        ((unsigned long long)md.slot_elems * (unsigned)h_elem_bytes * (unsigned)(s > 0 ? s : 1) + 255ull) & ~255ull;
    const uint4 z = make_uint4(0, 0, 0, 0);
    uint4* __restrict__ h = reinterpret_cast<uint4*>(md.H);
    const unsigned long long n16 = hb / 16, stride = (unsigned long long)gridDim.x * 256;
    for (unsigned long long i = (unsigned long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) h[i] = z;
    if (blockIdx.x == 0) {
        uint4* __restrict__ k = reinterpret_cast<uint4*>(md.K);
        for (unsigned long long i = threadIdx.x; i < k_bytes / 16; i += 256) k[i] = z;
    }
}

hipError_t launch_clear_history(const MatDev* mats, int n_mats, int s, int h_elem_bytes, size_t k_bytes,
                                hipStream_t stream) {
    if (n_mats <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_clear_history, dim3(128, n_mats), dim3(256), 0, stream, mats, s, h_elem_bytes,
                       (unsigned long long)k_bytes);
    return hipGetLastError();
}

// ------------------------------------------------------------------ Gram row
// One workgroup = one contiguous part of the flat r*ldn range of one matrix.
// Products and 4-term sums in fp32, running sums in fp64, fixed reduction order.
// HB: the slots hold bf16 (8 elements per 16-byte vector) instead of float (4 per vector).
template <int SMAX, bool HB>
__global__ __launch_bounds__(256) void k_gram_row(const MatDev* __restrict__ mats,
                                                  const MatDyn* __restrict__ dyn,
                                                  const TileRef* __restrict__ chunks, int s, int row_override) {
    const TileRef c = chunks[blockIdx.x];
    const MatDev& md = mats[c.mat];
    const int head = row_override >= 0 ? row_override : dyn[c.mat].head;
    const long long totalv = md.slot_elems >> (HB ? 3 : 2);   // 16-byte vectors from one slot to the next
    const FlatState fs = flat_state(md.r, md.ldn, md.pw, HB ? 8 : 4);   // positions q -> vectors of a slot
    const long long span = (long long)md.dot_iters * 256;
    const long long q0 = (long long)c.ti * span;
    long long q1 = q0 + span;
    if (q1 > (long long)fs.count) q1 = fs.count;
    const NG_AS1 u32x4_t* __restrict__ H = (const NG_AS1 u32x4_t*)md.H;
    const NG_AS1 u32x4_t* __restrict__ R = H + (long long)head * totalv;

    double acc[SMAX];
#pragma unroll
    for (int j = 0; j < SMAX; ++j) acc[j] = 0.0;

    if (!HB && (md.dot_iters & 3) == 0) {
        // Large float slots (the host makes a workgroup's span a whole number of 1024-vector passes):
        // four positions per thread and pass (q, q + 256, q + 512, q + 768), one slot at a time -- the
        // four loads of a slot are issued together and the compiler is kept from mixing the slots.
        // A workgroup streaming 16 KB of one slot after the other reads at 6.96 TB/s; with the loads
        // of all slots for one position in flight at once it was 6.74.  The order of the additions
        // into acc[j] is that of q, as in the loop below.
        const u32x4_t zero4 = {0u, 0u, 0u, 0u};
        for (long long q = q0 + threadIdx.x; q < q1; q += 1024) {
            u32x4_t rv[4];
            long long qq[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool ok = q + 256 * u < q1;
                qq[u] = fs.at((unsigned)(ok ? q + 256 * u : q));   // a position past the end re-reads q against a zero R
                rv[u] = ok ? R[qq[u]] : zero4;
            }
#pragma unroll
            for (int j = 0; j < SMAX; ++j) {
                if (j < s) {
                    u32x4_t hv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) hv[u] = __builtin_nontemporal_load(H + ((long long)j * totalv + qq[u]));
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        float p = __uint_as_float(hv[u].x) * __uint_as_float(rv[u].x);
                        p = fmaf(__uint_as_float(hv[u].y), __uint_as_float(rv[u].y), p);
                        p = fmaf(__uint_as_float(hv[u].z), __uint_as_float(rv[u].z), p);
                        p = fmaf(__uint_as_float(hv[u].w), __uint_as_float(rv[u].w), p);
                        acc[j] += (double)p;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
        // Small slots (a workgroup has one or a few positions per thread: latency, not bandwidth) and
        // bf16 slots (8 elements per vector; R is widened once per position, which the slot-at-a-time
        // order would do once per slot: 1.36 against 1.25 ms): all slots of one position together.
        // Branch-free: a slot index beyond s is clamped to s-1 (its sum is never written out), so
        // all SMAX loads of one position are issued back to back.
        long long slot_off[SMAX];
#pragma unroll
        for (int j = 0; j < SMAX; ++j) slot_off[j] = (long long)(j < s ? j : s - 1) * totalv;
        for (long long q = q0 + threadIdx.x; q < q1; q += 256) {
            const long long a = fs.at((unsigned)q);
            const u32x4_t rv = R[a];
            u32x4_t hv[SMAX];
#pragma unroll
            for (int j = 0; j < SMAX; ++j) hv[j] = __builtin_nontemporal_load(H + (slot_off[j] + a));
            if (HB) {
                float rf[8];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    rf[2 * d] = __uint_as_float(rv[d] << 16);
                    rf[2 * d + 1] = __uint_as_float(rv[d] & 0xffff0000u);
                }
#pragma unroll
                for (int j = 0; j < SMAX; ++j) {
                    float p = 0.f;
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        p = fmaf(__uint_as_float(hv[j][d] << 16), rf[2 * d], p);
                        p = fmaf(__uint_as_float(hv[j][d] & 0xffff0000u), rf[2 * d + 1], p);
                    }
                    acc[j] += (double)p;
                }
            } else {
#pragma unroll
                for (int j = 0; j < SMAX; ++j) {
                    float p = __uint_as_float(hv[j].x) * __uint_as_float(rv.x);
                    p = fmaf(__uint_as_float(hv[j].y), __uint_as_float(rv.y), p);
                    p = fmaf(__uint_as_float(hv[j].z), __uint_as_float(rv.z), p);
                    p = fmaf(__uint_as_float(hv[j].w), __uint_as_float(rv.w), p);
                    acc[j] += (double)p;
                }
            }
        }
    }

    __shared__ double red[4][SMAX];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int j = 0; j < SMAX; ++j) {
        double v = wave_sum(acc[j]);
        if (lane == 0) red[wv][j] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < s) {
        double v = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
        ((NG_AS1 double*)step_scratch<double>(dyn, md.dot_parts_off))[(long long)c.ti * s + threadIdx.x] = v;
    }
}

hipError_t launch_gram_row(const MatDev* mats, const MatDyn* dyn, const TileRef* chunks, int n_chunks, int s,
                           int hist_bf16, int row_override, hipStream_t stream) {
    if (n_chunks == 0) return hipSuccess;
    dim3 g(n_chunks), b(256);
#define NG_GRAM_CASE(S)                                                                          \
    do {                                                                                         \
        if (hist_bf16) hipLaunchKernelGGL((k_gram_row<S, true>), g, b, 0, stream, mats, dyn, chunks, s, row_override);  \
        else hipLaunchKernelGGL((k_gram_row<S, false>), g, b, 0, stream, mats, dyn, chunks, s, row_override);           \
    } while (0)
    if (s <= 1) NG_GRAM_CASE(1);
    else if (s <= 2) NG_GRAM_CASE(2);
    else if (s <= 3) NG_GRAM_CASE(3);
    else if (s <= 4) NG_GRAM_CASE(4);
    else if (s <= 6) NG_GRAM_CASE(6);
    else if (s <= 8) NG_GRAM_CASE(8);
    else if (s <= 12) NG_GRAM_CASE(12);
    else if (s <= 16) NG_GRAM_CASE(16);
    else if (s <= 24) NG_GRAM_CASE(24);
    else if (s <= 32) NG_GRAM_CASE(32);
    else if (s <= 48) NG_GRAM_CASE(48);
    else NG_GRAM_CASE(64);
#undef NG_GRAM_CASE
    return hipGetLastError();
}

// ------------------------------------------------------------------ s x s solve
// One wavefront per matrix.  Sums the partial dot products in a fixed order,
// writes row/column `head` of K, factors A = lambda I + K/s (Cholesky, fp64, in
// LDS) and solves A w = e_head.  A non-positive or non-finite pivot sets bit 0
// of *status; a non-finite w sets bit 1.
__global__ __launch_bounds__(64) void k_solve(const MatDev* __restrict__ mats, const MatDyn* __restrict__ dyn,
                                              int first, StepScalars sc, int row_override, int* status) {
    __shared__ double A[kMaxS][kMaxS + 1];
    __shared__ double bc[kMaxS];
    const MatDev& md = mats[first + blockIdx.x];
    const int s = sc.s;
    const int head = row_override >= 0 ? row_override : dyn[first + blockIdx.x].head;
    const int i = threadIdx.x;

    // old Gram matrix into LDS, then overwrite row and column `head` with the new dots
    if (i < s)
        for (int j = 0; j < s; ++j) A[i][j] = md.K[(long long)i * s + j];
    __syncthreads();
    // partial sums: lane (sub, j) adds parts sub, sub+nsub, ... in order; the nsub sub-sums of a
    // slot are then added in order (a fixed order: the result does not depend on timing)
    {
        const int nsub = 64 / s;
        const int j = i % s, sub = i / s;
        double v = 0.0;
        if (sub < nsub) {
            // eight loads in flight, added in the order of p
            const int np = md.dot_nparts;
            const double* __restrict__ parts = step_scratch<double>(dyn, md.dot_parts_off) + j;
            for (int p = sub; p < np; p += 8 * nsub) {
                double x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int pu = p + u * nsub;
                    x[u] = pu < np ? parts[(long long)pu * s] : 0.0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) v += x[u];
            }
        }
        bc[i] = v;
    }
    __syncthreads();
    if (i < s) {
        const int nsub = 64 / s;
        double v = 0.0;
        for (int q = 0; q < nsub; ++q) v += bc[q * s + i];
        md.K[(long long)head * s + i] = v;
        md.K[(long long)i * s + head] = v;
        A[head][i] = v;
        A[i][head] = v;
    }
    if (row_override >= 0) return;      // only the Gram matrix is rebuilt (history carry-over)
    __syncthreads();
    const double lam = (double)sc.lambda;
    // normaliser of the empirical Fisher: 1/s, or 1/(valid slots after this push) while the ring fills
    const double inv_s = 1.0 / (double)(sc.norm_count ? dyn[first + blockIdx.x].count : s);
    if (i < s)
        for (int j = 0; j < s; ++j) A[i][j] = A[i][j] * inv_s + (i == j ? lam : 0.0);
    __syncthreads();

    bool bad = false;
    for (int k = 0; k < s; ++k) {
        double d = A[k][k];
        if (!(d > 0.0) || !(d < 1.0e300)) {
            bad = true;
            d = 1.0;
        }
        d = sqrt(d);
        __syncthreads();
        if (i == k) A[k][k] = d;
        if (i > k && i < s) A[i][k] = A[i][k] / d;
        __syncthreads();
        if (i > k && i < s) {
            const double lik = A[i][k];
            for (int j = k + 1; j <= i; ++j) A[i][j] -= lik * A[j][k];
        }
        __syncthreads();
    }

    // forward: L y = e_head
    double b = (i == head) ? 1.0 : 0.0;
    for (int k = 0; k < s; ++k) {
        if (i == k) bc[k] = b / A[k][k];
        __syncthreads();
        if (i > k && i < s) b -= A[i][k] * bc[k];
        __syncthreads();
    }
    // backward: L^T w = y
    double y = (i < s) ? bc[i] : 0.0;
    __syncthreads();
    for (int k = s - 1; k >= 0; --k) {
        if (i == k) bc[k] = y / A[k][k];
        __syncthreads();
        if (i < k) y -= A[k][i] * bc[k];
        __syncthreads();
    }
    if (i < s) {
        const double w = bc[i];
        if (!(fabs(w) < 1.0e300)) bad = true;
        md.w64[i] = w;
        md.w32[i] = (float)w;
    }
    if (bad) atomicOr(status, 1);
}

hipError_t launch_solve(const MatDev* mats, const MatDyn* dyn, int first, int n_mats, StepScalars sc,
                        int row_override, int* status, hipStream_t stream) {
    hipLaunchKernelGGL(k_solve, dim3(n_mats), dim3(64), 0, stream, mats, dyn, first, sc, row_override, status);
    return hipGetLastError();
}

// ------------------------------------------------------------------ transform + Adam
//   g~ = sum_j w_j H_j          (second pass over the ring; w from k_solve)
//   M <- b1 M + (1-b1) g~ ; V <- b2 V + (1-b2) g~^2
//   N  = (M * bc1) / (sqrt(V) * bc2 + eps)         standard
//      = M / sqrt(V + eps)                          as printed
// N is stored either as float [r][ldn] or as bf16 [r/8][ldn][8] (eight
// consecutive rows of one column adjacent: the k-packing the update GEMM's MFMA
// operand wants, so that kernel needs no transpose).
// Four consecutive history elements of one row: a float4, or 4 bf16 (8 bytes) widened to float.
// `slot` is uniform over the workgroup and `off` a 32-bit byte offset, so the load takes its base
// from scalar registers and needs one address register per row (the host checks that a slot is
// below 2 GiB).
template <bool HB>
__device__ __forceinline__ f32x4_t load_hist4(const NG_AS1 unsigned char* slot, unsigned off) {
    if (HB) {
        const u32x2_t v = __builtin_nontemporal_load((const NG_AS1 u32x2_t*)(slot + off));
        f32x4_t o;
        o.x = __uint_as_float(v.x << 16);
        o.y = __uint_as_float(v.x & 0xffff0000u);
        o.z = __uint_as_float(v.y << 16);
        o.w = __uint_as_float(v.y & 0xffff0000u);
        return o;
    }
    return __builtin_nontemporal_load((const NG_AS1 f32x4_t*)(slot + off));
}

// A lane owns a 4 (rows) x 4 (columns) patch; the two lanes of a pair (even: rows 0..3, odd: rows
// 4..7 of an 8-row band) share the columns, so together they produce the 16-byte octets of N.  The
// small patch keeps the register count low and the occupancy high, which is what feeds HBM here.
// Wavefront = 8 rows x 128 columns, workgroup = 32 rows x 128 columns.
template <bool BF16_N, bool HB>
__global__ __launch_bounds__(256) void k_transform_adam(const MatDev* __restrict__ mats,
                                                        const MatDyn* __restrict__ dyn,
                                                        const TileRef* __restrict__ patches, StepScalars sc,
                                                        int* status) {
    constexpr int RT = 4;
    const TileRef pr = patches[blockIdx.x];
    const MatDev& md = mats[pr.mat];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
    const int band0 = pr.ti * 32 + wv * 8;                             // first row of the 8-row band
    const int half = lane & 1;
    const int row0 = band0 + RT * half;
    const int col0 = pr.tj * kAdamPatchCols + (lane >> 1) * 4;
    const int ldn = md.ldn, r = md.r;
    if (band0 >= r || col0 >= ldn) return;
    // rows of this lane inside the matrix (0 for the odd lane of a band that ends early)
    const int nrow = r - row0 < 0 ? 0 : (r - row0 < RT ? r - row0 : RT);
    // Branch-free loads: a row beyond nrow re-reads the band's last valid row and its result is dropped.
    // Element offsets of this thread's row segments inside a slot / inside M, V (32-bit).
    unsigned eoff[RT];
    const StatePanel sp = state_panel(r, md.pw, pr.tj * kAdamPatchCols);   // the same for the whole workgroup
#pragma unroll
    for (int e = 0; e < RT; ++e) {
        const int row = row0 + e < r ? row0 + e : r - 1;
        eoff[e] = sp.at(row, col0);
    }
    constexpr unsigned HS = HB ? 2u : 4u;   // bytes per history element

    f32x4_t g[RT];
#pragma unroll
    for (int e = 0; e < RT; ++e) g[e] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

    const int s = sc.s;
    const NG_AS1 unsigned char* __restrict__ Hbase = (const NG_AS1 unsigned char*)md.H;
    const long long slot_bytes = md.slot_elems * (long long)HS;
    if (sc.use_fisher) {
        const NG_AS1 float* __restrict__ w = (const NG_AS1 float*)md.w32;
#pragma unroll 2   // (the loads of two slots in flight: 3.69 -> 3.67 ms)
        for (int j = 0; j < s; ++j) {
            const float wj = w[j];
            const NG_AS1 unsigned char* slot = Hbase + (long long)j * slot_bytes;
            f32x4_t h[RT];
#pragma unroll
            for (int e = 0; e < RT; ++e) h[e] = load_hist4<HB>(slot, eoff[e] * HS);
#pragma unroll
            for (int e = 0; e < RT; ++e) {
                g[e].x = fmaf(wj, h[e].x, g[e].x);
                g[e].y = fmaf(wj, h[e].y, g[e].y);
                g[e].z = fmaf(wj, h[e].z, g[e].z);
                g[e].w = fmaf(wj, h[e].w, g[e].w);
            }
        }
    } else {
        // the single scratch slot holds R
#pragma unroll
        for (int e = 0; e < RT; ++e) g[e] = load_hist4<HB>(Hbase, eoff[e] * HS);
    }

    const float b1 = sc.beta1, b2 = sc.beta2, ob1 = 1.0f - sc.beta1, ob2 = 1.0f - sc.beta2;
    const float bc1 = dyn[pr.mat].bc1, bc2 = dyn[pr.mat].bc2;
    NG_AS1 unsigned char* Mb = (NG_AS1 unsigned char*)md.M;
    NG_AS1 unsigned char* Vb = (NG_AS1 unsigned char*)md.V;
    // two rows at a time (the moments of all four rows at once would cost occupancy)
    unsigned int lo[4], hi[4];     // bf16 N, per column: rows (0,1) and (2,3) of this lane's four rows
    bool bad = false;
#pragma unroll
    for (int pr2 = 0; pr2 < 2; ++pr2) {
        f32x4_t mv[2], vv[2], nv[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            mv[u] = __builtin_nontemporal_load((const NG_AS1 f32x4_t*)(Mb + eoff[2 * pr2 + u] * 4u));
            vv[u] = __builtin_nontemporal_load((const NG_AS1 f32x4_t*)(Vb + eoff[2 * pr2 + u] * 4u));
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int e = 2 * pr2 + u;
            f32x4_t m = mv[u], v = vv[u];
            const f32x4_t ge = g[e];
            m.x = fmaf(b1, m.x, ob1 * ge.x);
            m.y = fmaf(b1, m.y, ob1 * ge.y);
            m.z = fmaf(b1, m.z, ob1 * ge.z);
            m.w = fmaf(b1, m.w, ob1 * ge.w);
            v.x = fmaf(b2, v.x, ob2 * ge.x * ge.x);
            v.y = fmaf(b2, v.y, ob2 * ge.y * ge.y);
            v.z = fmaf(b2, v.z, ob2 * ge.z * ge.z);
            v.w = fmaf(b2, v.w, ob2 * ge.w * ge.w);
            f32x4_t o;
            if (sc.adam_mode == NG_ADAM_STANDARD) {
                o.x = (m.x * bc1) / (sqrtf(v.x) * bc2 + sc.eps);
                o.y = (m.y * bc1) / (sqrtf(v.y) * bc2 + sc.eps);
                o.z = (m.z * bc1) / (sqrtf(v.z) * bc2 + sc.eps);
                o.w = (m.w * bc1) / (sqrtf(v.w) * bc2 + sc.eps);
            } else {
                o.x = m.x / sqrtf(v.x + sc.eps);
                o.y = m.y / sqrtf(v.y + sc.eps);
                o.z = m.z / sqrtf(v.z + sc.eps);
                o.w = m.w / sqrtf(v.w + sc.eps);
            }
            const bool live = e < nrow;
            if (live) {
                __builtin_nontemporal_store(m, (NG_AS1 f32x4_t*)(Mb + eoff[e] * 4u));
                __builtin_nontemporal_store(v, (NG_AS1 f32x4_t*)(Vb + eoff[e] * 4u));
            }
            bad |= live && (!(fabsf(o.x) <= 3.0e38f) | !(fabsf(o.y) <= 3.0e38f) | !(fabsf(o.z) <= 3.0e38f) |
                            !(fabsf(o.w) <= 3.0e38f));
            nv[u].x = live ? o.x : 0.f;
            nv[u].y = live ? o.y : 0.f;
            nv[u].z = live ? o.z : 0.f;
            nv[u].w = live ? o.w : 0.f;
            if (!BF16_N && live) *(NG_AS1 f32x4_t*)((NG_AS1 unsigned char*)md.N + eoff[e] * 4u) = nv[u];
        }
        if (BF16_N) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const unsigned int pk = pack_bf16x2(nv[0][c], nv[1][c]);
                if (pr2 == 0) lo[c] = pk;
                else hi[c] = pk;
            }
        }
    }

    if (BF16_N) {
        // [octet][col][8]: this lane holds rows 4 half .. 4 half + 3 of the band's octet for its 4
        // columns, i.e. 8 of each octet's 16 bytes.  The pair swaps two columns so that each lane
        // stores two whole octets (32 contiguous bytes): the even lane columns 0 and 1, the odd
        // lane columns 2 and 3.
        // what the partner needs from this lane: even lane gives columns 2, 3; odd lane gives 0, 1
        const unsigned int s0 = half ? lo[0] : lo[2], s1 = half ? hi[0] : hi[2];
        const unsigned int s2 = half ? lo[1] : lo[3], s3 = half ? hi[1] : hi[3];
        const unsigned int p0 = (unsigned int)__builtin_amdgcn_mov_dpp((int)s0, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
        const unsigned int p1 = (unsigned int)__builtin_amdgcn_mov_dpp((int)s1, 0xB1, 0xf, 0xf, false);
        const unsigned int p2 = (unsigned int)__builtin_amdgcn_mov_dpp((int)s2, 0xB1, 0xf, 0xf, false);
        const unsigned int p3 = (unsigned int)__builtin_amdgcn_mov_dpp((int)s3, 0xB1, 0xf, 0xf, false);
        // columns kept by this lane: even 0, 1; odd 2, 3.  Octet = rows 0..3 (even lane's) then 4..7 (odd's).
        u32x4_t oa, ob;
        if (!half) {
            oa = (u32x4_t){lo[0], hi[0], p0, p1};
            ob = (u32x4_t){lo[1], hi[1], p2, p3};
        } else {
            oa = (u32x4_t){p0, p1, lo[2], hi[2]};
            ob = (u32x4_t){p2, p3, lo[3], hi[3]};
        }
        NG_AS1 u32x4_t* Np =
            (NG_AS1 u32x4_t*)((NG_AS1 bf16_t*)md.N + ((long long)(band0 >> 3) * ldn + col0 + 2 * half) * 8);
        Np[0] = oa;   // (a nontemporal store is slower here: measured)
        Np[1] = ob;
    }
    if (bad) atomicOr(status, 2);
}

hipError_t launch_transform_adam(const MatDev* mats, const MatDyn* dyn, const TileRef* patches, int n_patches,
                                 StepScalars sc, int grad_dtype, int* status, hipStream_t stream) {
    if (n_patches == 0) return hipSuccess;
    if (grad_dtype == NG_BF16 && sc.hist_bf16)
        hipLaunchKernelGGL((k_transform_adam<true, true>), dim3(n_patches), dim3(256), 0, stream, mats, dyn, patches,
                           sc, status);
    else if (grad_dtype == NG_BF16)
        hipLaunchKernelGGL((k_transform_adam<true, false>), dim3(n_patches), dim3(256), 0, stream, mats, dyn, patches,
                           sc, status);
    else
        hipLaunchKernelGGL((k_transform_adam<false, false>), dim3(n_patches), dim3(256), 0, stream, mats, dyn, patches,
                           sc, status);
    return hipGetLastError();
}

// ------------------------------------------------------------------ bf16 copies of P
// Both copies are k-blocked, [k / 32][rows][32] with the contraction index k split into blocks of 32:
//   Pb  (rows = i < m,   k = rho < ldr): Pb[((rho / 32) * m + i) * 32 + rho % 32] = bf16(P[i][rho]), zero for rho >= r
//   PbT (rows = rho < r, k = i < ldk):   PbT[((i / 32) * r + rho) * 32 + i % 32]  = bf16(P[i][rho]), zero for i >= m
// One workgroup converts a 32 x 32 tile through LDS: both writes are 2 KB of consecutive memory.
__global__ __launch_bounds__(256) void k_make_bf16_copies(const MatDev* __restrict__ mats) {
    __shared__ float tile[32][33];
    const MatDev& md = mats[blockIdx.z];
    const int i0 = blockIdx.y * 32, r0 = blockIdx.x * 32;
    if (i0 >= md.ldk || r0 >= md.ldr) return;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int yy = ty; yy < 32; yy += 8) {
        const int i = i0 + yy, rho = r0 + tx;
        float v = 0.f;
        if (i < md.m && rho < md.r) v = md.P[(long long)i * md.r + rho];
        tile[yy][tx] = v;
        if (i < md.m) md.Pb[((long long)(r0 >> 5) * md.m + i) * 32 + tx] = f32_to_bf16_rne(v);
    }
    __syncthreads();
    for (int yy = ty; yy < 32; yy += 8) {
        const int rho = r0 + yy;
        if (rho < md.r) md.PbT[((long long)(i0 >> 5) * md.r + rho) * 32 + tx] = f32_to_bf16_rne(tile[tx][yy]);
    }
}

// ------------------------------------------------------------------ history carry-over helpers
__global__ __launch_bounds__(256) void k_save_projector(const MatDev* __restrict__ mats) {
    const MatDev& md = mats[blockIdx.y];
    const long long total = (long long)md.m * md.r;
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < total; q += (long long)gridDim.x * 256)
        md.Yc[q] = md.P[q];
}

hipError_t launch_save_projector(const MatDev* mats, int n_mats, hipStream_t stream) {
    hipLaunchKernelGGL(k_save_projector, dim3(256, n_mats), dim3(256), 0, stream, mats);
    return hipGetLastError();
}

// H[slot] <- carry (float -> the slot's type)
template <bool HB>
__global__ __launch_bounds__(256) void k_carry_store(const MatDev* __restrict__ mats, int slot) {
    const MatDev& md = mats[blockIdx.y];
    const long long total = md.slot_elems;
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < total; q += (long long)gridDim.x * 256) {
        const float v = md.carry[q];
        if (HB) ((bf16_t*)md.H)[(long long)slot * total + q] = f32_to_bf16_rne(v);
        else md.H[(long long)slot * total + q] = v;
    }
}

hipError_t launch_carry_store(const MatDev* mats, int n_mats, int slot, int hist_bf16, hipStream_t stream) {
    if (hist_bf16) hipLaunchKernelGGL(k_carry_store<true>, dim3(512, n_mats), dim3(256), 0, stream, mats, slot);
    else hipLaunchKernelGGL(k_carry_store<false>, dim3(512, n_mats), dim3(256), 0, stream, mats, slot);
    return hipGetLastError();
}

hipError_t launch_make_bf16_copies(const MatDev* mats, int n_mats, int max_m, int max_r, hipStream_t stream) {
    dim3 g((max_r + 31) / 32, (max_m + 8 + 31) / 32, n_mats);
    hipLaunchKernelGGL(k_make_bf16_copies, g, dim3(256), 0, stream, mats);
    return hipGetLastError();
}

}  // namespace ng
