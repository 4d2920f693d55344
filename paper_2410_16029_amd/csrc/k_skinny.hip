// Projection and update of fp32 gradients / weights for ranks far below an MFMA tile (r <= 16, left
// side): the fine-tuning regime of the paper's Sec. 3.2 (ranks 4 and 8).  With so few rows of R the
// two contractions are pure streams over the gradient and the weight (2r flop per element), so they
// run on the vector ALU with the gradient / weight read exactly once, coalesced, and nothing padded
// up to a tile (the fp32 MFMA GEMM spends a 64-row tile on them).  bf16 layer sets keep the bf16 MFMA
// kernels, which are bandwidth-bound at these ranks already.
//
//   k_project_skinny   partial R over a chunk of rows:  part[c][rho][j] = sum_{i in chunk c} P[i][rho] G[i][j]
//   k_skinny_reduce    R[rho][j] = sum_c part[c][rho][j] in a fixed order, into the ring slot `head`
//   k_update_skinny    W[i][j] <- W[i][j] - (lr scale sum_rho P[i][rho] N[rho][j] + lr wd W[i][j])
//
// The rows are split over workgroups (a whole-column workgroup would leave a few hundred very
// unequal workgroups for 256 CUs); the chunk sums meet in a second pass instead of atomics so the
// result does not depend on the order of arrival.
// Workgroup = 128 rows x 256 columns: a lane owns 4 consecutive columns, the four wavefronts take
// every fourth row.  The row of P a wavefront needs is the same for all its lanes (scalar loads).
#include "ng_internal.h"

namespace ng {

#define NG_AS1 __attribute__((address_space(1)))
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, 4-byte aligned

namespace {

// Four consecutive floats of a row that has n_left valid elements from this position on (the caller's
// rows are only 4-byte aligned in general).
__device__ __forceinline__ f32x4_t load_row4(const NG_AS1 float* base, long long elem, int n_left) {
    f32x4_t o = {0.f, 0.f, 0.f, 0.f};
    if (n_left >= 4) {
        o = *(const NG_AS1 f32x4_a4*)(base + elem);
    } else {
#pragma unroll
        for (int c = 0; c < 3; ++c)
            if (c < n_left) o[c] = base[elem + c];
    }
    return o;
}

__device__ __forceinline__ void store_row4(NG_AS1 float* base, long long elem, int n_left, f32x4_t v) {
    if (n_left >= 4) {
        *(NG_AS1 f32x4_a4*)(base + elem) = v;
    } else {
#pragma unroll
        for (int c = 0; c < 3; ++c)
            if (c < n_left) base[elem + c] = v[c];
    }
}

// Row i of P as RK wave-uniform floats (entries >= r read as zero).
template <int RK>
__device__ __forceinline__ void load_p_row(const float* __restrict__ P, int i, int r, float (&p)[RK]) {
    const float* __restrict__ row = P + (long long)i * r;
#pragma unroll
    for (int q = 0; q < RK; ++q) {
        const float v = row[q < r ? q : 0];
        p[q] = q < r ? v : 0.f;
    }
}

}  // namespace

// ------------------------------------------------------------------ projection, first pass
template <int RK>
__global__ __launch_bounds__(256) void k_project_skinny(const MatDev* __restrict__ mats,
                                                        const MatDyn* __restrict__ dyn,
                                                        const TileRef* __restrict__ tiles) {
    __shared__ float red[3][RK][kSkinnyCols];
    const TileRef t = tiles[blockIdx.x];
    if (t.mat < 0) return;
    const MatDev& md = mats[t.mat];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m = md.m, n = md.n, r = md.r, ldn = md.ldn;
    const int col = t.tj * kSkinnyCols + lane * 4;
    const int row0 = t.ti * kSkinnyRows;
    const int row1 = row0 + kSkinnyRows < m ? row0 + kSkinnyRows : m;
    const int n_left = n - col;                       // valid gradient columns from `col` on (may be <= 0)
    const NG_AS1 float* G = (const NG_AS1 float*)dyn[t.mat].g;
    const long long ld_g = md.ld_g;

    f32x4_t acc[RK];
#pragma unroll
    for (int q = 0; q < RK; ++q) acc[q] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

    // four rows per pass and wavefront: their loads are in flight together
    for (int i = row0 + wv; i < row1; i += 16) {
        f32x4_t g[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int iu = i + 4 * u;
            g[u] = (iu < row1 && n_left > 0) ? load_row4(G, (long long)iu * ld_g + col, n_left)
                                             : (f32x4_t){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int iu = i + 4 * u;                 // (uniform over the wavefront)
            if (iu >= row1) break;
            float p[RK];
            load_p_row<RK>(md.P, iu, r, p);
#pragma unroll
            for (int q = 0; q < RK; ++q) {
                acc[q].x = fmaf(p[q], g[u].x, acc[q].x);
                acc[q].y = fmaf(p[q], g[u].y, acc[q].y);
                acc[q].z = fmaf(p[q], g[u].z, acc[q].z);
                acc[q].w = fmaf(p[q], g[u].w, acc[q].w);
            }
        }
    }
    // wavefronts 1..3 hand their sums to wavefront 0, which adds them in order
    if (wv > 0) {
#pragma unroll
        for (int q = 0; q < RK; ++q) *reinterpret_cast<f32x4_t*>(&red[wv - 1][q][lane * 4]) = acc[q];
    }
    __syncthreads();
    if (wv == 0 && col < ldn) {
        float* __restrict__ part = step_scratch<float>(dyn, md.skinny_parts_off) + (long long)t.ti * RK * ldn;
#pragma unroll
        for (int q = 0; q < RK; ++q) {
            f32x4_t s = acc[q];
#pragma unroll
            for (int w = 0; w < 3; ++w) {
                const f32x4_t o = *reinterpret_cast<const f32x4_t*>(&red[w][q][lane * 4]);
                s.x += o.x;
                s.y += o.y;
                s.z += o.z;
                s.w += o.w;
            }
            *reinterpret_cast<f32x4_t*>(part + (long long)q * ldn + col) = s;
        }
    }
}

// ------------------------------------------------------------------ projection, second pass
// One thread per four columns of one row of R: the chunk sums in chunk order, into slot `head` of the
// ring.  Columns >= n hold zeros (their gradient entries were never read).
__global__ __launch_bounds__(64) void k_skinny_reduce(const MatDev* __restrict__ mats,
                                                      const MatDyn* __restrict__ dyn, int rk) {
    const MatDev& md = mats[blockIdx.z];
    const int col = (blockIdx.x * 64 + threadIdx.x) * 4, q = blockIdx.y;
    const int ldn = md.ldn;
    if (col >= ldn || q >= md.r) return;
    const int chunks = (md.m + kSkinnyRows - 1) / kSkinnyRows;
    const float* __restrict__ part = step_scratch<float>(dyn, md.skinny_parts_off) + (long long)q * ldn + col;
    const long long cstride = (long long)rk * ldn;
    f32x4_t s = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < chunks; c += 8) {             // eight loads in flight, added in chunk order
        f32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = c + u < chunks ? *reinterpret_cast<const f32x4_t*>(part + (c + u) * cstride)
                                  : (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            s.x += v[u].x;
            s.y += v[u].y;
            s.z += v[u].z;
            s.w += v[u].w;
        }
    }
    const long long slot = (long long)dyn[blockIdx.z].head * md.slot_elems;
    *reinterpret_cast<f32x4_t*>(md.H + slot + (long long)q * ldn + col) = s;
}

// ------------------------------------------------------------------ update
// N is float [r][ldn].
template <int RK>
__global__ __launch_bounds__(256) void k_update_skinny(const MatDev* __restrict__ mats,
                                                       const MatDyn* __restrict__ dyn,
                                                       const TileRef* __restrict__ tiles, StepScalars sc) {
    const TileRef t = tiles[blockIdx.x];
    if (t.mat < 0) return;
    const MatDev& md = mats[t.mat];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m = md.m, n = md.n, r = md.r, ldn = md.ldn;
    const int col = t.tj * kSkinnyCols + lane * 4;
    const int n_left = n - col;
    if (n_left <= 0) return;                          // (col < n <= ldn and ldn % 4 == 0: col + 4 <= ldn)
    const int row0 = t.ti * kSkinnyRows;
    const int row1 = row0 + kSkinnyRows < m ? row0 + kSkinnyRows : m;

    // this lane's four columns of N, all r rows (the entries of P beyond r read as zero)
    f32x4_t nv[RK];
    const float* __restrict__ N = reinterpret_cast<const float*>(md.N);
#pragma unroll
    for (int q = 0; q < RK; ++q)
        nv[q] = q < r ? *reinterpret_cast<const f32x4_t*>(N + (long long)q * ldn + col) : (f32x4_t){0.f, 0.f, 0.f, 0.f};

    NG_AS1 float* W = (NG_AS1 float*)dyn[t.mat].w;
    const long long ld_w = md.ld_w;
    for (int i = row0 + wv; i < row1; i += 16) {
        f32x4_t w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int iu = i + 4 * u;
            w[u] = iu < row1 ? load_row4(W, (long long)iu * ld_w + col, n_left) : (f32x4_t){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int iu = i + 4 * u;                 // (uniform over the wavefront)
            if (iu >= row1) break;
            float p[RK];
            load_p_row<RK>(md.P, iu, r, p);
            f32x4_t x = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < RK; ++q) {
                x.x = fmaf(p[q], nv[q].x, x.x);
                x.y = fmaf(p[q], nv[q].y, x.y);
                x.z = fmaf(p[q], nv[q].z, x.z);
                x.w = fmaf(p[q], nv[q].w, x.w);
            }
            f32x4_t o;
            o.x = w[u].x - (sc.lr_scale * x.x + sc.lr_wd * w[u].x);
            o.y = w[u].y - (sc.lr_scale * x.y + sc.lr_wd * w[u].y);
            o.z = w[u].z - (sc.lr_scale * x.z + sc.lr_wd * w[u].z);
            o.w = w[u].w - (sc.lr_scale * x.w + sc.lr_wd * w[u].w);
            store_row4(W, (long long)iu * ld_w + col, n_left, o);
        }
    }
}

// ------------------------------------------------------------------ launchers
hipError_t launch_project_skinny(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles, int n_mats,
                                 int max_ldn, int rk, hipStream_t stream) {
    if (n_tiles <= 0) return hipSuccess;
    if (rk == 4) hipLaunchKernelGGL(k_project_skinny<4>, dim3(n_tiles), dim3(256), 0, stream, mats, dyn, tiles);
    else if (rk == 8) hipLaunchKernelGGL(k_project_skinny<8>, dim3(n_tiles), dim3(256), 0, stream, mats, dyn, tiles);
    else if (rk == 16) hipLaunchKernelGGL(k_project_skinny<16>, dim3(n_tiles), dim3(256), 0, stream, mats, dyn, tiles);
    else return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_skinny_reduce, dim3((max_ldn + 255) / 256, rk, n_mats), dim3(64), 0, stream, mats, dyn, rk);
    return hipGetLastError();
}

hipError_t launch_update_skinny(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles, int rk,
                                StepScalars sc, hipStream_t stream) {
    if (n_tiles <= 0) return hipSuccess;
    if (rk == 4) hipLaunchKernelGGL(k_update_skinny<4>, dim3(n_tiles), dim3(256), 0, stream, mats, dyn, tiles, sc);
    else if (rk == 8) hipLaunchKernelGGL(k_update_skinny<8>, dim3(n_tiles), dim3(256), 0, stream, mats, dyn, tiles, sc);
    else if (rk == 16) hipLaunchKernelGGL(k_update_skinny<16>, dim3(n_tiles), dim3(256), 0, stream, mats, dyn, tiles, sc);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ng
