// Small dense linear algebra of the projector refresh (paper Sec. 1: P = leading
// left singular vectors of the gradient, recomputed every ~200 steps).  The
// large products run on the grouped fp32 MFMA GEMM (or, for bf16 gradients, on the
// split-sketch bf16 MFMA kernel); this file holds what sits between them, one launch for all matrices of the layer set:
//
//   k_fill_gaussian     random sketch Omega (counter-based generator, Box-Muller)
//   k_chol_*            T = L L^T in place (fp64, right-looking, panels of 32 columns)
//   k_tri_*             Linv = L^{-1} as float, by 32 x 32 blocks (the GEMM then applies X <- X Linv^T)
//   k_jacobi_*          blocked one-sided Jacobi on the rows of the l x l Rayleigh-Ritz matrix
//                       T = (Q^T G)(Q^T G)^T (a float copy in the Linv buffer): at convergence
//                       row i = ritz_i * u_i^T
//   k_ritz_sort / k_build_rotation   order by descending Ritz value, stage U[:, top r]
//   k_sign_fix          copy the orthonormalised basis into P, largest-magnitude entry of each
//                       column made positive
#include "ng_internal.h"

namespace ng {

// ------------------------------------------------------------------ random sketch
__device__ __forceinline__ unsigned long long mix64(unsigned long long z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void k_fill_gaussian(const MatDev* __restrict__ mats, unsigned long long seed,
                                                       unsigned long long call_id) {
    const MatDev& md = mats[blockIdx.y];
    const long long total = (long long)md.n * md.l;
    const unsigned long long key =
        mix64(seed ^ (call_id * 0x9E3779B97F4A7C15ULL) ^ ((unsigned long long)(blockIdx.y + 1) * 0xD1B54A32D192ED03ULL));
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        const unsigned long long z = mix64(key + (unsigned long long)(i + 1) * 0x9E3779B97F4A7C15ULL);
        const float u1 = ((float)(unsigned int)(z >> 40) + 1.0f) * (1.0f / 16777216.0f);      // (0, 1]
        const float u2 = (float)(unsigned int)((z >> 8) & 0xFFFFFFu) * (1.0f / 16777216.0f);   // [0, 1)
        md.Yb[i] = sqrtf(-2.0f * logf(u1)) * cosf(6.28318530717958647692f * u2);
    }
}

hipError_t launch_fill_gaussian(const MatDev* mats, int n_mats, int max_rows, unsigned long long seed,
                                unsigned long long call_id, hipStream_t stream) {
    int gx = (max_rows + 3) / 4;   // grid-stride loop covers the rest
    if (gx < 1) gx = 1;
    if (gx > 4096) gx = 4096;
    hipLaunchKernelGGL(k_fill_gaussian, dim3(gx, n_mats), dim3(256), 0, stream, mats, seed, call_id);
    return hipGetLastError();
}

// ------------------------------------------------------------------ Cholesky (fp64, in place, lower)
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// Right-looking blocked factorisation, panels of kCholNB columns, three launches per panel:
//   k_chol_diag    factor the kCholNB x kCholNB diagonal block in LDS (one workgroup per matrix)
//   k_chol_panel   rows below it: X L11^T = A21, one thread per row
//   k_chol_update  trailing lower triangle -= L21 L21^T, 64 x 64 tiles
// which: 0 -> order l, 1 -> order r.  T has leading dimension lp.  k_chol_shift first adds
// shift_rel * trace(T) to the diagonal.  A non-positive pivot sets bit 2 of *status (the pivot is
// replaced by 1).  Only the lower triangle is read and written.
constexpr int kCholNB = 32;

__global__ __launch_bounds__(256) void k_chol_shift(const MatDev* __restrict__ mats, int which, double shift_rel) {
    __shared__ double red[4];
    const MatDev& md = mats[blockIdx.x];
    const int nn = which == 0 ? md.l : md.r;
    const long long ld = md.lp;
    double* __restrict__ A = md.T;
    const int tid = threadIdx.x;
    double tr = 0.0;
    for (int i = tid; i < nn; i += 256) tr += A[i * ld + i];
    tr = wave_sum_d(tr);
    if ((tid & 63) == 0) red[tid >> 6] = tr;
    __syncthreads();
    const double shift = shift_rel * (((red[0] + red[1]) + red[2]) + red[3]);
    for (int i = tid; i < nn; i += 256) A[i * ld + i] += shift;
}

__global__ __launch_bounds__(256) void k_chol_diag(const MatDev* __restrict__ mats, int which, int k0, int* status) {
    __shared__ double D[kCholNB][kCholNB + 1];
    const MatDev& md = mats[blockIdx.x];
    const int nn = which == 0 ? md.l : md.r;
    if (k0 >= nn) return;
    const long long ld = md.lp;
    double* __restrict__ A = md.T;
    const int tid = threadIdx.x;
    for (int q = tid; q < kCholNB * kCholNB; q += 256) {
        const int i = q / kCholNB, j = q % kCholNB;
        double v = i == j ? 1.0 : 0.0;            // identity padding past the matrix order
        if (k0 + i < nn && j <= i) v = A[(long long)(k0 + i) * ld + k0 + j];
        D[i][j] = v;
    }
    __syncthreads();
    bool bad = false;
    for (int k = 0; k < kCholNB; ++k) {
        double d = D[k][k];
        if (!(d > 0.0) || !(d < 1.0e300)) {
            bad = true;
            d = 1.0;
        }
        const double rd = 1.0 / d;
        // rank-one update of the columns right of k with the still unscaled column k
        for (int q = tid; q < kCholNB * kCholNB; q += 256) {
            const int i = q / kCholNB, j = q % kCholNB;
            if (j > k && i >= j) D[i][j] -= D[i][k] * D[j][k] * rd;
        }
        __syncthreads();
        // column k is final now and not read again: scale it
        if (tid < kCholNB) {
            const double sd = sqrt(d);
            if (tid == k) D[k][k] = sd;
            else if (tid > k) D[tid][k] *= 1.0 / sd;
        }
    }
    __syncthreads();
    for (int q = tid; q < kCholNB * kCholNB; q += 256) {
        const int i = q / kCholNB, j = q % kCholNB;
        if (k0 + i < nn && j <= i) A[(long long)(k0 + i) * ld + k0 + j] = D[i][j];
    }
    if (bad && tid == 0) atomicOr(status, 4);
}

__global__ __launch_bounds__(256) void k_chol_panel(const MatDev* __restrict__ mats, int which, int k0) {
    __shared__ double Ls[kCholNB][kCholNB + 1];
    __shared__ double invd[kCholNB];
    const MatDev& md = mats[blockIdx.y];
    const int nn = which == 0 ? md.l : md.r;
    const int row0 = k0 + kCholNB + blockIdx.x * 256;
    if (row0 >= nn) return;               // (then k0 + kCholNB < nn: all panel columns exist)
    const long long ld = md.lp;
    double* __restrict__ A = md.T;
    const int tid = threadIdx.x;
    for (int q = tid; q < kCholNB * kCholNB; q += 256) {
        const int i = q / kCholNB, j = q % kCholNB;
        Ls[i][j] = j <= i ? A[(long long)(k0 + i) * ld + k0 + j] : 0.0;
    }
    __syncthreads();
    if (tid < kCholNB) invd[tid] = 1.0 / Ls[tid][tid];
    __syncthreads();
    const int i = row0 + tid;
    if (i >= nn) return;
    double* __restrict__ row = A + (long long)i * ld + k0;
    double x[kCholNB];
#pragma unroll
    for (int j = 0; j < kCholNB; ++j) x[j] = row[j];
#pragma unroll
    for (int j = 0; j < kCholNB; ++j) {
        double acc = x[j];
#pragma unroll
        for (int t = 0; t < j; ++t) acc -= x[t] * Ls[j][t];
        x[j] = acc * invd[j];
    }
#pragma unroll
    for (int j = 0; j < kCholNB; ++j) row[j] = x[j];
}

__global__ __launch_bounds__(256) void k_chol_update(const MatDev* __restrict__ mats, int which, int k0) {
    __shared__ double As[64][kCholNB + 1];
    __shared__ double Bs[64][kCholNB + 1];
    if (blockIdx.y > blockIdx.x) return;  // lower triangle of tiles only
    const MatDev& md = mats[blockIdx.z];
    const int nn = which == 0 ? md.l : md.r;
    const int base = k0 + kCholNB;
    const int r0 = base + 64 * blockIdx.x, c0 = base + 64 * blockIdx.y;
    if (r0 >= nn) return;
    const long long ld = md.lp;
    double* __restrict__ A = md.T;
    const int tid = threadIdx.x;
    for (int q = tid; q < 64 * kCholNB; q += 256) {
        const int rr = q / kCholNB, t = q % kCholNB;
        As[rr][t] = r0 + rr < nn ? A[(long long)(r0 + rr) * ld + k0 + t] : 0.0;
        Bs[rr][t] = c0 + rr < nn ? A[(long long)(c0 + rr) * ld + k0 + t] : 0.0;
    }
    __syncthreads();
    const int tx = tid & 15, ty = tid >> 4;   // outputs (ty + 16 e, tx + 16 f)
    double acc[4][4] = {};
#pragma unroll 4
    for (int t = 0; t < kCholNB; ++t) {
        double av[4], bv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            av[e] = As[ty + 16 * e][t];
            bv[e] = Bs[tx + 16 * e][t];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int f = 0; f < 4; ++f) acc[e][f] += av[e] * bv[f];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const int i = r0 + ty + 16 * e, j = c0 + tx + 16 * f;
            if (i < nn && j <= i) A[(long long)i * ld + j] -= acc[e][f];
        }
}

hipError_t launch_cholesky(const MatDev* mats, int n_mats, int which, int max_order, double shift_rel,
                           int* status, hipStream_t stream) {
    if (shift_rel > 0.0)
        hipLaunchKernelGGL(k_chol_shift, dim3(n_mats), dim3(256), 0, stream, mats, which, shift_rel);
    for (int k0 = 0; k0 < max_order; k0 += kCholNB) {
        hipLaunchKernelGGL(k_chol_diag, dim3(n_mats), dim3(256), 0, stream, mats, which, k0, status);
        const int below = max_order - k0 - kCholNB;
        if (below <= 0) break;
        hipLaunchKernelGGL(k_chol_panel, dim3((below + 255) / 256, n_mats), dim3(256), 0, stream, mats, which, k0);
        const int nt = (below + 63) / 64;
        hipLaunchKernelGGL(k_chol_update, dim3(nt, nt, n_mats), dim3(256), 0, stream, mats, which, k0);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ inverse of the Cholesky factor
// Linv = L^{-1} (lower triangular, float), by 32 x 32 blocks: X_ii = L_ii^{-1}, and below the diagonal
//   X_ij = -L_ii^{-1} (sum_{k=j..i-1} L_ik X_kj),
// so a block column of the inverse depends only on itself.  k_tri_diag_inverse inverts the diagonal
// blocks by forward substitution (one lane per column); k_tri_inverse_blocks gives a workgroup one block
// column and walks down its block rows: both products of a block run on fp64 MFMA (16x16x4; lane L
// supplies A[L%16][L/16] and B[L/16][L%16], element e of its result is D[4e + L/16][L%16]), the sum
// over k from L in global memory and the solved blocks above (LDS, floats), the multiplication by
// the inverted diagonal block from that block (global, floats) and the sum (LDS, doubles).  16
// dependent block steps at order 512 instead of the 128 four-row steps of a substitution over the
// whole column.  A solved entry is rounded to float before anything reads it back, so the stored
// inverse is what the rows below were computed from.  Rows and columns >= the order read as
// those of an identity and are not written.
typedef double double4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
constexpr int kTriNB = 32;

__global__ __launch_bounds__(64) void k_tri_diag_inverse(const MatDev* __restrict__ mats, int which) {
    __shared__ double Ls[2][kTriNB][kTriNB + 1], Xl[2][kTriNB][kTriNB + 1];
    const MatDev& md = mats[blockIdx.y];
    const int nn = which == 0 ? md.l : md.r;
    const long long ld = md.lp;
    const int half = threadIdx.x >> 5, c = threadIdx.x & 31;
    const int r0 = (2 * (int)blockIdx.x + half) * kTriNB;
    const double* __restrict__ L = md.T;
    // (no early return: both halves meet at the barrier; a half past the order works on an identity)
    for (int i = 0; i < kTriNB; ++i) {
        const int gi = r0 + i, gc = r0 + c;
        double v = (i == c) ? 1.0 : 0.0;
        if (gi < nn && gc < nn && c <= i) v = L[(long long)gi * ld + gc];
        Ls[half][i][c] = v;
    }
    __syncthreads();
    // column c of the inverse: x_i = (e_i - sum_{k=c..i-1} L_ik x_k) / L_ii, x_i = 0 above the diagonal
    float* __restrict__ Xg = md.Linv;
    for (int i = 0; i < kTriNB; ++i) {
        double xi = 0.0;
        if (i >= c) {
            double tot = 0.0;
            for (int k = c; k < i; ++k) tot += Ls[half][i][k] * Xl[half][k][c];
            xi = (double)(float)(((i == c ? 1.0 : 0.0) - tot) / Ls[half][i][i]);
        }
        Xl[half][i][c] = xi;       // read back by this lane only
        if (r0 + i < nn && r0 + c < nn) Xg[(long long)(r0 + i) * ld + r0 + c] = (float)xi;
    }
}

// XLDS: the solved blocks of the column are kept in LDS (as two 16-column halves, [half][row][16]:
// the four rows of an MFMA operand are 64 consecutive floats); otherwise they are read back from Linv
// in global memory, which the barrier of each block step makes visible inside the workgroup.
template <bool XLDS>
__global__ __launch_bounds__(256) void k_tri_inverse_blocks(const MatDev* __restrict__ mats, int which) {
    extern __shared__ __attribute__((aligned(16))) unsigned char tri_smem[];
    const MatDev& md = mats[blockIdx.y];
    const int nn = which == 0 ? md.l : md.r;
    const int nb = (nn + kTriNB - 1) / kTriNB;
    // Block column b costs (nb - b)^2.  Workgroup ids go round-robin over the 8 XCDs, so with a block
    // count that is a multiple of 8 a plain b = blockIdx.x would give one XCD the two most expensive
    // columns of every matrix; rotating by the matrix index spreads them.
    const int jb = (int)((blockIdx.x + blockIdx.y) % gridDim.x);
    if (jb >= nb) return;
    const long long ld = md.lp;
    const double* __restrict__ L = md.T;
    float* __restrict__ Xg = md.Linv;
    const int c0 = jb * kTriNB;
    const int rows = (nb - jb) * kTriNB;                     // rows c0 .. of the block column, padded
    double* Ssm = reinterpret_cast<double*>(tri_smem);       // [2][32][16]
    float* Xs = reinterpret_cast<float*>(Ssm + 2 * kTriNB * 16);   // [2][rows][16] (XLDS)
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4, tr = wv >> 1, tc = wv & 1;
    const int col = c0 + 16 * tc + l16;                      // this lane's column of the result tiles
    const bool col_ok = col < nn;

    // rows above the block column: exact zeros
    for (int q = tid; q < c0 * kTriNB; q += 256) {
        const int i = q / kTriNB, cc = q % kTriNB;
        if (c0 + cc < nn) Xg[(long long)i * ld + c0 + cc] = 0.f;
    }
    if (XLDS) {
        // the diagonal block, as the first kernel left it
        for (int q = tid; q < kTriNB * kTriNB; q += 256) {
            const int i = q / kTriNB, cc = q % kTriNB;
            const bool in = c0 + i < nn && c0 + cc < nn;
            Xs[((cc >> 4) * rows + i) * 16 + (cc & 15)] = in ? Xg[(long long)(c0 + i) * ld + c0 + cc] : 0.f;
        }
    }
    __syncthreads();

    for (int ib = jb + 1; ib < nb; ++ib) {
        const int r0 = ib * kTriNB;
        // the inverted diagonal block of this block row (does not depend on the sum: fetched first)
        float dinv[8];
        {
            const int gi = r0 + 16 * tr + l16;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int gk = r0 + 4 * u + lq;
                dinv[u] = (gi < nn && gk < nn) ? Xg[(long long)gi * ld + gk] : 0.f;
            }
        }
        // S = sum_k L[ib][k] X[k][jb] over the columns c0 .. r0-1 (all below the order): tile (tr, tc)
        double4_t acc = {0.0, 0.0, 0.0, 0.0};
        {
            const int gi = r0 + 16 * tr + l16;
            const bool rok = gi < nn;
            const double* __restrict__ lrow = L + (long long)(rok ? gi : 0) * ld + c0 + lq;
            const int nk = r0 - c0;
            for (int k = 0; k < nk; k += 16) {              // nk % 32 == 0: four k-steps per pass
                double a[4];
                float b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    a[u] = rok ? lrow[k + 4 * u] : 0.0;
                    const int kr = k + 4 * u + lq;           // row of the block column, from c0
                    b[u] = XLDS ? Xs[(tc * rows + kr) * 16 + l16]
                                : (col_ok ? Xg[(long long)(c0 + kr) * ld + col] : 0.f);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u], (double)b[u], acc, 0, 0, 0);
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) Ssm[(tc * kTriNB + 16 * tr + 4 * e + lq) * 16 + l16] = acc[e];
        __syncthreads();
        // X[ib][jb] = -Dinv S
        double4_t o = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int u = 0; u < 8; ++u)
            o = __builtin_amdgcn_mfma_f64_16x16x4f64((double)dinv[u], Ssm[(tc * kTriNB + 4 * u + lq) * 16 + l16], o, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 16 * tr + 4 * e + lq;              // row inside the block
            const float xf = (float)(-o[e]);
            if (XLDS) Xs[(tc * rows + (r0 - c0) + i) * 16 + l16] = xf;
            if (r0 + i < nn && col_ok) Xg[(long long)(r0 + i) * ld + col] = xf;
        }
        __syncthreads();
    }
}

hipError_t launch_tri_inverse(const MatDev* mats, int n_mats, int which, int max_order, hipStream_t stream) {
    const int nb = (max_order + kTriNB - 1) / kTriNB;
    if (nb <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_tri_diag_inverse, dim3((nb + 1) / 2, n_mats), dim3(64), 0, stream, mats, which);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    static bool attr_done = false;
    constexpr size_t kBudget = 150 * 1024;
    if (!attr_done) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_tri_inverse_blocks<true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBudget);
        attr_done = true;
    }
    const size_t s_bytes = (size_t)2 * kTriNB * 16 * sizeof(double);
    const size_t x_bytes = (size_t)2 * nb * kTriNB * 16 * sizeof(float);
    if (s_bytes + x_bytes <= kBudget)
        hipLaunchKernelGGL(k_tri_inverse_blocks<true>, dim3(nb, n_mats), dim3(256), s_bytes + x_bytes, stream, mats, which);
    else
        hipLaunchKernelGGL(k_tri_inverse_blocks<false>, dim3(nb, n_mats), dim3(256), s_bytes, stream, mats, which);
    return hipGetLastError();
}

// ------------------------------------------------------------------ blocked one-sided Jacobi
// X (lp x lp, row-major) starts as the symmetric matrix T (rows/columns >= l zero).
// Rotating ROWS until they are mutually orthogonal gives X = Lambda U^T: row i is
// ritz_i * u_i^T.  Rows are grouped in blocks of 16; one workgroup takes a pair of blocks (a
// "visit"): it forms the 32 x 32 Gram matrix of the 32 rows, runs one cyclic Jacobi sweep on that
// small matrix with the rotations accumulated in V, and applies X <- V X to the rows.  Block pairs
// follow a round-robin tournament so the lp/16 - 1 rounds of one sweep meet every block pair once.
__device__ __forceinline__ void tournament_pair(int players, int round, int k, int* a, int* b) {
    const int N = players - 1;
    if (k == 0) {
        *a = N;
        *b = round % N;
    } else {
        *a = (round + k) % N;
        *b = (round - k + N) % N;
    }
}

// The rows that the Jacobi rotates are kept as floats (the result, a rotation stored as floats, needs
// no more; every product and sum on them is still formed in fp64): X = T rounded, zero in the padding,
// in the buffer of the inverse Cholesky factor, which is free between the last orthonormalisation
// and the one of the new projector.
__device__ __forceinline__ float* jacobi_rows(const MatDev& md) { return md.Linv; }

__global__ __launch_bounds__(256) void k_jacobi_prepare(const MatDev* __restrict__ mats) {
    const MatDev& md = mats[blockIdx.y];
    const int lp = md.lp, l = md.l;
    const long long total = (long long)lp * lp;
    float* __restrict__ X = jacobi_rows(md);
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < total; q += (long long)gridDim.x * 256) {
        const int i = (int)(q / lp), j = (int)(q % lp);
        // (the product that made T wrote only its tiles on and below the diagonal)
        const long long src = i >= j ? q : (long long)j * lp + i;
        X[q] = (i < l && j < l) ? (float)md.T[src] : 0.f;
    }
    if (blockIdx.x == 0 && threadIdx.x < 4) md.jflag[threadIdx.x] = 0;
}

hipError_t launch_jacobi_prepare(const MatDev* mats, int n_mats, hipStream_t stream) {
    hipLaunchKernelGGL(k_jacobi_prepare, dim3(64, n_mats), dim3(256), 0, stream, mats);
    return hipGetLastError();
}

// v + (v of the partner lane under a DPP lane pattern).  Used with the symmetric patterns below, so
// both partners form the same sum with the operands swapped and hold bit-identical results.
template <int CTRL>
__device__ __forceinline__ double dpp_pair_add(double v) {
    const int lo = __double2loint(v), hi = __double2hiint(v);
    const int plo = __builtin_amdgcn_mov_dpp(lo, CTRL, 0xf, 0xf, false);
    const int phi = __builtin_amdgcn_mov_dpp(hi, CTRL, 0xf, 0xf, false);
    return v + __hiloint2double(phi, plo);
}
// All-reduce over the 64 lanes; every lane ends with the same bits.  Lanes 1 and 2 apart are paired by
// quad permutes, quads and half rows by the mirror patterns (a lane's partner holds the other
// quad's / half's sum), the four 16-lane rows by two cross-lane exchanges.
__device__ __forceinline__ double wave_allreduce(double v) {
    v = dpp_pair_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_pair_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_pair_add<0x141>(v);   // row_half_mirror
    v = dpp_pair_add<0x140>(v);   // row_mirror
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}


// ------------------------------------------------------------------ block rotation through the Gram matrix
// One visit of a pair of 16-row blocks (32 rows of length lp, floats in global memory):
//   S = X X^T          32 x 32 Gram of the rows, fp64 MFMA (16x16x4), the columns split over eight wavefronts
//   small sweep        cyclic rounds of 16 disjoint rotations each, applied two-sidedly to S (S <- J S J^T)
//                      and accumulated in V (V <- J V): the rotations that a row-by-row Jacobi would
//                      apply, decided from S instead of fresh dot products.  Round 0 of a sweep takes
//                      all 496 row pairs of the visit (31 rounds), every other round the 256 pairs
//                      with a row in each block (16 rounds)
//   X <- V X           fp64 MFMA, each wavefront owns 16-column tiles, written straight back to memory
// so the 32 rows are read twice per visit instead of 2 x 31 times.
// (operand and result layout of v_mfma_f64_16x16x4_f64 as stated at the triangular inverse; checked on
// the device)
constexpr int kJgLdS = 36;     // row length of S and V in LDS (32 + 4: 16 rows land on distinct banks)
constexpr int kJgParts = 8;    // wavefronts that share the Gram product (a slice of the columns each)

// cs, sn of the rotation that orthogonalises two rows with squared norms al, be and inner product ga
// (the same angle as the row-by-row kernel).  Reciprocal and reciprocal square root start from the
// hardware approximations and take Newton steps to full precision; cs^2 + sn^2 = 1 to rounding
// whatever the error of the angle.
__device__ __forceinline__ double rsq_nr(double x) {
    double y = __builtin_amdgcn_rsq(x);
    y = y * (1.5 - 0.5 * x * y * y);
    return y * (1.5 - 0.5 * x * y * y);
}
__device__ __forceinline__ void rotation_params(double al, double be, double ga, double* cs, double* sn) {
    const double d = be - al, g2 = 2.0 * ga;
    const double q = d * d + g2 * g2;
    // (the angle only has to be good enough to shrink the coupling quadratically: one Newton step)
    double y = __builtin_amdgcn_rsq(q);
    y = y * (1.5 - 0.5 * q * y * y);
    const double h = q * y;                                          // sqrt(d^2 + 4 ga^2)
    const double den = fabs(d) + h;
    double rd = __builtin_amdgcn_rcp(den);
    rd = rd * (2.0 - den * rd);
    const double tn = (d >= 0.0 ? g2 : -g2) * rd;                    // tan of the angle
    const double c = rsq_nr(1.0 + tn * tn);
    *cs = c;
    *sn = c * tn;
}

// State of one row index in the 32-player tournament, advanced round by round without divisions:
// in round ir the pairs are (31, ir) and ((ir + k) % 31, (ir - k) % 31), k = 1..15.
struct TournamentRow {
    int i, q, k;     // q = (2 ir - i) mod 31, k = (i - ir) mod 31
    __device__ __forceinline__ void init(int row) {
        i = row;
        q = (62 - row) % 31;
        k = row % 31;
    }
    __device__ __forceinline__ int partner(int ir) const { return i == 31 ? ir : (q == i ? 31 : q); }
    __device__ __forceinline__ void advance() {
        q += 2;
        if (q >= 31) q -= 31;
        k = k == 0 ? 30 : k - 1;
    }
};

__global__ __launch_bounds__(512, 8) void k_jacobi_round_gram(const MatDev* __restrict__ mats, int round) {
    extern __shared__ __attribute__((aligned(16))) double smem_d[];
    __shared__ double cc[32], tt[32];
    __shared__ int nrot_s;
    __shared__ double smax_s;
    const MatDev& md = mats[blockIdx.y];
    const int lp = md.lp;
    const int nb = lp / 16;
    if ((int)blockIdx.x >= nb / 2 || round >= nb - 1) return;
    if (md.jflag[1] != 0) return;       // converged in an earlier sweep
    int bp, bq;
    tournament_pair(nb, round, blockIdx.x, &bp, &bq);
    // Round 0 of a sweep (every block is in exactly one pair) rotates all 496 row pairs of a visit;
    // the other rounds only the 256 pairs with one row in each block: the pairs inside a block
    // would otherwise be rotated again in each of its nb - 1 visits of the sweep.
    const bool cross = round != 0;
    // a block of padding rows only has nothing to rotate (in round 0 its partner still has its own pairs)
    if (cross ? (bp * 16 >= md.l || bq * 16 >= md.l) : (bp * 16 >= md.l && bq * 16 >= md.l)) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // The 32 rows of the pair stay in global memory: the Gram product and X <- V X take their MFMA
    // operands straight from there (the second read mostly from the L2).  More than half of a visit
    // is the dependent rounds of its small sweep, in which a CU is mostly idle, so what counts is
    // how many visits a CU holds: eight wavefronts and 48 KB of LDS per visit (S and V take the place
    // of the Gram partials once those are summed) make it three.
    double* part = smem_d;                          // [kJgParts / 2][3][256] Gram partials
    double* Ss = smem_d;                            // [32][kJgLdS], after the partials are summed
    double* Vs = Ss + 32 * kJgLdS;                  // [32][kJgLdS]
    float* __restrict__ X = jacobi_rows(md);
    float* __restrict__ Xp = X + (long long)bp * 16 * lp;   // rows 0..15 of the pair
    float* __restrict__ Xq = X + (long long)bq * 16 * lp;   // rows 16..31
    if (tid == 0) nrot_s = 0;

    // ---- Gram: each wavefront takes an eighth of the columns and computes the tiles (0,0), (1,0),
    // (1,1) from the same two operands per k-step; (0,1) is the transpose of (1,0).  The partials are
    // added in a fixed order.
    const int l16 = lane & 15, lq = lane >> 4;
    {
        double4_t g00 = {0.0, 0.0, 0.0, 0.0}, g10 = {0.0, 0.0, 0.0, 0.0}, g11 = {0.0, 0.0, 0.0, 0.0};
        const int cols = lp / kJgParts;            // lp % 32 == 0: cols % 4 == 0
        // A lane reads four consecutive columns of its row, 16 columns per 16 lanes and chunk; k-step
        // u of a chunk contracts over element u of every lane, i.e. over the columns 4 (L/16) + u:
        // both operands are the same rows, so any order of the contraction serves.
        const float* p0 = Xp + (long long)l16 * lp + wv * cols + 4 * lq;
        const float* p1 = Xq + (long long)l16 * lp + wv * cols + 4 * lq;
        const f32x4_t zero4 = {0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < cols; k += 16) {
            const bool in = k + 4 * lq < cols;
            const f32x4_t x0 = in ? *reinterpret_cast<const f32x4_t*>(p0 + k) : zero4;
            const f32x4_t x1 = in ? *reinterpret_cast<const f32x4_t*>(p1 + k) : zero4;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const double a0 = (double)x0[u], a1 = (double)x1[u];
                g00 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, a0, g00, 0, 0, 0);
                g10 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, a0, g10, 0, 0, 0);
                g11 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, a1, g11, 0, 0, 0);
            }
        }
        // wavefronts 4..7 hand their tiles to wavefronts 0..3, which add their own and publish the four
        // sums: half the LDS of eight partial sets
        double* dst = part + (wv & 3) * 768;
        if (wv >= 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dst[e * 64 + lane] = g00[e];
                dst[256 + e * 64 + lane] = g10[e];
                dst[512 + e * 64 + lane] = g11[e];
            }
        }
        __syncthreads();
        if (wv < 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                g00[e] += dst[e * 64 + lane];
                g10[e] += dst[256 + e * 64 + lane];
                g11[e] += dst[512 + e * 64 + lane];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {     // (each lane overwrites exactly what it has just read)
                dst[e * 64 + lane] = g00[e];
                dst[256 + e * 64 + lane] = g10[e];
                dst[512 + e * 64 + lane] = g11[e];
            }
        }
    }
    __syncthreads();
    {
        // entries tid and tid + 512 (the latter below 768) of the three tiles; the sums wait in
        // registers until every partial has been read, because S overwrites them
        double v0 = 0.0, v1 = 0.0;
#pragma unroll
        for (int w = 0; w < kJgParts / 2; ++w) v0 += part[w * 768 + tid];
        if (tid < 256) {
#pragma unroll
            for (int w = 0; w < kJgParts / 2; ++w) v1 += part[w * 768 + 512 + tid];
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (k == 1 && tid >= 256) break;
            const int idx = tid + 512 * k;
            const double v = k ? v1 : v0;
            // element e of lane L is entry (4e + L/16, L%16) of its tile
            const int tile = idx >> 8, e = (idx >> 6) & 3, ln = idx & 63;
            const int ii = 4 * e + (ln >> 4), jj = ln & 15;
            if (tile == 0) {
                Ss[ii * kJgLdS + jj] = v;
            } else if (tile == 1) {
                Ss[(16 + ii) * kJgLdS + jj] = v;
                Ss[jj * kJgLdS + 16 + ii] = v;
            } else {
                Ss[(16 + ii) * kJgLdS + 16 + jj] = v;
            }
        }
    }
    // ---- V = I (its place held no partials that anyone still needs: all were read before the barrier)
    const int pk = tid >> 5, vj = tid & 31;        // thread (pk, vj): row pair pk of a round, column vj
    Vs[pk * kJgLdS + vj] = pk == vj ? 1.0 : 0.0;
    Vs[(16 + pk) * kJgLdS + vj] = 16 + pk == vj ? 1.0 : 0.0;
    __syncthreads();
    // largest diagonal entry of S (scale of the rounding noise inside this visit)
    if (wv == 0) {
        double d = lane < 32 ? Ss[lane * kJgLdS + lane] : 0.0;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) d = fmax(d, __shfl_xor(d, off, 64));
        if (lane == 0) smax_s = d;
    }
    __syncthreads();

    // ---- the small sweep on S, accumulated in V.  A round rotates 16 disjoint row pairs (a, b);
    // thread (pk, vj) owns both rows of pair pk in column vj: S[a][vj], S[b][vj], V[a][vj], V[b][vj].
    TournamentRow rj;
    rj.init(vj);
    int nrot = 0;
    const int nir = cross ? 16 : 31;
    for (int ir = 0; ir < nir; ++ir) {
        int a, b;
        tournament_pair(32, ir, pk, &a, &b);
        if (cross) { a = pk; b = 16 + ((pk + ir) & 15); }
        const int pj = cross ? (vj < 16 ? 16 + ((vj + ir) & 15) : ((vj - ir) & 15)) : rj.partner(ir);
        // old values first (their addresses depend on the round only), rotation parameters meanwhile
        const double sav = Ss[a * kJgLdS + vj], sbv = Ss[b * kJgLdS + vj];
        const double sap = Ss[a * kJgLdS + pj], sbp = Ss[b * kJgLdS + pj];
        const double va = Vs[a * kJgLdS + vj], vb = Vs[b * kJgLdS + vj];
        if (tid < 16) {      // one thread per pair, all in one wavefront
            int a, b;
            tournament_pair(32, ir, tid, &a, &b);
            if (cross) { a = tid; b = 16 + ((tid + ir) & 15); }
            const double al = Ss[a * kJgLdS + a], be = Ss[b * kJgLdS + b], ga = Ss[a * kJgLdS + b];
            double cs = 1.0, sn = 0.0;
            if ((al > 0.0) && (be > 0.0) && (ga * ga > 1.0e-15 * al * be)) {
                rotation_params(al, be, ga, &cs, &sn);
                // a coupling below the visit's own rounding noise (entries that went through
                // rotations with much larger rows), or one below ~3e-4 of the two rows' norms (what is
                // left after a sweep of such rotations is quadratically smaller, ~1e-7: the rounding
                // of the float the result is stored in), is applied but does not keep the sweep loop
                // alive
                if (fabs(ga) > 8.0e-15 * smax_s && ga * ga > 1.0e-7 * al * be) ++nrot;
            }
            cc[a] = cs;
            cc[b] = cs;
            tt[a] = -sn;     // row a <- cs * a - sn * b
            tt[b] = sn;      // row b <- sn * a + cs * b
        }
        __syncthreads();     // every old value has been read; the parameters are published
        const double cs = cc[a], sn = tt[b], cj = cc[vj], tj_ = tt[vj];
        Ss[a * kJgLdS + vj] = cj * (cs * sav - sn * sbv) + tj_ * (cs * sap - sn * sbp);
        Ss[b * kJgLdS + vj] = cj * (sn * sav + cs * sbv) + tj_ * (sn * sap + cs * sbp);
        Vs[a * kJgLdS + vj] = cs * va - sn * vb;
        Vs[b * kJgLdS + vj] = sn * va + cs * vb;
        rj.advance();
        __syncthreads();
    }
    if (nrot) atomicAdd(&nrot_s, nrot);

    // ---- X <- V X: wavefront wv takes the 16-column tiles wv, wv + 8, ...; both 16-row halves
    const int nct = lp / 16;
    const double* va0 = Vs + l16 * kJgLdS + lq;                // A[L%16][k + L/16] = V[L%16][k + L/16], k = 4u
    const double* va1 = Vs + (16 + l16) * kJgLdS + lq;
    const unsigned rowoff = (unsigned)lq * (unsigned)lp + (unsigned)l16, lp4 = 4u * (unsigned)lp;
    for (int ct = wv; ct < nct; ct += 8) {
        // B[k + L/16][L%16] = X[k + L/16][c0 + L%16], k = 4u: rows 0..15 from Xp, 16..31 from Xq; element e
        // of a result tile is row 4e + L/16 of its half: the same offsets
        const unsigned base = rowoff + 16u * (unsigned)ct;
        float bx[8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            bx[u] = Xp[base + u * lp4];
            bx[4 + u] = Xq[base + u * lp4];
        }
        double4_t o0 = {0.0, 0.0, 0.0, 0.0}, o1 = {0.0, 0.0, 0.0, 0.0};
        // V is read from LDS for every tile: held across tiles its 32 registers spill.  The offset is
        // opaque to the compiler so that it does not hoist the reads out of the loop.
        int vo = 0;
        asm volatile("" : "+v"(vo));
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            o0 = __builtin_amdgcn_mfma_f64_16x16x4f64(va0[4 * u + vo], (double)bx[u], o0, 0, 0, 0);
            o1 = __builtin_amdgcn_mfma_f64_16x16x4f64(va1[4 * u + vo], (double)bx[u], o1, 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            Xp[base + e * lp4] = (float)o0[e];
            Xq[base + e * lp4] = (float)o1[e];
        }
    }
    __syncthreads();
    if (tid == 0 && nrot_s) atomicAdd(&md.jflag[0], nrot_s);
}

hipError_t launch_jacobi_round(const MatDev* mats, int n_mats, int max_pairs, int round, hipStream_t stream) {
    static bool attr_done = false;
    constexpr int lds = kJgParts / 2 * 768 * (int)sizeof(double);   // S and V (2 x 32 x kJgLdS doubles) fit inside
    static_assert(2 * 32 * kJgLdS <= kJgParts / 2 * 768, "S and V take the place of the Gram partials");
    if (!attr_done) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_jacobi_round_gram),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_done = true;
    }
    hipLaunchKernelGGL(k_jacobi_round_gram, dim3(max_pairs, n_mats), dim3(512), lds, stream, mats, round);
    return hipGetLastError();
}

__global__ void k_jacobi_sweep_end(const MatDev* __restrict__ mats, int n_mats) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_mats) return;
    int* f = mats[i].jflag;
    if (f[1] == 0) {
        f[2] += 1;                 // sweeps performed
        if (f[0] == 0) f[1] = 1;   // no rotation in this sweep: converged
    }
    f[0] = 0;
}

hipError_t launch_jacobi_sweep_end(const MatDev* mats, int n_mats, hipStream_t stream) {
    hipLaunchKernelGGL(k_jacobi_sweep_end, dim3((n_mats + 63) / 64), dim3(64), 0, stream, mats, n_mats);
    return hipGetLastError();
}

// Ritz values (row norms), descending order, then the l x r rotation U[:, top r] as floats in Bm.
__global__ __launch_bounds__(256) void k_ritz_sort(const MatDev* __restrict__ mats, int* status) {
    const MatDev& md = mats[blockIdx.x];
    const int lp = md.lp;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int i = wv; i < lp; i += 4) {
        const float* __restrict__ row = jacobi_rows(md) + (long long)i * lp;
        double a = 0.0;
        for (int c = lane; c < lp; c += 64) a += (double)row[c] * (double)row[c];
        a = wave_sum_d(a);
        if (lane == 0) md.ritz[i] = sqrt(a);
    }
    __syncthreads();
    __threadfence_block();
    bool bad = false;
    for (int i = threadIdx.x; i < lp; i += 256) {
        const double vi = md.ritz[i];
        int rank = 0;
        for (int j = 0; j < lp; ++j) {
            const double vj = md.ritz[j];
            rank += (vj > vi) || (vj == vi && j < i);
        }
        md.order[rank] = i;
        if (rank < md.r && !(vi > 0.0)) bad = true;
    }
    if (bad) atomicOr(status, 8);
    // no sweep without a rotation was seen before the sweep limit
    if (threadIdx.x == 0 && md.jflag[1] == 0) atomicOr(status, kStatusNotConverged);
}

__global__ __launch_bounds__(256) void k_build_rotation(const MatDev* __restrict__ mats) {
    const MatDev& md = mats[blockIdx.y];
    const int l = md.l, r = md.r, lp = md.lp;
    const long long total = (long long)l * r;
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < total; q += (long long)gridDim.x * 256) {
        const int k = (int)(q / r), j = (int)(q % r);
        const int src = md.order[j];
        const double nrm = md.ritz[src];
        md.Bm[q] = nrm > 0.0 ? (float)((double)jacobi_rows(md)[(long long)src * lp + k] / nrm) : 0.f;
    }
}

hipError_t launch_jacobi_finish(const MatDev* mats, int n_mats, int* status, hipStream_t stream) {
    hipLaunchKernelGGL(k_ritz_sort, dim3(n_mats), dim3(256), 0, stream, mats, status);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_build_rotation, dim3(128, n_mats), dim3(256), 0, stream, mats);
    return hipGetLastError();
}

// ------------------------------------------------------------------ sign convention, copy into P
// Source: Ya viewed as [m][r].  Each column is multiplied by the sign of its entry of largest
// magnitude (first one on ties) and written to P.
__global__ __launch_bounds__(256) void k_sign_fix(const MatDev* __restrict__ mats) {
    __shared__ float best[4][64];
    __shared__ int besti[4][64];
    const MatDev& md = mats[blockIdx.y];
    const int r = md.r, m = md.m;
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int rg = threadIdx.x >> 6;
    if (blockIdx.x * 64 >= r) return;
    const float* __restrict__ src = md.Ya;
    float bv = -1.f;
    int bi = 0;
    if (c < r)
        for (int i = rg; i < m; i += 4) {
            const float a = fabsf(src[(long long)i * r + c]);
            if (a > bv) { bv = a; bi = i; }
        }
    best[rg][threadIdx.x & 63] = bv;
    besti[rg][threadIdx.x & 63] = bi;
    __syncthreads();
    float sgn = 1.f;
    if (c < r) {
        float v = best[0][threadIdx.x & 63];
        int idx = besti[0][threadIdx.x & 63];
        for (int g = 1; g < 4; ++g) {
            const float v2 = best[g][threadIdx.x & 63];
            const int i2 = besti[g][threadIdx.x & 63];
            if (v2 > v || (v2 == v && i2 < idx)) { v = v2; idx = i2; }
        }
        sgn = src[(long long)idx * r + c] < 0.f ? -1.f : 1.f;
        for (int i = rg; i < m; i += 4) md.P[(long long)i * r + c] = sgn * src[(long long)i * r + c];
    }
}

hipError_t launch_sign_fix(const MatDev* mats, int n_mats, int max_r, hipStream_t stream) {
    hipLaunchKernelGGL(k_sign_fix, dim3((max_r + 63) / 64, n_mats), dim3(256), 0, stream, mats);
    return hipGetLastError();
}

}  // namespace ng
