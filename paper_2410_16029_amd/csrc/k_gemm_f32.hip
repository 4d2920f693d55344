// Grouped fp32 GEMM on the fp32 MFMA (v_mfma_f32_32x32x2_f32), one launch for
// all matrices of the layer set.  It serves the NG_F32 step (projection
// R = P^T G, paper Sec. 1; update W -= lr (scale P N + wd W), paper Sec. 2.2)
// and every dense product of the projector refresh.  Operands are described as
// strided views A(i,k), B(k,j) so one kernel covers all transpositions; an
// operand may be stored as float or bf16 (gradients).
//
// Tile 64 x 64 per workgroup (4 wavefronts, one 32 x 32 MFMA block each), BK = 16.
// MFMA 32x32x2 f32 operand layout: lane L supplies A[i = L%32][k = L/32] and
// B[k = L/32][j = L%32]; the 16 accumulators of lane L are
// D[8*g + 4*(L/32) + e][L%32], index 4*g + e.
#include "ng_internal.h"

namespace ng {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

enum { EPI_F32 = 0, EPI_F64 = 1, EPI_W_F32 = 2 };

struct GemmView {
    const void* A;
    const void* B;
    void* C;
    long long sAi, sAk, sBk, sBj, ldc;
    int M, N, K;      // C is M x N, contraction length K
    int Nvalid;       // columns j >= Nvalid of B read as zero (padding columns of the r x ldn space)
    int a_bf16, b_bf16;
    int epi;
};

__host__ __device__ inline GemmView gemm_view(int op, const MatDev& md, const MatDyn* dy, int grad_dtype) {
    GemmView v;
    v.a_bf16 = 0;
    v.b_bf16 = 0;
    v.epi = EPI_F32;
    const int gb = (grad_dtype == NG_BF16) ? 1 : 0;
    const void* G = dy ? dy->g : nullptr;
    switch (op) {
        case OP_PROJECT_F32:
            v.A = md.P; v.sAi = 1; v.sAk = md.r;
            v.B = G; v.sBk = md.ld_g; v.sBj = 1; v.b_bf16 = gb;
            v.M = md.r; v.N = md.ldn; v.Nvalid = md.n; v.K = md.m;
            v.C = md.H + (long long)(dy ? dy->head : 0) * md.slot_elems; v.ldc = md.ldn;
            break;
        case OP_UPDATE_F32:
            v.A = md.P; v.sAi = md.r; v.sAk = 1;
            v.B = md.N; v.sBk = md.ldn; v.sBj = 1;
            v.M = md.m; v.N = md.n; v.Nvalid = md.n; v.K = md.r;
            v.C = dy ? dy->w : nullptr; v.ldc = md.ld_w; v.epi = EPI_W_F32;
            break;
        case OP_G_B2A:
        case OP_G_C2A:
            v.A = G; v.sAi = md.ld_g; v.sAk = 1; v.a_bf16 = gb;
            v.B = (op == OP_G_B2A) ? md.Yb : md.Yc; v.sBk = md.l; v.sBj = 1;
            v.M = md.m; v.N = md.l; v.Nvalid = md.l; v.K = md.n;
            v.C = md.Ya; v.ldc = md.l;
            break;
        case OP_GT_A2B:
        case OP_GT_C2B:
            v.A = G; v.sAi = 1; v.sAk = md.ld_g; v.a_bf16 = gb;
            v.B = (op == OP_GT_A2B) ? md.Ya : md.Yc; v.sBk = md.l; v.sBj = 1;
            v.M = md.n; v.N = md.l; v.Nvalid = md.l; v.K = md.m;
            v.C = md.Yb; v.ldc = md.l;
            break;
        case OP_GRAM_A:
        case OP_GRAM_B:
        case OP_GRAM_CA:
        case OP_GRAM_CB: {
            const float* Y = (op == OP_GRAM_A) ? md.Ya : (op == OP_GRAM_B) ? md.Yb : md.Yc;
            v.A = Y; v.sAi = 1; v.sAk = md.l;
            v.B = Y; v.sBk = md.l; v.sBj = 1;
            v.M = md.l; v.N = md.l; v.Nvalid = md.l;
            v.K = (op == OP_GRAM_A || op == OP_GRAM_CA) ? md.m : md.n;
            v.C = md.T; v.ldc = md.lp; v.epi = EPI_F64;
            break;
        }
        case OP_APPLY_A2C:
        case OP_APPLY_B2C:
        case OP_APPLY_C2A:
        case OP_APPLY_C2B: {
            const bool rows_m = (op == OP_APPLY_A2C || op == OP_APPLY_C2A);
            v.A = (op == OP_APPLY_A2C) ? md.Ya : (op == OP_APPLY_B2C) ? md.Yb : md.Yc;
            v.sAi = md.l; v.sAk = 1;
            v.B = md.Linv; v.sBk = 1; v.sBj = md.lp;          // B(k, j) = Linv[j][k]
            v.M = rows_m ? md.m : md.n; v.N = md.l; v.Nvalid = md.l; v.K = md.l;
            v.C = (op == OP_APPLY_C2A) ? md.Ya : (op == OP_APPLY_C2B) ? md.Yb : md.Yc;
            v.ldc = md.l;
            break;
        }
        case OP_QT_G:
            v.A = md.Ya; v.sAi = 1; v.sAk = md.l;
            v.B = G; v.sBk = md.ld_g; v.sBj = 1; v.b_bf16 = gb;
            v.M = md.l; v.N = md.ldn; v.Nvalid = md.n; v.K = md.m;
            v.C = md.Bm; v.ldc = md.ldn;
            break;
        case OP_B_BT:
            v.A = md.Bm; v.sAi = md.ldn; v.sAk = 1;
            v.B = md.Bm; v.sBk = 1; v.sBj = md.ldn;
            v.M = md.l; v.N = md.l; v.Nvalid = md.l; v.K = md.n;
            v.C = md.T; v.ldc = md.lp; v.epi = EPI_F64;
            break;
        case OP_ROTATE:   // P = Ya * Urot, Urot (l x r, float) staged in Bm
            v.A = md.Ya; v.sAi = md.l; v.sAk = 1;
            v.B = md.Bm; v.sBk = md.r; v.sBj = 1;
            v.M = md.m; v.N = md.r; v.Nvalid = md.r; v.K = md.l;
            v.C = md.P; v.ldc = md.r;
            break;
        case OP_GRAM_P:
            v.A = md.P; v.sAi = 1; v.sAk = md.r;
            v.B = md.P; v.sBk = md.r; v.sBj = 1;
            v.M = md.r; v.N = md.r; v.Nvalid = md.r; v.K = md.m;
            v.C = md.T; v.ldc = md.lp; v.epi = EPI_F64;
            break;
        case OP_APPLY_P2A:
        default:
            v.A = md.P; v.sAi = md.r; v.sAk = 1;
            v.B = md.Linv; v.sBk = 1; v.sBj = md.lp;
            v.M = md.m; v.N = md.r; v.Nvalid = md.r; v.K = md.r;
            v.C = md.Ya; v.ldc = md.r;
            break;
    }
    return v;
}

void gemm_f32_dims(int op, const MatDev& md, int* M, int* N) {
    GemmView v = gemm_view(op, md, nullptr, NG_F32);
    *M = v.M;
    *N = v.N;
}

__device__ __forceinline__ float load_elem(const void* p, long long idx, int is_bf16) {
    if (is_bf16) {
        unsigned int u = (unsigned int)reinterpret_cast<const unsigned short*>(p)[idx];
        return __uint_as_float(u << 16);
    }
    return reinterpret_cast<const float*>(p)[idx];
}

constexpr int TS = 64;   // tile side
constexpr int BK = 16;
constexpr int LDT = TS + 4;

__global__ __launch_bounds__(256) void k_gemm_f32(int op, const MatDev* __restrict__ mats,
                                                  const MatDyn* __restrict__ dyn, int grad_dtype,
                                                  StepScalars sc) {
    __shared__ float As[BK][LDT];
    __shared__ float Bs[BK][LDT];
    const MatDev& md = mats[blockIdx.z];
    const GemmView v = gemm_view(op, md, &dyn[blockIdx.z], grad_dtype);
    const int i0 = blockIdx.y * TS, j0 = blockIdx.x * TS;
    if (i0 >= v.M || j0 >= v.N) return;

    const int t = threadIdx.x;
    const int lane = t & 63, wv = t >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int li = lane & 31, h = lane >> 5;

    // loader mappings: 4 elements per thread for each operand
    const bool a_i_fast = (v.sAi == 1);
    const bool b_j_fast = (v.sBj == 1);
    int ai[4], ak[4], bk[4], bj[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        if (a_i_fast) { ai[p] = t & 63; ak[p] = (t >> 6) + 4 * p; }
        else          { ak[p] = t & 15; ai[p] = (t >> 4) + 16 * p; }
        if (b_j_fast) { bj[p] = t & 63; bk[p] = (t >> 6) + 4 * p; }
        else          { bk[p] = t & 15; bj[p] = (t >> 4) + 16 * p; }
    }

    floatx16 acc;
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[x] = 0.f;

    float ra[4], rb[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int i = i0 + ai[p], k = k0 + ak[p];
            ra[p] = (i < v.M && k < v.K) ? load_elem(v.A, (long long)i * v.sAi + (long long)k * v.sAk, v.a_bf16) : 0.f;
            const int kb = k0 + bk[p], j = j0 + bj[p];
            rb[p] = (kb < v.K && j < v.Nvalid) ? load_elem(v.B, (long long)kb * v.sBk + (long long)j * v.sBj, v.b_bf16) : 0.f;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            As[ak[p]][ai[p]] = ra[p];
            Bs[bk[p]][bj[p]] = rb[p];
        }
    };

    const int nk = (v.K + BK - 1) / BK;
    fetch(0);
    stage();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) fetch((kt + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const float a = As[kk + h][wm * 32 + li];
            const float b = Bs[kk + h][wn * 32 + li];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
        if (kt + 1 < nk) stage();
        __syncthreads();
    }

    const int col = j0 + wn * 32 + li;
    if (col >= v.N) return;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int row = i0 + wm * 32 + 8 * g + 4 * h + e;
            if (row < v.M) {
                const float x = acc[4 * g + e];
                const long long idx = (long long)row * v.ldc + col;
                if (v.epi == EPI_F32) {
                    reinterpret_cast<float*>(v.C)[idx] = x;
                } else if (v.epi == EPI_F64) {
                    reinterpret_cast<double*>(v.C)[idx] = (double)x;
                } else {
                    float* W = reinterpret_cast<float*>(v.C);
                    const float w = W[idx];
                    W[idx] = w - (sc.lr_scale * x + sc.lr_wd * w);
                }
            }
        }
    }
}

hipError_t launch_gemm_f32(GemmOp op, const MatDev* mats, const MatDyn* dyn, int n_mats, int max_tiles_i,
                           int max_tiles_j, int grad_dtype, StepScalars sc, hipStream_t stream) {
    dim3 g(max_tiles_j, max_tiles_i, n_mats);
    hipLaunchKernelGGL(k_gemm_f32, g, dim3(256), 0, stream, (int)op, mats, dyn, grad_dtype, sc);
    return hipGetLastError();
}

}  // namespace ng
