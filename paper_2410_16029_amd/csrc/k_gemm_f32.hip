// Grouped fp32 GEMM on the fp32 MFMA (v_mfma_f32_32x32x2_f32), one launch for
// all matrices of the layer set.  It serves the NG_F32 step (projection
// R = P^T G, paper Sec. 1; update W -= lr (scale P N + wd W), paper Sec. 2.2)
// and every dense product of the projector refresh.  Operands are described as
// strided views A(i,k), B(k,j) so one kernel covers all transpositions; an
// operand may be stored as float or bf16 (gradients).
//
// Tile 128 x 128 per workgroup (4 wavefronts of 64 x 64), BK = 16, two LDS tile buffers (one barrier
// per k-step) and two register sets (a tile's loads are issued two k-steps ahead).
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
    long long sAi, sAk, sBk, sBj, ldc;     // C is always row-major with leading dimension ldc
    int M, N, K;      // C is M x N, contraction length K
    int Nvalid;       // columns j >= Nvalid of B read as zero (padding columns of the r x ldn space)
    int a_bf16, b_bf16;
    int epi;
    int b_tri;        // B(k, j) = 0 for k > j (the transposed inverse Cholesky factor): a tile stops at its last column
    int sym;          // C = X^T X (fp64): only tiles on or below the diagonal are computed, each as two halves of
                      // the contraction added into a zeroed C
};

__host__ __device__ inline GemmView gemm_view(int op, const MatDev& md, const MatDyn* dy, int grad_dtype,
                                              int slot = 0, int hist_bf16 = 0) {
    GemmView v;
    v.a_bf16 = 0;
    v.b_bf16 = 0;
    v.epi = EPI_F32;
    v.b_tri = 0;
    v.sym = 0;
    const int gb = (grad_dtype == NG_BF16) ? 1 : 0;
    const void* G = dy ? dy->g : nullptr;
    // Strides of the m x n matrix the kernels see inside the caller's row-major gradient: for the
    // right side that matrix is the transpose of the caller's.
    const bool right = md.side == NG_SIDE_RIGHT;
    const long long g_row = right ? 1 : md.ld_g, g_col = right ? md.ld_g : 1;
    switch (op) {
        case OP_PROJECT_F32:
            v.A = md.P; v.sAi = 1; v.sAk = md.r;
            v.B = G; v.sBk = g_row; v.sBj = g_col; v.b_bf16 = gb;
            v.M = md.r; v.N = md.ldn; v.Nvalid = md.n; v.K = md.m;
            v.C = md.H + (long long)(dy ? dy->head : 0) * md.slot_elems; v.ldc = md.ldn;
            break;
        case OP_UPDATE_F32:
            if (!right) {       // W (m x n) -= P N
                v.A = md.P; v.sAi = md.r; v.sAk = 1;
                v.B = md.N; v.sBk = md.ldn; v.sBj = 1;
                v.M = md.m; v.N = md.n; v.Nvalid = md.n;
            } else {            // the caller's W is n x m here: W -= N^T P^T, in W's own orientation
                v.A = md.N; v.sAi = 1; v.sAk = md.ldn;
                v.B = md.P; v.sBk = 1; v.sBj = md.r;
                v.M = md.n; v.N = md.m; v.Nvalid = md.m;
            }
            v.K = md.r;
            v.C = dy ? dy->w : nullptr; v.ldc = md.ld_w; v.epi = EPI_W_F32;
            break;
        case OP_G_B2A:
        case OP_G_C2A:
            v.A = G; v.sAi = g_row; v.sAk = g_col; v.a_bf16 = gb;
            v.B = (op == OP_G_B2A) ? md.Yb : md.Yc; v.sBk = md.l; v.sBj = 1;
            v.M = md.m; v.N = md.l; v.Nvalid = md.l; v.K = md.n;
            v.C = md.Ya; v.ldc = md.l;
            break;
        case OP_GT_C2B:
            v.A = G; v.sAi = g_col; v.sAk = g_row; v.a_bf16 = gb;
            v.B = md.Yc; v.sBk = md.l; v.sBj = 1;
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
            v.C = md.T; v.ldc = md.lp; v.epi = EPI_F64; v.sym = 1;
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
            v.ldc = md.l; v.b_tri = 1;
            break;
        }
        case OP_QT_G:
            v.A = md.Ya; v.sAi = 1; v.sAk = md.l;
            v.B = G; v.sBk = g_row; v.sBj = g_col; v.b_bf16 = gb;
            v.M = md.l; v.N = md.ldn; v.Nvalid = md.n; v.K = md.m;
            v.C = md.Bm; v.ldc = md.ldn;
            break;
        case OP_B_BT:
            v.A = md.Bm; v.sAi = md.ldn; v.sAk = 1;
            v.B = md.Bm; v.sBk = 1; v.sBj = md.ldn;
            v.M = md.l; v.N = md.l; v.Nvalid = md.l; v.K = md.n;
            v.C = md.T; v.ldc = md.lp; v.epi = EPI_F64; v.sym = 1;
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
            v.C = md.T; v.ldc = md.lp; v.epi = EPI_F64; v.sym = 1;
            break;
        case OP_T_CARRY:   // change of basis T = P_new^T P_old, P_old saved in Yc
            v.A = md.P; v.sAi = 1; v.sAk = md.r;
            v.B = md.Yc; v.sBk = md.r; v.sBj = 1;
            v.M = md.r; v.N = md.r; v.Nvalid = md.r; v.K = md.m;
            v.C = md.Linv; v.ldc = md.lp;
            break;
        case OP_CARRY_SLOT:   // carry = T H[slot]
            v.A = md.Linv; v.sAi = md.lp; v.sAk = 1;
            if (hist_bf16) v.B = reinterpret_cast<const unsigned short*>(md.H) + (long long)slot * md.slot_elems;
            else v.B = md.H + (long long)slot * md.slot_elems;
            v.b_bf16 = hist_bf16;
            v.sBk = md.ldn; v.sBj = 1;
            v.M = md.r; v.N = md.ldn; v.Nvalid = md.ldn; v.K = md.r;
            v.C = md.carry; v.ldc = md.ldn;
            break;
        case OP_APPLY_P2A:
        default:
            v.A = md.P; v.sAi = md.r; v.sAk = 1;
            v.B = md.Linv; v.sBk = 1; v.sBj = md.lp;
            v.M = md.m; v.N = md.r; v.Nvalid = md.r; v.K = md.r;
            v.C = md.Ya; v.ldc = md.r; v.b_tri = 1;
            break;
    }
    return v;
}

void gemm_f32_dims(int op, const MatDev& md, int* M, int* N, int* K) {
    GemmView v = gemm_view(op, md, nullptr, NG_F32);
    *M = v.M;
    *N = v.N;
    *K = v.K;
}

#define NG_AS1 __attribute__((address_space(1)))
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef f32x4_t __attribute__((aligned(4))) f32x4_a4;          // 16-byte access at 4-byte alignment
typedef unsigned short u16x4_t __attribute__((ext_vector_type(4)));
typedef u16x4_t __attribute__((aligned(2))) u16x4_a2;          // 8-byte access at 2-byte alignment

__device__ __forceinline__ float load_elem(const NG_AS1 void* p, long long idx, int is_bf16) {
    if (is_bf16) {
        unsigned int u = (unsigned int)reinterpret_cast<const NG_AS1 unsigned short*>(p)[idx];
        return __uint_as_float(u << 16);
    }
    return reinterpret_cast<const NG_AS1 float*>(p)[idx];
}

// Four operand elements along the operand's contiguous dimension, starting at (fast index f, slow
// index s): one vector load when all four exist, element loads with zero fill at the edges.
__device__ __forceinline__ f32x4_t load_vec4(const NG_AS1 void* p, long long base, int f, int f_lim, bool s_ok,
                                             int is_bf16) {
    f32x4_t o = {0.f, 0.f, 0.f, 0.f};
    if (!s_ok || f >= f_lim) return o;
    if (f + 4 <= f_lim) {
        if (is_bf16) {
            const u16x4_t v = *reinterpret_cast<const NG_AS1 u16x4_a2*>(reinterpret_cast<const NG_AS1 unsigned short*>(p) + base);
            o.x = __uint_as_float((unsigned int)v.x << 16);
            o.y = __uint_as_float((unsigned int)v.y << 16);
            o.z = __uint_as_float((unsigned int)v.z << 16);
            o.w = __uint_as_float((unsigned int)v.w << 16);
        } else {
            o = *reinterpret_cast<const NG_AS1 f32x4_a4*>(reinterpret_cast<const NG_AS1 float*>(p) + base);
        }
        return o;
    }
    o.x = load_elem(p, base, is_bf16);
    if (f + 1 < f_lim) o.y = load_elem(p, base + 1, is_bf16);
    if (f + 2 < f_lim) o.z = load_elem(p, base + 2, is_bf16);
    return o;
}

// Four consecutive operand elements (float or bf16) from a byte address, as floats.
template <bool BF>
__device__ __forceinline__ f32x4_t load4(const NG_AS1 unsigned char* p) {
    if (BF) {
        const u16x4_t u = *reinterpret_cast<const NG_AS1 u16x4_a2*>(p);
        f32x4_t o;
        o.x = __uint_as_float((unsigned int)u.x << 16);
        o.y = __uint_as_float((unsigned int)u.y << 16);
        o.z = __uint_as_float((unsigned int)u.z << 16);
        o.w = __uint_as_float((unsigned int)u.w << 16);
        return o;
    }
    return *reinterpret_cast<const NG_AS1 f32x4_a4*>(p);
}

// Tile TS x TS per workgroup (128: four wavefronts of 64 x 64 = 2 x 2 MFMA blocks of 32 x 32; 64: one
// block per wavefront, for products with a short side or a short contraction), BK = 16.  Each
// thread moves 4-element vectors per operand and k-step, taken along the operand's contiguous
// dimension (tile index or contraction index, whichever has stride 1).
// ABF / BBF: operand A / B is stored as bf16.  zero16: 16 bytes of zeros in device memory.
template <int TS, int BK, bool ABF, bool BBF>
__global__ __launch_bounds__(256) void k_gemm_f32(int op, const MatDev* __restrict__ mats,
                                                  const MatDyn* __restrict__ dyn, int grad_dtype,
                                                  StepScalars sc, const void* zero16, int nx, int ny) {
    constexpr int LDT = TS + 4;
    constexpr int NB = TS / 64;          // 32 x 32 blocks per wavefront and dimension
    constexpr int NV = TS * BK / 1024;   // vectors per thread, operand and k-step
    constexpr int KT = BK / 4;           // threads along the contraction index (k-fast mapping)
    constexpr int RPP = 256 / KT;        // tile rows per pass of the k-fast mapping
    constexpr int TPR = TS / 4;          // threads along the tile index (tile-fast mapping)
    __shared__ __attribute__((aligned(16))) float Asm[2][BK][LDT];   // two tile buffers: one barrier per k-step
    __shared__ __attribute__((aligned(16))) float Bsm[2][BK][LDT];
    const MatDev& md = mats[blockIdx.z];
    GemmView v = gemm_view(op, md, &dyn[blockIdx.z], grad_dtype, sc.slot, sc.hist_bf16);
    // The grid is 1-D over the tiles of the largest matrix, padded to a multiple of 8: hardware workgroup
    // id w runs on XCD w % 8, and it takes this matrix's tile with logical index (w % 8) per + w / 8, so
    // each XCD works through a contiguous run of the matrix's tiles (the column tiles of one row tile
    // share the rows of A through that XCD's L2).
    const int nxm = (v.N + TS - 1) / TS, nym = (v.M + TS - 1) / TS;   // this matrix's own tiles
    // symmetric results: nym (nym + 1) / 2 tiles, two work items each (the halves of the contraction)
    const int items = v.sym ? nym * (nym + 1) : nxm * nym;
    const int per = (items + 7) / 8;
    const int slot = (int)(blockIdx.x / 8);
    int tile = (int)(blockIdx.x % 8) * per + slot;
    if (slot >= per || tile >= items) return;
    int i0, j0;
    const NG_AS1 void* Ap = (const NG_AS1 void*)v.A;
    const NG_AS1 void* Bp = (const NG_AS1 void*)v.B;
    if (v.sym) {
        const int half = tile & 1;
        tile >>= 1;
        int ti = 0;
        while (tile >= ti + 1) {      // row ti of the triangle holds ti + 1 tiles
            tile -= ti + 1;
            ++ti;
        }
        i0 = ti * TS;
        j0 = tile * TS;
        // second half: the operands start kh further along the contraction
        const int kh = ((v.K + 1) / 2 + BK - 1) / BK * BK;
        if (half) {
            if (kh >= v.K) return;
            Ap = (const NG_AS1 unsigned char*)Ap + (long long)kh * v.sAk * (ABF ? 2 : 4);
            Bp = (const NG_AS1 unsigned char*)Bp + (long long)kh * v.sBk * (BBF ? 2 : 4);
            v.K -= kh;
        } else if (kh < v.K) {
            v.K = kh;
        }
    } else {
        i0 = (tile / nxm) * TS;
        j0 = (tile % nxm) * TS;
    }
    if (v.b_tri && j0 + TS < v.K) v.K = j0 + TS;   // rows k > j of B are zero

    const int t = threadIdx.x;
    const int lane = t & 63, wv = t >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int li = lane & 31, h = lane >> 5;

    // loader mappings: vector q of this thread covers 4 consecutive positions of the stride-1
    // dimension.  tile-fast: positions 4 (t % TPR) of the tile index at k = t / TPR + (256 / TPR) q;
    // k-fast: k = 4 (t % KT) at tile index t / KT + RPP q.
    const bool a_i_fast = (v.sAi == 1);
    const bool b_j_fast = (v.sBj == 1);
    constexpr int KSTEP = 256 / TPR;
    const int tf = 4 * (t % TPR), tk = t / TPR;    // tile-fast mapping
    const int kf = 4 * (t % KT), kt_ = t / KT;     // k-fast mapping

    floatx16 acc[NB][NB];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[a][b][x] = 0.f;

    // Per-thread, per-vector state of the loads, fixed over the contraction: byte offset in k-step 0,
    // whether the vector lies wholly inside the operand along the dimension that does not move
    // (whole), or straddles its end there (part, tile-fast only).  Inside the loop a whole vector is
    // one load from its address (or from the block of zeros once k runs out); only vectors that
    // straddle an operand's end take the element-wise path.
    const NG_AS1 unsigned char* zp = (const NG_AS1 unsigned char*)zero16;
    constexpr int AES = ABF ? 2 : 4, BES = BBF ? 2 : 4;
    long long a_off[NV], b_off[NV];
    unsigned a_whole = 0, a_part = 0, b_whole = 0, b_part = 0;   // bit q
    const long long a_step = (a_i_fast ? (long long)BK * v.sAk : (long long)BK) * AES;
    const long long b_step = (b_j_fast ? (long long)BK * v.sBk : (long long)BK) * BES;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        if (a_i_fast) {
            const int i = i0 + tf;
            a_whole |= (i + 4 <= v.M) ? (1u << q) : 0u;
            a_part |= (i < v.M && i + 4 > v.M) ? (1u << q) : 0u;
            a_off[q] = ((long long)i + (long long)(tk + KSTEP * q) * v.sAk) * AES;
        } else {
            const int i = i0 + kt_ + RPP * q;
            a_whole |= (i < v.M) ? (1u << q) : 0u;
            a_off[q] = ((long long)i * v.sAi + kf) * AES;
        }
        if (b_j_fast) {
            const int j = j0 + tf;
            b_whole |= (j + 4 <= v.Nvalid) ? (1u << q) : 0u;
            b_part |= (j < v.Nvalid && j + 4 > v.Nvalid) ? (1u << q) : 0u;
            b_off[q] = ((long long)(tk + KSTEP * q) * v.sBk + (long long)j) * BES;
        } else {
            const int j = j0 + kt_ + RPP * q;
            b_whole |= (j < v.Nvalid) ? (1u << q) : 0u;
            b_off[q] = ((long long)kf + (long long)j * v.sBj) * BES;
        }
    }
    // Two register sets: a tile's loads are issued two k-steps before it is written to LDS (one step
    // ahead is not enough for operands that stream from HBM).
    f32x4_t ra0[NV], rb0[NV], ra1[NV], rb1[NV];
    auto fetch = [&](int kt, f32x4_t (&ra)[NV], f32x4_t (&rb)[NV]) {
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            {
                const int k = a_i_fast ? k0 + tk + KSTEP * q : k0 + kf;
                const bool w = (a_whole >> q) & 1u;
                const bool ok = w && (a_i_fast ? k < v.K : k + 4 <= v.K);
                const bool part = a_i_fast ? (((a_part >> q) & 1u) && k < v.K) : (w && k < v.K && k + 4 > v.K);
                ra[q] = load4<ABF>(ok ? (const NG_AS1 unsigned char*)Ap + (a_off[q] + kt * a_step) : zp);
                if (part) {
                    if (a_i_fast) {
                        const int i = i0 + tf;
                        ra[q] = load_vec4(Ap, (long long)i + (long long)k * v.sAk, i, v.M, true, ABF);
                    } else {
                        const int i = i0 + kt_ + RPP * q;
                        ra[q] = load_vec4(Ap, (long long)i * v.sAi + (long long)k, k, v.K, true, ABF);
                    }
                }
            }
            {
                const int k = b_j_fast ? k0 + tk + KSTEP * q : k0 + kf;
                const bool w = (b_whole >> q) & 1u;
                const bool ok = w && (b_j_fast ? k < v.K : k + 4 <= v.K);
                const bool part = b_j_fast ? (((b_part >> q) & 1u) && k < v.K) : (w && k < v.K && k + 4 > v.K);
                rb[q] = load4<BBF>(ok ? (const NG_AS1 unsigned char*)Bp + (b_off[q] + kt * b_step) : zp);
                if (part) {
                    if (b_j_fast) {
                        const int j = j0 + tf;
                        rb[q] = load_vec4(Bp, (long long)k * v.sBk + (long long)j, j, v.Nvalid, true, BBF);
                    } else {
                        const int j = j0 + kt_ + RPP * q;
                        rb[q] = load_vec4(Bp, (long long)k + (long long)j * v.sBj, k, v.K, true, BBF);
                    }
                }
            }
        }
    };
    auto stage = [&](const f32x4_t (&ra)[NV], const f32x4_t (&rb)[NV], int buf) {
        float (*As)[LDT] = Asm[buf];
        float (*Bs)[LDT] = Bsm[buf];
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            if (a_i_fast) {
                *reinterpret_cast<f32x4_t*>(&As[tk + KSTEP * q][tf]) = ra[q];
            } else {
                As[kf][kt_ + RPP * q] = ra[q].x;
                As[kf + 1][kt_ + RPP * q] = ra[q].y;
                As[kf + 2][kt_ + RPP * q] = ra[q].z;
                As[kf + 3][kt_ + RPP * q] = ra[q].w;
            }
            if (b_j_fast) {
                *reinterpret_cast<f32x4_t*>(&Bs[tk + KSTEP * q][tf]) = rb[q];
            } else {
                Bs[kf][kt_ + RPP * q] = rb[q].x;
                Bs[kf + 1][kt_ + RPP * q] = rb[q].y;
                Bs[kf + 2][kt_ + RPP * q] = rb[q].z;
                Bs[kf + 3][kt_ + RPP * q] = rb[q].w;
            }
        }
    };

    // 32 x 32 blocks that lie wholly outside the product (the tail tile of a dimension such as
    // l = r + 8) are skipped: their operands are zero fill and their results are never stored.
    bool vx[NB], vy[NB];
#pragma unroll
    for (int x = 0; x < NB; ++x) {
        vx[x] = i0 + wm * (TS / 2) + 32 * x < v.M;
        vy[x] = j0 + wn * (TS / 2) + 32 * x < v.N;
    }
    auto multiply = [&](int buf) {
        const float (*As)[LDT] = Asm[buf];
        const float (*Bs)[LDT] = Bsm[buf];
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a[NB], b[NB];
#pragma unroll
            for (int x = 0; x < NB; ++x) {
                a[x] = As[kk + h][wm * (TS / 2) + 32 * x + li];
                b[x] = Bs[kk + h][wn * (TS / 2) + 32 * x + li];
            }
#pragma unroll
            for (int x = 0; x < NB; ++x)
#pragma unroll
                for (int y = 0; y < NB; ++y)
                    if (vx[x] && vy[y])
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[x], b[y], acc[x][y], 0, 0, 0);
        }
    };

    // Iteration kt: tile kt + 1 goes from its register set into the LDS buffer that tile kt - 1 was read
    // from (everyone has passed the barrier that ended that step), the set is refilled with the loads
    // of tile kt + 3, tile kt is multiplied, one barrier.
    const int nk = (v.K + BK - 1) / BK;
    fetch(0, ra0, rb0);
    stage(ra0, rb0, 0);
    if (nk > 1) fetch(1, ra1, rb1);
    if (nk > 2) fetch(2, ra0, rb0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
        if (kt + 1 < nk) stage(ra1, rb1, 1);
        if (kt + 3 < nk) fetch(kt + 3, ra1, rb1);
        multiply(0);
        __syncthreads();
        if (kt + 1 >= nk) break;
        if (kt + 2 < nk) stage(ra0, rb0, 0);
        if (kt + 4 < nk) fetch(kt + 4, ra0, rb0);
        multiply(1);
        __syncthreads();
    }

#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int bj = 0; bj < NB; ++bj) {
            const int col = j0 + wn * (TS / 2) + bj * 32 + li;
            if (col >= v.N) continue;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = i0 + wm * (TS / 2) + bi * 32 + 8 * g + 4 * h + e;
                    if (row < v.M) {
                        const float x = acc[bi][bj][4 * g + e];
                        const long long idx = (long long)row * v.ldc + col;
                        if (v.epi == EPI_F32) {
                            reinterpret_cast<float*>(v.C)[idx] = x;
                        } else if (v.epi == EPI_F64) {
                            // two addends onto zero: the same sum in either order
                            if (v.sym) unsafeAtomicAdd(reinterpret_cast<double*>(v.C) + idx, (double)x);
                            else reinterpret_cast<double*>(v.C)[idx] = (double)x;
                        } else {
                            float* W = reinterpret_cast<float*>(v.C);
                            const float w = W[idx];
                            W[idx] = w - (sc.lr_scale * x + sc.lr_wd * w);
                        }
                    }
                }
            }
        }
}

// T (lp x lp doubles) of every matrix, the target of the symmetric products
__global__ __launch_bounds__(256) void k_zero_sym_result(const MatDev* __restrict__ mats) {
    const MatDev& md = mats[blockIdx.y];
    const long long total = (long long)md.lp * md.lp;
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < total; q += (long long)gridDim.x * 256)
        md.T[q] = 0.0;
}

// max_m, max_n, max_k: the largest dimensions of this product over the layer set.  The 128 tile is used
// when neither side nor the contraction is short (a short side wastes most of a big tile, a short
// contraction leaves only the read-modify-write of the output, which wants many small workgroups).
template <int TS, int BK>
static void run_gemm_f32(dim3 g, int op, const MatDev* mats, const MatDyn* dyn, int grad_dtype, StepScalars sc,
                         const void* zero16, bool a_bf16, bool b_bf16, bool sym, hipStream_t stream) {
    const int nx = (int)g.x, ny = (int)g.y;
    const int items = sym ? ny * (ny + 1) : nx * ny;
    const dim3 g1((unsigned)((items + 7) / 8 * 8), 1, g.z);
    if (a_bf16)
        k_gemm_f32<TS, BK, true, false><<<g1, dim3(256), 0, stream>>>(op, mats, dyn, grad_dtype, sc, zero16, nx, ny);
    else if (b_bf16)
        k_gemm_f32<TS, BK, false, true><<<g1, dim3(256), 0, stream>>>(op, mats, dyn, grad_dtype, sc, zero16, nx, ny);
    else
        k_gemm_f32<TS, BK, false, false><<<g1, dim3(256), 0, stream>>>(op, mats, dyn, grad_dtype, sc, zero16, nx, ny);
}

hipError_t launch_gemm_f32(GemmOp op, const MatDev* mats, const MatDyn* dyn, int n_mats, int max_m, int max_n,
                           int max_k, int grad_dtype, StepScalars sc, const void* zero16, hipStream_t stream) {
    const bool big = max_m >= 128 && max_n >= 128 && max_k >= 64;
    const int ts = big ? 128 : 64;
    dim3 g((max_n + ts - 1) / ts, (max_m + ts - 1) / ts, n_mats);
    // which operand is stored as bf16 is a property of the product (the same for every matrix)
    const MatDev probe{};
    const GemmView v = gemm_view((int)op, probe, nullptr, grad_dtype, sc.slot, sc.hist_bf16);
    if (v.sym) {   // the halves of the contraction are added into C
        hipLaunchKernelGGL(k_zero_sym_result, dim3(32, n_mats), dim3(256), 0, stream, mats);
    }
    if (big) run_gemm_f32<128, 16>(g, (int)op, mats, dyn, grad_dtype, sc, zero16, v.a_bf16, v.b_bf16, v.sym != 0, stream);
    else run_gemm_f32<64, 16>(g, (int)op, mats, dyn, grad_dtype, sc, zero16, v.a_bf16, v.b_bf16, v.sym != 0, stream);
    return hipGetLastError();
}

}  // namespace ng
