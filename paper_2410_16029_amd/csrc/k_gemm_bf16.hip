// bf16 MFMA GEMMs of the Natural GaLore step for bf16 gradients / weights.
//
//   k_project_bf16   R = P^T G        (paper Sec. 1, projection equation)
//                    A = PbT [r][ldk] (bf16 copy of P^T, contraction index contiguous)
//                    B = G   [m][ld_g] (caller's gradient: contraction index is the ROW, so the tile
//                                       is transposed in registers on its way into LDS)
//                    C -> ring slot `head` of H, float [r][ldn]
//   k_update_bf16    W <- W - lr (scale P N + wd W)   (paper Sec. 2.2, update equation)
//                    A = Pb [m][ldr], B = N in the octet layout [r/8][ldn][8] written by the
//                    transform+Adam kernel (already k-packed: no transpose), epilogue
//                    read-modify-writes W through an LDS-staged tile so every lane touches 16
//                    contiguous bytes of a weight row.
//
// v_mfma_f32_32x32x16_bf16: lane L supplies 8 bf16 of A row (L%32) and 8 bf16 of B column (L%32),
// both for the k-slots 8*(L/32)..+7 of the 16-deep step (any k assignment works as long as A and B
// agree); accumulator index 4*g+e of lane L is D[8*g + 4*(L/32) + e][L%32].
//
// LDS tiles are [row][BK + 8] bf16: the 16-byte pad makes the 16-byte fragment reads of 8
// consecutive rows hit disjoint banks.
#include "ng_internal.h"

namespace ng {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef uint4 __attribute__((aligned(2))) uint4_a2;   // 16-byte access at 2-byte alignment

__device__ __forceinline__ unsigned short f2bf(float x) {
    unsigned int u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf2f(unsigned int lo16) { return __uint_as_float(lo16 << 16); }

template <int BM_, int BN_, int WM_, int WN_, int BK_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_;
    static constexpr int NWM = BM / WM, NWN = BN / WN, NW = NWM * NWN, NT = NW * 64;
    static constexpr int MI = WM / 32, NJ = WN / 32;
    static constexpr int LDS_K = BK + 8;                    // bf16 elements per LDS row
    static constexpr int KC = BK / 8;                       // 16-byte chunks per row
    static constexpr int A_CHUNKS = BM * KC / NT;           // per thread
    static constexpr int BN8_CHUNKS = BN * KC / NT;         // per thread, octet-layout B
    static constexpr int BT_BLOCKS = (BK / 4) * (BN / 8) / NT;   // per thread, transposing B: 4k x 8j blocks
    static constexpr int OPER_BYTES = (BM + BN) * LDS_K * 2;
    static constexpr int LDC = BN + 8;                      // floats per staged C row
    static constexpr int STAGE_BYTES = NWM * 32 * LDC * 4;
    static constexpr int LDS_BYTES = OPER_BYTES > STAGE_BYTES ? OPER_BYTES : STAGE_BYTES;
    static_assert(BM * KC % NT == 0 && BN * KC % NT == 0 && (BK / 4) * (BN / 8) % NT == 0, "tile/thread mismatch");
};

// ---- A operand: bf16 [rows][ld], contraction contiguous; rows >= row_lim and k >= k_lim read as 0
template <class C>
__device__ __forceinline__ void load_a(uint4 (&ra)[C::A_CHUNKS], const bf16_t* __restrict__ A, long long ld,
                                       int row0, int row_lim, int k0, int k_lim, int t) {
#pragma unroll
    for (int p = 0; p < C::A_CHUNKS; ++p) {
        const int c = t + C::NT * p;
        const int row = row0 + c / C::KC, k = k0 + (c % C::KC) * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < row_lim && k < k_lim) v = *reinterpret_cast<const uint4*>(A + (long long)row * ld + k);
        ra[p] = v;
    }
}
template <class C>
__device__ __forceinline__ void store_a(const uint4 (&ra)[C::A_CHUNKS], bf16_t* As, int t) {
#pragma unroll
    for (int p = 0; p < C::A_CHUNKS; ++p) {
        const int c = t + C::NT * p;
        *reinterpret_cast<uint4*>(As + (c / C::KC) * C::LDS_K + (c % C::KC) * 8) = ra[p];
    }
}

// ---- B operand in the octet layout [k/8][ldn][8]
template <class C>
__device__ __forceinline__ void load_b8(uint4 (&rb)[C::BN8_CHUNKS], const bf16_t* __restrict__ N8, int ldn, int roct,
                                        int j0, int k0, int t) {
#pragma unroll
    for (int p = 0; p < C::BN8_CHUNKS; ++p) {
        const int c = t + C::NT * p;
        const int j = j0 + c % C::BN, oct = (k0 >> 3) + c / C::BN;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (j < ldn && oct < roct) v = *reinterpret_cast<const uint4*>(N8 + ((long long)oct * ldn + j) * 8);
        rb[p] = v;
    }
}
template <class C>
__device__ __forceinline__ void store_b8(const uint4 (&rb)[C::BN8_CHUNKS], bf16_t* Bs, int t) {
#pragma unroll
    for (int p = 0; p < C::BN8_CHUNKS; ++p) {
        const int c = t + C::NT * p;
        *reinterpret_cast<uint4*>(Bs + (c % C::BN) * C::LDS_K + (c / C::BN) * 8) = rb[p];
    }
}

// ---- B operand = gradient G [k][ld_g] (k = row): each thread takes 4 rows x 8 columns
template <class C>
__device__ __forceinline__ void load_bt(uint4 (&rb)[C::BT_BLOCKS][4], const bf16_t* __restrict__ G, long long ld_g,
                                        int m, int n, int j0, int k0, int t) {
#pragma unroll
    for (int p = 0; p < C::BT_BLOCKS; ++p) {
        const int b = t + C::NT * p;
        const int jg = b % (C::BN / 8), kg = b / (C::BN / 8);
        const int j = j0 + jg * 8;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = k0 + kg * 4 + q;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (k < m) {
                const bf16_t* src = G + (long long)k * ld_g + j;
                if (j + 8 <= n) {
                    v = *reinterpret_cast<const uint4_a2*>(src);
                } else if (j < n) {
                    unsigned int e[8];
#pragma unroll
                    for (int x = 0; x < 8; ++x) e[x] = (j + x < n) ? (unsigned int)src[x] : 0u;
                    v.x = e[0] | (e[1] << 16);
                    v.y = e[2] | (e[3] << 16);
                    v.z = e[4] | (e[5] << 16);
                    v.w = e[6] | (e[7] << 16);
                }
            }
            rb[p][q] = v;
        }
    }
}
template <class C>
__device__ __forceinline__ void store_bt(const uint4 (&rb)[C::BT_BLOCKS][4], bf16_t* Bs, int t) {
#pragma unroll
    for (int p = 0; p < C::BT_BLOCKS; ++p) {
        const int b = t + C::NT * p;
        const int jg = b % (C::BN / 8), kg = b / (C::BN / 8);
        bf16_t* dst = Bs + (jg * 8) * C::LDS_K + kg * 4;
        const unsigned int* r0 = reinterpret_cast<const unsigned int*>(&rb[p][0]);
        const unsigned int* r1 = reinterpret_cast<const unsigned int*>(&rb[p][1]);
        const unsigned int* r2 = reinterpret_cast<const unsigned int*>(&rb[p][2]);
        const unsigned int* r3 = reinterpret_cast<const unsigned int*>(&rb[p][3]);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint2 even, odd;   // columns 2d and 2d+1: four consecutive k each
            even.x = (r0[d] & 0xffffu) | (r1[d] << 16);
            even.y = (r2[d] & 0xffffu) | (r3[d] << 16);
            odd.x = (r0[d] >> 16) | (r1[d] & 0xffff0000u);
            odd.y = (r2[d] >> 16) | (r3[d] & 0xffff0000u);
            *reinterpret_cast<uint2*>(dst + (2 * d) * C::LDS_K) = even;
            *reinterpret_cast<uint2*>(dst + (2 * d + 1) * C::LDS_K) = odd;
        }
    }
}

// ---- one BK-deep MFMA sweep over the LDS tiles
template <class C>
__device__ __forceinline__ void mma_tile(floatx16 (&acc)[C::MI][C::NJ], const bf16_t* As, const bf16_t* Bs, int wm,
                                         int wn, int li, int h) {
#pragma unroll
    for (int kk = 0; kk < C::BK / 16; ++kk) {
        bf16x8_t a[C::MI], b[C::NJ];
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi) {
            uint4 v = *reinterpret_cast<const uint4*>(As + (wm * C::WM + mi * 32 + li) * C::LDS_K + kk * 16 + h * 8);
            a[mi] = *reinterpret_cast<bf16x8_t*>(&v);
        }
#pragma unroll
        for (int nj = 0; nj < C::NJ; ++nj) {
            uint4 v = *reinterpret_cast<const uint4*>(Bs + (wn * C::WN + nj * 32 + li) * C::LDS_K + kk * 16 + h * 8);
            b[nj] = *reinterpret_cast<bf16x8_t*>(&v);
        }
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
            for (int nj = 0; nj < C::NJ; ++nj)
                acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[nj], acc[mi][nj], 0, 0, 0);
    }
}

// =================================================================== projection
template <class C>
__global__ __launch_bounds__(C::NT) void k_project_bf16(const MatDev* __restrict__ mats,
                                                        const MatDyn* __restrict__ dyn,
                                                        const TileRef* __restrict__ tiles) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* As = reinterpret_cast<bf16_t*>(smem);
    bf16_t* Bs = As + C::BM * C::LDS_K;

    const TileRef tr = tiles[blockIdx.x];
    if (tr.mat < 0) return;   // padding entry of the XCD-ordered table
    const MatDev& md = mats[tr.mat];
    const MatDyn dy = dyn[tr.mat];
    const int i0 = tr.ti * C::BM, j0 = tr.tj * C::BN;
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv / C::NWN, wn = wv % C::NWN, li = lane & 31, h = lane >> 5;
    const int m = md.m, n = md.n, r = md.r, ldn = md.ldn;
    const bf16_t* __restrict__ A = md.PbT;
    const bf16_t* __restrict__ G = reinterpret_cast<const bf16_t*>(dy.g);

    floatx16 acc[C::MI][C::NJ];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int nj = 0; nj < C::NJ; ++nj)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[mi][nj][x] = 0.f;

    uint4 ra[C::A_CHUNKS];
    uint4 rb[C::BT_BLOCKS][4];
    const int nk = (m + C::BK - 1) / C::BK;
    load_a<C>(ra, A, md.ldk, i0, r, 0, md.ldk, t);
    load_bt<C>(rb, G, md.ld_g, m, n, j0, 0, t);
    store_a<C>(ra, As, t);
    store_bt<C>(rb, Bs, t);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) {
            load_a<C>(ra, A, md.ldk, i0, r, (kt + 1) * C::BK, md.ldk, t);
            load_bt<C>(rb, G, md.ld_g, m, n, j0, (kt + 1) * C::BK, t);
        }
        mma_tile<C>(acc, As, Bs, wm, wn, li, h);
        __syncthreads();
        if (kt + 1 < nk) {
            store_a<C>(ra, As, t);
            store_bt<C>(rb, Bs, t);
        }
        __syncthreads();
    }

    float* __restrict__ R = md.H + (long long)dy.head * md.slot_elems;
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int nj = 0; nj < C::NJ; ++nj) {
            const int col = j0 + wn * C::WN + nj * 32 + li;
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = i0 + wm * C::WM + mi * 32 + 8 * g + 4 * h + e;
                    if (row < r && col < ldn) R[(long long)row * ldn + col] = acc[mi][nj][4 * g + e];
                }
        }
}

// =================================================================== update
template <class C>
__global__ __launch_bounds__(C::NT) void k_update_bf16(const MatDev* __restrict__ mats,
                                                       const MatDyn* __restrict__ dyn,
                                                       const TileRef* __restrict__ tiles, StepScalars sc) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* As = reinterpret_cast<bf16_t*>(smem);
    bf16_t* Bs = As + C::BM * C::LDS_K;
    float* Cs = reinterpret_cast<float*>(smem);

    const TileRef tr = tiles[blockIdx.x];
    if (tr.mat < 0) return;   // padding entry of the XCD-ordered table
    const MatDev& md = mats[tr.mat];
    const MatDyn dy = dyn[tr.mat];
    const int i0 = tr.ti * C::BM, j0 = tr.tj * C::BN;
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv / C::NWN, wn = wv % C::NWN, li = lane & 31, h = lane >> 5;
    const int m = md.m, n = md.n, ldn = md.ldn;
    const int kdim = md.roct * 8;
    const bf16_t* __restrict__ A = md.Pb;
    const bf16_t* __restrict__ N8 = reinterpret_cast<const bf16_t*>(md.N);

    floatx16 acc[C::MI][C::NJ];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int nj = 0; nj < C::NJ; ++nj)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[mi][nj][x] = 0.f;

    uint4 ra[C::A_CHUNKS];
    uint4 rb[C::BN8_CHUNKS];
    const int nk = (kdim + C::BK - 1) / C::BK;
    load_a<C>(ra, A, md.ldr, i0, m, 0, md.ldr, t);
    load_b8<C>(rb, N8, ldn, md.roct, j0, 0, t);
    store_a<C>(ra, As, t);
    store_b8<C>(rb, Bs, t);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) {
            load_a<C>(ra, A, md.ldr, i0, m, (kt + 1) * C::BK, md.ldr, t);
            load_b8<C>(rb, N8, ldn, md.roct, j0, (kt + 1) * C::BK, t);
        }
        mma_tile<C>(acc, As, Bs, wm, wn, li, h);
        __syncthreads();
        if (kt + 1 < nk) {
            store_a<C>(ra, As, t);
            store_b8<C>(rb, Bs, t);
        }
        __syncthreads();
    }

    // Epilogue, one 32-row block of every wave-row at a time: accumulators -> LDS (float),
    // then each thread read-modify-writes 8 consecutive bf16 of one weight row.
    bf16_t* __restrict__ W = reinterpret_cast<bf16_t*>(dy.w);
    const long long ld_w = md.ld_w;
    constexpr int ROWS = C::NWM * 32;
    constexpr int CH = C::BN / 8;                         // 8-column chunks per row
    constexpr int PER_T = ROWS * CH / C::NT;
    static_assert(ROWS * CH % C::NT == 0, "epilogue mapping");
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) {
#pragma unroll
        for (int nj = 0; nj < C::NJ; ++nj)
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    Cs[(wm * 32 + 8 * g + 4 * h + e) * C::LDC + wn * C::WN + nj * 32 + li] = acc[mi][nj][4 * g + e];
        __syncthreads();
#pragma unroll
        for (int p = 0; p < PER_T; ++p) {
            const int q = t + C::NT * p;
            const int lr = q / CH, cc = q % CH;
            const int row = i0 + (lr / 32) * C::WM + mi * 32 + (lr % 32);
            const int col = j0 + cc * 8;
            if (row < m && col < n) {
                const float* cp = Cs + lr * C::LDC + cc * 8;
                const float4 c0 = *reinterpret_cast<const float4*>(cp);
                const float4 c1 = *reinterpret_cast<const float4*>(cp + 4);
                const float cv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
                bf16_t* wp = W + (long long)row * ld_w + col;
                if (col + 8 <= n) {
                    const uint4 wv4 = *reinterpret_cast<const uint4_a2*>(wp);
                    const unsigned int wi[4] = {wv4.x, wv4.y, wv4.z, wv4.w};
                    unsigned int wo[4];
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const float w0 = bf2f(wi[d] & 0xffffu), w1 = __uint_as_float(wi[d] & 0xffff0000u);
                        const float n0 = w0 - (sc.lr_scale * cv[2 * d] + sc.lr_wd * w0);
                        const float n1 = w1 - (sc.lr_scale * cv[2 * d + 1] + sc.lr_wd * w1);
                        wo[d] = (unsigned int)f2bf(n0) | ((unsigned int)f2bf(n1) << 16);
                    }
                    *reinterpret_cast<uint4_a2*>(wp) = make_uint4(wo[0], wo[1], wo[2], wo[3]);
                } else {
#pragma unroll
                    for (int x = 0; x < 8; ++x)
                        if (col + x < n) {
                            const float w0 = bf2f((unsigned int)wp[x]);
                            wp[x] = f2bf(w0 - (sc.lr_scale * cv[x] + sc.lr_wd * w0));
                        }
                }
            }
        }
        __syncthreads();
    }
}

// =================================================================== launchers
typedef Cfg<128, 128, 64, 64, 64> CfgA;

static int g_attr_done = 0;

hipError_t launch_project_bf16(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles,
                               hipStream_t stream) {
    if (n_tiles == 0) return hipSuccess;
    if (!(g_attr_done & 1)) {
        hipFuncSetAttribute(reinterpret_cast<const void*>(k_project_bf16<CfgA>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, CfgA::LDS_BYTES);
        g_attr_done |= 1;
    }
    hipLaunchKernelGGL(k_project_bf16<CfgA>, dim3(n_tiles), dim3(CfgA::NT), CfgA::LDS_BYTES, stream, mats, dyn,
                       tiles);
    return hipGetLastError();
}

hipError_t launch_update_bf16(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles,
                              StepScalars sc, hipStream_t stream) {
    if (n_tiles == 0) return hipSuccess;
    if (!(g_attr_done & 2)) {
        hipFuncSetAttribute(reinterpret_cast<const void*>(k_update_bf16<CfgA>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, CfgA::LDS_BYTES);
        g_attr_done |= 2;
    }
    hipLaunchKernelGGL(k_update_bf16<CfgA>, dim3(n_tiles), dim3(CfgA::NT), CfgA::LDS_BYTES, stream, mats, dyn,
                       tiles, sc);
    return hipGetLastError();
}

void bf16_tile_shape(int* bm, int* bn) {
    *bm = CfgA::BM;
    *bn = CfgA::BN;
}

}  // namespace ng
