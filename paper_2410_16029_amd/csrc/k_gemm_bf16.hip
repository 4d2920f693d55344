// bf16 MFMA GEMMs of the Natural GaLore step for bf16 gradients / weights.
//
//   k_project_bf16_dl  R = P^T G      (paper Sec. 1, projection equation), left side
//                    A = PbT (bf16 copy of P^T, k-blocked [ldk/32][r][32]), B = the caller's gradient
//                    G [m][ld_g] (contraction index = row).  16-byte chunks of both go from memory
//                    straight into LDS; the gradient's MFMA fragments (8 consecutive k of one
//                    column) are assembled by transposing LDS reads.
//                    C -> ring slot `head` of H, float or bf16 [r][ldn]
//   k_project_bf16   the same product with register-staged operands: the right side (the problem is
//                    transposed and the gradient's rows are contraction-contiguous columns) and
//                    left-side gradients of fewer than 8 columns (tile transposed in registers)
//   k_update_bf16_dl W <- W - lr (scale P N + wd W)   (paper Sec. 2.2, update equation)
//                    A = Pb (k-blocked [ldr/32][m][32]), B = N in the octet layout [r/8][ldn][8]
//                    written by the transform+Adam kernel (both k-packed: 16-byte chunks go from
//                    memory straight into LDS, no register pass), epilogue read-modify-writes W
//                    through an LDS-staged tile so every lane touches 16 contiguous bytes of a
//                    weight row.
//
// v_mfma_f32_32x32x16_bf16: lane L supplies 8 bf16 of A row (L%32) and 8 bf16 of B column (L%32),
// both for the k-slots 8*(L/32)..+7 of the 16-deep step (any k assignment works as long as A and B
// agree); accumulator index 4*g+e of lane L is D[8*g + 4*(L/32) + e][L%32].
//
// LDS tiles of the register-staged projection are [row][BK + 8] bf16: the 16-byte pad makes the
// 16-byte fragment reads of 16 consecutive rows hit disjoint banks.
//
// Memory access rules followed here (each was measured to matter):
//   * every pointer read out of a table is cast to the global address space, so loads are
//     global_load (not flat_load, which also ticks the LDS counter);
//   * loads are branch-free: an out-of-range row / k / column is clamped to a valid address and
//     the value is zeroed later, when it is written to LDS (register-staged kernel), or fetched
//     from a 16-byte block of zeros (direct-to-LDS kernels) -- a guarded load in its own branch,
//     or a select right after the load, makes the compiler wait for the load before the MFMAs
//     of the current tile instead of after them;
//   * offsets are 32-bit in the register-staged kernel (the host checks that every matrix is
//     below 2 GiB).
#include "ng_internal.h"

namespace ng {

#define NG_AS1 __attribute__((address_space(1)))

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef u32x4_t __attribute__((aligned(2))) u32x4_a2;   // 16-byte access at 2-byte alignment
typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access at 4-byte alignment
typedef const NG_AS1 bf16_t* gbf16_cptr;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two floats -> two bf16 (round to nearest even) in one v_cvt_pk_bf16_f32; a in the low half
__device__ __forceinline__ unsigned int pack_bf16x2(float a, float b) {
    const f32x2_t f = {a, b};
    bf16x2_t hv = __builtin_convertvector(f, bf16x2_t);
    return *reinterpret_cast<unsigned int*>(&hv);
}
__device__ __forceinline__ unsigned int f2bf(float x) { return pack_bf16x2(x, 0.f) & 0xffffu; }
__device__ __forceinline__ u32x4_t zero_unless(bool ok, u32x4_t v) {
    v.x = ok ? v.x : 0u;
    v.y = ok ? v.y : 0u;
    v.z = ok ? v.z : 0u;
    v.w = ok ? v.w : 0u;
    return v;
}

template <int BM_, int BN_, int WM_, int WN_, int BK_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_;
    static constexpr int NWM = BM / WM, NWN = BN / WN, NW = NWM * NWN, NT = NW * 64;
    static constexpr int MI = WM / 32, NJ = WN / 32;
    static constexpr int LDS_K = BK + 8;                    // bf16 elements per LDS row
    static constexpr int KC = BK / 8;                       // 16-byte chunks per row
    static constexpr int KG = BK / 4;                       // 4-row groups of the transposed operand
    static constexpr int A_CHUNKS = BM * KC / NT;           // per thread
    static constexpr int BT_BLOCKS = KG * (BN / 8) / NT;    // per thread, transposing B: 4k x 8j blocks
    static constexpr int OPER_BYTES = (BM + BN) * LDS_K * 2;
    static constexpr int LDC = BN + 8;                      // floats per staged C row
    static constexpr int STAGE_BYTES = NWM * 32 * LDC * 4;
    static constexpr int LDS_BYTES = OPER_BYTES > STAGE_BYTES ? OPER_BYTES : STAGE_BYTES;
    static_assert(BM * KC % NT == 0 && BN * KC % NT == 0 && KG * (BN / 8) % NT == 0, "tile/thread mismatch");
    static_assert(NT % KC == 0 && NT % BN == 0 && NT % KG == 0, "per-thread invariants");
};

// ------------------------------------------------------------------ A operand
// bf16 copy of P^T in the k-blocked layout [k / 32][rows][32] (see MatDev::PbT): element (row, k) at
// ((k / 32) * rows + row) * 32 + k % 32.  Chunk c = t + NT*p: row c / KC, k-chunk c % KC (the same
// k-chunk for every p).  Rows >= row_lim and k >= k_lim are zero (k_lim % 32 == 0).
template <class C>
struct ALoader {
    gbf16_cptr base;
    unsigned rowoff[C::A_CHUNKS];
    unsigned rowok;    // bit p
    unsigned blk;      // elements per 32-deep k-block = rows * 32
    int kofs, k_lim;
    u32x4_t r[C::A_CHUNKS];
    bool kok;

    __device__ __forceinline__ void init(const bf16_t* A, int rows, int row0, int k_lim_, int t) {
        base = (gbf16_cptr)A;
        kofs = (t % C::KC) * 8;
        k_lim = k_lim_;
        blk = (unsigned)rows * 32u;
        rowok = 0;
#pragma unroll
        for (int p = 0; p < C::A_CHUNKS; ++p) {
            const int row = row0 + (t + C::NT * p) / C::KC;
            const bool ok = row < rows;
            rowok |= ok ? (1u << p) : 0u;
            rowoff[p] = (unsigned)(ok ? row : rows - 1) * 32u;
        }
    }
    __device__ __forceinline__ void load(int k0) {
        const int k = k0 + kofs;
        kok = k < k_lim;
        const unsigned kk = (unsigned)(kok ? k : k_lim - 8);
        const unsigned kc = (kk >> 5) * blk + (kk & 31u);
#pragma unroll
        for (int p = 0; p < C::A_CHUNKS; ++p) r[p] = *(const NG_AS1 u32x4_t*)(base + (rowoff[p] + kc));
    }
    __device__ __forceinline__ void store(bf16_t* As, int t) const {
#pragma unroll
        for (int p = 0; p < C::A_CHUNKS; ++p) {
            const int c = t + C::NT * p;
            const bool ok = kok && ((rowok >> p) & 1u);
            *reinterpret_cast<u32x4_t*>(As + (c / C::KC) * C::LDS_K + (c % C::KC) * 8) = zero_unless(ok, r[p]);
        }
    }
};

// ------------------------------------------------------------------ B operand = gradient G [k][ld_g]
// (k = row).  Block b = t + NT*p: 4 rows x 8 columns; kg = b % KG runs fastest over the lanes so
// that the transposed 8-byte LDS stores of one instruction spread over all banks.
// FULL: every 8-column chunk of the tile is either wholly inside or wholly outside the matrix.
template <class C>
struct BTLoader {
    gbf16_cptr base;
    unsigned ld;
    int m, n, kg4;
    unsigned coloff[C::BT_BLOCKS];
    int jcol[C::BT_BLOCKS];
    unsigned colok;   // bit p
    unsigned rowok;   // bit q (set by load)
    u32x4_t r[C::BT_BLOCKS][4];

    __device__ __forceinline__ void init(const void* G, long long ld_g, int m_, int n_, int j0, int t) {
        base = (gbf16_cptr)G;
        ld = (unsigned)ld_g;
        m = m_;
        n = n_;
        kg4 = (t % C::KG) * 4;
        colok = 0;
#pragma unroll
        for (int p = 0; p < C::BT_BLOCKS; ++p) {
            const int jg = (t + C::NT * p) / C::KG;
            const int j = j0 + jg * 8;
            jcol[p] = j;
            const bool ok = j + 8 <= n;
            colok |= ok ? (1u << p) : 0u;
            coloff[p] = (unsigned)(ok ? j : (n >= 8 ? n - 8 : 0));
        }
    }
    template <bool FULL>
    __device__ __forceinline__ void load(int k0) {
        rowok = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = k0 + kg4 + q;
            const bool ok = k < m;
            rowok |= ok ? (1u << q) : 0u;
            const unsigned ro = (unsigned)(ok ? k : m - 1) * ld;
#pragma unroll
            for (int p = 0; p < C::BT_BLOCKS; ++p) {
                if (FULL) {
                    r[p][q] = *(const NG_AS1 u32x4_a2*)(base + (ro + coloff[p]));
                } else {
                    // ragged right edge (n % 8 != 0 and the tile crosses n): element loads
                    u32x4_t v = {0u, 0u, 0u, 0u};
                    const int j = jcol[p];
                    if (j + 8 <= n) {
                        v = *(const NG_AS1 u32x4_a2*)(base + (ro + (unsigned)j));
                    } else if (j < n) {
                        unsigned int e[8];
#pragma unroll
                        for (int x = 0; x < 8; ++x) e[x] = (j + x < n) ? (unsigned int)base[ro + (unsigned)(j + x)] : 0u;
                        v.x = e[0] | (e[1] << 16);
                        v.y = e[2] | (e[3] << 16);
                        v.z = e[4] | (e[5] << 16);
                        v.w = e[6] | (e[7] << 16);
                    }
                    r[p][q] = v;
                }
            }
        }
    }
    template <bool FULL>
    __device__ __forceinline__ void store(bf16_t* Bs, int t) const {
#pragma unroll
        for (int p = 0; p < C::BT_BLOCKS; ++p) {
            const int jg = (t + C::NT * p) / C::KG;
            bf16_t* dst = Bs + (jg * 8) * C::LDS_K + kg4;
            const bool cok = FULL ? ((colok >> p) & 1u) : true;   // the ragged path already zero-filled
            const u32x4_t r0 = zero_unless(cok && (rowok & 1u), r[p][0]);
            const u32x4_t r1 = zero_unless(cok && (rowok & 2u), r[p][1]);
            const u32x4_t r2 = zero_unless(cok && (rowok & 4u), r[p][2]);
            const u32x4_t r3 = zero_unless(cok && (rowok & 8u), r[p][3]);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                u32x2_t even, odd;   // columns 2d and 2d+1: four consecutive k each
                even.x = (r0[d] & 0xffffu) | (r1[d] << 16);
                even.y = (r2[d] & 0xffffu) | (r3[d] << 16);
                odd.x = (r0[d] >> 16) | (r1[d] & 0xffff0000u);
                odd.y = (r2[d] >> 16) | (r3[d] & 0xffff0000u);
                *reinterpret_cast<u32x2_t*>(dst + (2 * d) * C::LDS_K) = even;
                *reinterpret_cast<u32x2_t*>(dst + (2 * d + 1) * C::LDS_K) = odd;
            }
        }
    }
};

// ------------------------------------------------------------------ B operand = rows of G, contraction contiguous
// Right-side projection: B(k, j) = G[j][k], so a tile column is a row of the caller's gradient and
// needs no transpose.  Chunk c = t + NT*p: column c / KC, k-chunk c % KC (the same for every p).
// Columns >= j_lim and k >= k_lim are zero.  K8: k_lim % 8 == 0 (every chunk whole or empty);
// otherwise the one chunk that straddles k_lim is read element by element.
template <class C>
struct BKLoader {
    static constexpr int CH = C::BN * C::KC / C::NT;
    gbf16_cptr base;
    unsigned coloff[CH];
    unsigned colok;    // bit p
    int kofs, k_lim;
    int nvalid;        // elements of the current chunk inside k_lim (0..8), set by load
    u32x4_t r[CH];

    __device__ __forceinline__ void init(const void* G, long long ld, int j0, int j_lim, int k_lim_, int t) {
        base = (gbf16_cptr)G;
        kofs = (t % C::KC) * 8;
        k_lim = k_lim_;
        colok = 0;
#pragma unroll
        for (int p = 0; p < CH; ++p) {
            const int j = j0 + (t + C::NT * p) / C::KC;
            const bool ok = j < j_lim;
            colok |= ok ? (1u << p) : 0u;
            coloff[p] = (unsigned)(ok ? j : j_lim - 1) * (unsigned)ld;
        }
    }
    template <bool K8>
    __device__ __forceinline__ void load(int k0) {
        const int k = k0 + kofs;
        nvalid = k_lim - k;
        nvalid = nvalid < 0 ? 0 : (nvalid > 8 ? 8 : nvalid);
        if (K8 || nvalid == 8 || nvalid == 0) {
            const unsigned kc = (unsigned)(nvalid == 8 ? k : (k_lim >= 8 ? k_lim - 8 : 0));
            if (K8 || k_lim >= 8) {
#pragma unroll
                for (int p = 0; p < CH; ++p) r[p] = *(const NG_AS1 u32x4_a2*)(base + (coloff[p] + kc));
            }
        } else {
#pragma unroll
            for (int p = 0; p < CH; ++p) {
                unsigned int e[8];
#pragma unroll
                for (int x = 0; x < 8; ++x) e[x] = x < nvalid ? (unsigned int)base[coloff[p] + (unsigned)(k + x)] : 0u;
                r[p].x = e[0] | (e[1] << 16);
                r[p].y = e[2] | (e[3] << 16);
                r[p].z = e[4] | (e[5] << 16);
                r[p].w = e[6] | (e[7] << 16);
            }
        }
    }
    __device__ __forceinline__ void store(bf16_t* Bs, int t) const {
#pragma unroll
        for (int p = 0; p < CH; ++p) {
            const int c = t + C::NT * p;
            const bool ok = nvalid > 0 && ((colok >> p) & 1u);
            *reinterpret_cast<u32x4_t*>(Bs + (c / C::KC) * C::LDS_K + (c % C::KC) * 8) = zero_unless(ok, r[p]);
        }
    }
};

template <class C, bool K8>
struct BKView {
    BKLoader<C>& l;
    __device__ __forceinline__ void load(int k0) { l.template load<K8>(k0); }
    __device__ __forceinline__ void store(bf16_t* Bs, int t) const { l.store(Bs, t); }
};

// ------------------------------------------------------------------ one BK-deep MFMA sweep
// Fragments of step kk+1 are read from LDS while the MFMAs of step kk run.
template <class C>
__device__ __forceinline__ void mma_tile(floatx16 (&acc)[C::MI][C::NJ], const bf16_t* As, const bf16_t* Bs, int wm,
                                         int wn, int li, int h) {
    constexpr int KK = C::BK / 16;
    const bf16_t* ap = As + (wm * C::WM + li) * C::LDS_K + h * 8;
    const bf16_t* bp = Bs + (wn * C::WN + li) * C::LDS_K + h * 8;
    u32x4_t a[2][C::MI], b[2][C::NJ];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) a[0][mi] = *reinterpret_cast<const u32x4_t*>(ap + mi * 32 * C::LDS_K);
#pragma unroll
    for (int nj = 0; nj < C::NJ; ++nj) b[0][nj] = *reinterpret_cast<const u32x4_t*>(bp + nj * 32 * C::LDS_K);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int cur = kk & 1, nxt = cur ^ 1;
        if (kk + 1 < KK) {
#pragma unroll
            for (int mi = 0; mi < C::MI; ++mi)
                a[nxt][mi] = *reinterpret_cast<const u32x4_t*>(ap + mi * 32 * C::LDS_K + (kk + 1) * 16);
#pragma unroll
            for (int nj = 0; nj < C::NJ; ++nj)
                b[nxt][nj] = *reinterpret_cast<const u32x4_t*>(bp + nj * 32 * C::LDS_K + (kk + 1) * 16);
        }
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
            for (int nj = 0; nj < C::NJ; ++nj)
                acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    *reinterpret_cast<const bf16x8_t*>(&a[cur][mi]), *reinterpret_cast<const bf16x8_t*>(&b[cur][nj]),
                    acc[mi][nj], 0, 0, 0);
    }
}

template <class C>
__device__ __forceinline__ void zero_acc(floatx16 (&acc)[C::MI][C::NJ]) {
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int nj = 0; nj < C::NJ; ++nj)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[mi][nj][x] = 0.f;
}

// =================================================================== projection
// Adapter: the gradient loader with its FULL flag fixed at compile time.
template <class C, bool FULL>
struct BTView {
    BTLoader<C>& l;
    __device__ __forceinline__ void load(int k0) { l.template load<FULL>(k0); }
    __device__ __forceinline__ void store(bf16_t* Bs, int t) const { l.template store<FULL>(Bs, t); }
};

// Main loop over the contraction.  LA / LB: load(k0) issues the global loads of one BK-deep
// tile into registers, store(ptr, t) writes them (masked) to LDS.  The loads of tile kt+1 are in
// flight during the MFMAs of tile kt; two barriers per k-step.
template <class C, class LA, class LB>
__device__ __forceinline__ void gemm_mainloop(floatx16 (&acc)[C::MI][C::NJ], LA& la, LB& lb, unsigned char* smem,
                                              int nk, int t, int wm, int wn, int li, int h) {
    bf16_t* As0 = reinterpret_cast<bf16_t*>(smem);
    bf16_t* Bs0 = As0 + C::BM * C::LDS_K;
    la.load(0);
    lb.load(0);
    la.store(As0, t);
    lb.store(Bs0, t);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) {
            la.load((kt + 1) * C::BK);
            lb.load((kt + 1) * C::BK);
        }
        mma_tile<C>(acc, As0, Bs0, wm, wn, li, h);
        __syncthreads();
        if (kt + 1 < nk) {
            la.store(As0, t);
            lb.store(Bs0, t);
        }
        __syncthreads();
    }
}

// Accumulators of one projection tile -> ring slot `head`.  Called after a barrier that ends the
// main loop (the bf16 form stages the tile through the operand LDS).
template <class C, bool HB>
__device__ __forceinline__ void project_epilogue(floatx16 (&acc)[C::MI][C::NJ], const MatDev& md, const MatDyn& dy,
                                                 unsigned char* smem, int i0, int j0, int t, int wm, int wn, int li,
                                                 int h) {
    const int r = md.r, ldn = md.ldn, n = md.n;   // columns n..ldn-1 of the slot are zero
    const StatePanel sp = state_panel(r, md.pw, j0);   // a tile lies in one column panel of the slot
    if (!HB) {
        NG_AS1 float* R = (NG_AS1 float*)md.H + (long long)dy.head * md.slot_elems;
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
                        // (two stores under lane masks: a select on the value would pull every
                        // accumulator into an ordinary register at once)
                        if (row < r) {
                            if (col < n) __builtin_nontemporal_store(acc[mi][nj][4 * g + e], &R[sp.at(row, col)]);
                            else if (col < ldn) __builtin_nontemporal_store(0.f, &R[sp.at(row, col)]);
                        }
                    }
            }
    } else {
        // bf16 slot: the tile goes through LDS (float), one 32-row block of every wave-row at a
        // time, so that each thread converts and stores 8 consecutive columns (16 bytes) of a row
        // (the main loop ended on a barrier; ldn % 32 == 0, so a chunk that starts inside a row
        // ends inside it)
        constexpr int ROWS = C::NWM * 32, CH = C::BN / 8, PER_T = ROWS * CH / C::NT;
        static_assert(ROWS * CH % C::NT == 0, "epilogue mapping");
        float* Cs = reinterpret_cast<float*>(smem);
        NG_AS1 bf16_t* Rb = (NG_AS1 bf16_t*)md.H + (long long)dy.head * md.slot_elems;
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
                if (row < r && col < ldn) {
                    const float* cp = Cs + lr * C::LDC + cc * 8;
                    f32x4_t c0 = *reinterpret_cast<const f32x4_t*>(cp);
                    f32x4_t c1 = *reinterpret_cast<const f32x4_t*>(cp + 4);
                    if (col + 8 > n) {   // columns n..ldn-1 of the slot are zero
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            if (col + x >= n) c0[x] = 0.f;
                            if (col + 4 + x >= n) c1[x] = 0.f;
                        }
                    }
                    u32x4_t ov;
                    ov.x = pack_bf16x2(c0.x, c0.y);
                    ov.y = pack_bf16x2(c0.z, c0.w);
                    ov.z = pack_bf16x2(c1.x, c1.y);
                    ov.w = pack_bf16x2(c1.z, c1.w);
                    *(NG_AS1 u32x4_t*)(Rb + sp.at(row, col)) = ov;
                }
            }
            __syncthreads();
        }
    }
}

// HB: the ring slot receives bf16 instead of float.  RIGHT: the right-side form (the kernel's m x n
// problem is the transpose of the caller's gradient: its columns are the gradient's rows).
template <class C, bool HB, bool RIGHT>
__global__ __launch_bounds__(C::NT) void k_project_bf16(const MatDev* __restrict__ mats,
                                                        const MatDyn* __restrict__ dyn,
                                                        const TileRef* __restrict__ tiles) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const TileRef tr = tiles[blockIdx.x];
    if (tr.mat < 0) return;   // padding entry of the XCD-ordered table
    const MatDev& md = mats[tr.mat];
    if ((md.side == NG_SIDE_RIGHT) != RIGHT) return;   // the other instance of the launch pair takes it
    const MatDyn dy = dyn[tr.mat];
    const int i0 = tr.ti * C::BM, j0 = tr.tj * C::BN;
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv / C::NWN, wn = wv % C::NWN, li = lane & 31, h = lane >> 5;
    const int m = md.m, n = md.n, r = md.r, ldn = md.ldn;

    floatx16 acc[C::MI][C::NJ];
    zero_acc<C>(acc);

    ALoader<C> la;
    la.init(md.PbT, r, i0, md.ldk, t);
    const int nk = (m + C::BK - 1) / C::BK;
    if (!RIGHT) {
        BTLoader<C> lb;
        lb.init(dy.g, md.ld_g, m, n, j0, t);
        // uniform per workgroup: are all 8-column chunks of this tile whole?
        const bool full = (n >= 8) && ((n & 7) == 0 || j0 + C::BN <= n);
        if (full) {
            BTView<C, true> v{lb};
            gemm_mainloop<C>(acc, la, v, smem, nk, t, wm, wn, li, h);
        } else {
            BTView<C, false> v{lb};
            gemm_mainloop<C>(acc, la, v, smem, nk, t, wm, wn, li, h);
        }
    } else {
        BKLoader<C> lb;
        lb.init(dy.g, md.ld_g, j0, n, m, t);
        if ((m & 7) == 0) {
            BKView<C, true> v{lb};
            gemm_mainloop<C>(acc, la, v, smem, nk, t, wm, wn, li, h);
        } else {
            BKView<C, false> v{lb};
            gemm_mainloop<C>(acc, la, v, smem, nk, t, wm, wn, li, h);
        }
    }

    project_epilogue<C, HB>(acc, md, dy, smem, i0, j0, t, wm, wn, li, h);
}

// =================================================================== update
// Epilogue of the update: accumulators -> LDS (float), one 32-row block of every wave-row at a
// time, then each thread read-modify-writes 8 consecutive bf16 of one weight row.
template <class C>
struct UpdateTile {
    static constexpr int ROWS = C::NWM * 32;
    static constexpr int CH = C::BN / 8;                         // 8-column chunks per row
    static constexpr int PER_T = ROWS * CH / C::NT;
    static_assert(ROWS * CH % C::NT == 0, "epilogue mapping");
};

// Loads the whole weight tile (8 bf16 per chunk, clamped addresses) -- issued before the main
// loop, so the HBM latency and bandwidth of the weight read overlap the contraction.
template <class C>
__device__ __forceinline__ void update_load_w(u32x4_t (&wv4)[C::MI][UpdateTile<C>::PER_T], const NG_AS1 bf16_t* W,
                                              unsigned ld_w, int m, int n, int i0, int j0, int t) {
    constexpr int CH = UpdateTile<C>::CH, PER_T = UpdateTile<C>::PER_T;
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int p = 0; p < PER_T; ++p) {
            const int q = t + C::NT * p;
            const int lr = q / CH, cc = q % CH;
            const int row = i0 + (lr / 32) * C::WM + mi * 32 + (lr % 32);
            const int col = j0 + cc * 8;
            const unsigned rc = (unsigned)(row < m ? row : m - 1);
            const unsigned jc = (unsigned)((col + 8 <= n) ? col : n - 8);
            // read once, written once: streamed through the L2 so it does not evict the operand panels
            wv4[mi][p] = __builtin_nontemporal_load((const NG_AS1 u32x4_a2*)(W + (rc * ld_w + jc)));
        }
}

template <class C>
__device__ __forceinline__ void update_epilogue(floatx16 (&acc)[C::MI][C::NJ],
                                                u32x4_t (&wv4)[C::MI][UpdateTile<C>::PER_T], bool vec,
                                                bool cols_full, float* Cs, NG_AS1 bf16_t* W, unsigned ld_w, int m, int n, int i0,
                                                int j0, int t, int wm, int wn, int li, int h,
                                                const StepScalars& sc) {
    constexpr int CH = UpdateTile<C>::CH, PER_T = UpdateTile<C>::PER_T;
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
        if (vec) {
#pragma unroll
            for (int p = 0; p < PER_T; ++p) {
                const int q = t + C::NT * p;
                const int lr = q / CH, cc = q % CH;
                const int row = i0 + (lr / 32) * C::WM + mi * 32 + (lr % 32);
                const int col = j0 + cc * 8;
                const float* cp = Cs + lr * C::LDC + cc * 8;
                const f32x4_t c0 = *reinterpret_cast<const f32x4_t*>(cp);
                const f32x4_t c1 = *reinterpret_cast<const f32x4_t*>(cp + 4);
                const float cv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
                u32x4_t ov;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const unsigned wi = wv4[mi][p][d];
                    const float w0 = __uint_as_float(wi << 16), w1 = __uint_as_float(wi & 0xffff0000u);
                    const float n0 = w0 - (sc.lr_scale * cv[2 * d] + sc.lr_wd * w0);
                    const float n1 = w1 - (sc.lr_scale * cv[2 * d + 1] + sc.lr_wd * w1);
                    ov[d] = pack_bf16x2(n0, n1);
                }
                if (row < m && col + 8 <= n)
                    __builtin_nontemporal_store(ov, (NG_AS1 u32x4_a2*)(W + ((unsigned)row * ld_w + (unsigned)col)));
                // the one chunk of a row that straddles column n - 1 (n % 8 != 0: only in the tiles of the
                // last tile column): its leading n - col elements one by one.  The vector loaded for this
                // chunk came from the clamped address n - 8 and is not used.
                if (!cols_full && row < m && col < n && col + 8 > n) {
                    NG_AS1 bf16_t* wp = W + ((unsigned)row * ld_w + (unsigned)col);
#pragma unroll
                    for (int x = 0; x < 7; ++x)
                        if (col + x < n) {
                            const float w0 = __uint_as_float((unsigned int)wp[x] << 16);
                            wp[x] = (bf16_t)f2bf(w0 - (sc.lr_scale * cv[x] + sc.lr_wd * w0));
                        }
                }
            }
        } else {
#pragma unroll
            for (int p = 0; p < PER_T; ++p) {
                const int q = t + C::NT * p;
                const int lr = q / CH, cc = q % CH;
                const int row = i0 + (lr / 32) * C::WM + mi * 32 + (lr % 32);
                const int col = j0 + cc * 8;
                if (row < m && col < n) {
                    const float* cp = Cs + lr * C::LDC + cc * 8;
                    NG_AS1 bf16_t* wp = W + ((unsigned)row * ld_w + (unsigned)col);
#pragma unroll
                    for (int x = 0; x < 8; ++x)
                        if (col + x < n) {
                            const float w0 = __uint_as_float((unsigned int)wp[x] << 16);
                            wp[x] = (bf16_t)f2bf(w0 - (sc.lr_scale * cp[x] + sc.lr_wd * w0));
                        }
                }
            }
        }
        __syncthreads();
    }
}

// =================================================================== update, operands loaded straight into LDS
// Both operands of the update are stored k-packed (Pb rows, the octet layout of N), so a 16-byte
// chunk in memory is exactly one MFMA fragment and no register pass is needed:
// global_load_lds_dwordx4 moves 16 bytes per lane into LDS (lane L of a wavefront writes at
// wave base + 16 L; M0 carries the base).  DBK-deep stages in a ring of NST: the loads of the next
// NST-1 stages are in flight while one stage is multiplied; one barrier per stage.
//   A stage: slot(row, kc) = row * KC + (kc ^ swz(row)), 16 bytes per slot, KC = DBK/8 chunks per
//            row; the XOR spreads the fragment reads of consecutive rows over the banks while the
//            global side stays coalesced (KC lanes cover the contiguous bytes of one row)
//   B stage: slot(kc, col) = kc * BN + col  (64 consecutive columns of one octet per instruction)
// A chunk outside the matrix (row >= m, k >= ldr, octet >= roct, column >= ldn) is fetched from a
// 16-byte block of zeros instead.  The stage ring (NST * (BM + BN) * DBK * 2 bytes) is sized so that
// two workgroups share a CU: one is in its HBM-bound epilogue while the other multiplies.
#define NG_AS3 __attribute__((address_space(3)))

template <class C, int DBK, int NST>
struct DlCfg {
    static constexpr int KC = DBK / 8;
    static constexpr int A_BYTES = C::BM * DBK * 2, B_BYTES = C::BN * DBK * 2, STAGE = A_BYTES + B_BYTES;
    static constexpr int A_INSTR = C::BM * KC / C::NT, B_INSTR = C::BN * KC / C::NT;
    static constexpr int RING = NST * STAGE;
    static constexpr int LDS_BYTES = RING > C::STAGE_BYTES ? RING : C::STAGE_BYTES;
    static_assert(DBK == 32 || DBK == 64, "4 or 8 chunks per row");
    static_assert(C::BM * KC % C::NT == 0 && C::BN * KC % C::NT == 0 && C::BN % 64 == 0, "chunk mapping");
    static_assert(A_INSTR + B_INSTR <= 15, "the wait count of one stage must fit the counter");
};

template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // at most N vector-memory loads still in flight
    static_assert(N >= 0 && N <= 15, "low counter bits only");
    __builtin_amdgcn_s_waitcnt(0x0F70 | N);       // expcnt 7, lgkmcnt 15: not waited for
}

// One operand of the update as a source of 16-byte chunks, R tile rows (of A) or columns (of B):
//   RowMajorSrc: the k-blocked bf16 layout [k / 32][rows][32] of Pb / PbT: the 64 bytes a row gives to
//                one 32-deep stage lie next to those of the neighbouring rows, so a wave-instruction
//                (64 / KC rows) reads 1 KB of consecutive memory; chunk kc of a row sits at LDS slot
//                row * KC + (kc ^ swz(row)).
//   OctetSrc:    the octet layout [r/8][ldn][8] of N.  A wave-instruction covers 64 consecutive
//                rows of one octet; slot kc * R + row.
template <class C, int DBK, int R>
struct RowMajorSrc {
    static constexpr int KC = DBK / 8, INSTR = R * KC / C::NT, RPI = 64 / KC;
    static_assert(DBK == 32, "one 32-deep k-block of the blocked layout per stage");
    const NG_AS1 unsigned char* ptr[INSTR];
    unsigned ok;
    int kc, k_lim;
    long long step;   // bytes from one k-block to the next
    // base: [k_lim / 32][rows][32] bf16; the tile takes rows row0 .. row0 + R - 1
    __device__ __forceinline__ void init(const bf16_t* base, int rows, int k_lim_, int row0, int lane, int wv) {
        const int lrow = lane / KC;
        kc = (lane & 3) ^ ((lrow >> 2) & 3);
        k_lim = k_lim_;
        step = (long long)rows * 64;
        ok = 0;
#pragma unroll
        for (int p = 0; p < INSTR; ++p) {
            const int row = row0 + (p * C::NW + wv) * RPI + lrow;
            const bool in = row < rows;
            ok |= in ? (1u << p) : 0u;
            ptr[p] = (const NG_AS1 unsigned char*)base + ((long long)(in ? row : 0) * 32 + kc * 8) * 2;
        }
    }
    __device__ __forceinline__ void issue(int kt, unsigned char* stage, const NG_AS1 unsigned char* zp, int wv) const {
        const bool kok = kt * DBK + kc * 8 < k_lim;
#pragma unroll
        for (int p = 0; p < INSTR; ++p) {
            const bool in = kok && ((ok >> p) & 1u);
            const NG_AS1 unsigned char* g = in ? ptr[p] + kt * step : zp;
            __builtin_amdgcn_global_load_lds((const NG_AS1 void*)g, (NG_AS3 void*)(stage + (p * C::NW + wv) * 1024), 16,
                                             0, 0);
        }
    }
    // byte offset of the fragment (tile row `row`, k-slot ks) inside the operand's stage
    static __device__ __forceinline__ int frag(int row, int sw, int ks) { return (row * KC + (ks ^ sw)) * 16; }
    static __device__ __forceinline__ int swz(int li) { return (li >> 2) & 3; }
};

template <class C, int DBK, int R>
struct OctetSrc {
    static constexpr int KC = DBK / 8, INSTR = R * KC / C::NT, GR = R / 64;
    const NG_AS1 unsigned char* ptr[INSTR];
    int oct[INSTR];
    bool rowok[INSTR];
    int roct;
    long long step;
    __device__ __forceinline__ void init(const void* base, int ldn, int roct_, int row0, int lane, int wv) {
        roct = roct_;
        step = (long long)ldn * KC * 16;   // KC octets per stage
#pragma unroll
        for (int p = 0; p < INSTR; ++p) {
            const int q = p * C::NW + wv;
            const int row = row0 + (q % GR) * 64 + lane;
            oct[p] = q / GR;
            rowok[p] = row < ldn;
            ptr[p] = (const NG_AS1 unsigned char*)base + ((long long)oct[p] * ldn + (rowok[p] ? row : 0)) * 16;
        }
    }
    __device__ __forceinline__ void issue(int kt, unsigned char* stage, const NG_AS1 unsigned char* zp, int wv) const {
#pragma unroll
        for (int p = 0; p < INSTR; ++p) {
            const bool in = rowok[p] && (kt * KC + oct[p] < roct);
            const NG_AS1 unsigned char* g = in ? ptr[p] + kt * step : zp;
            __builtin_amdgcn_global_load_lds((const NG_AS1 void*)g, (NG_AS3 void*)(stage + (p * C::NW + wv) * 1024), 16,
                                             0, 0);
        }
    }
    static __device__ __forceinline__ int frag(int row, int, int ks) { return (ks * R + row) * 16; }
    static __device__ __forceinline__ int swz(int) { return 0; }
};

// RIGHT: the right-side form.  The tile still covers the caller's weight in its own orientation
// (rows = the weight's rows); the roles of the two stored operands swap: A rows come from the octet
// layout of N (r x ldn with n = the weight's row count), B columns from Pb (one row per weight column).
template <class C, int DBK, int NST, bool RIGHT>
__global__ __launch_bounds__(C::NT) void k_update_bf16_dl(const MatDev* __restrict__ mats,
                                                          const MatDyn* __restrict__ dyn,
                                                          const TileRef* __restrict__ tiles, StepScalars sc,
                                                          const void* zero16) {
    typedef DlCfg<C, DBK, NST> D;
    constexpr int KK = DBK / 16;
    typedef RowMajorSrc<C, DBK, C::BM> ARows;
    typedef OctetSrc<C, DBK, C::BM> AOct;
    typedef RowMajorSrc<C, DBK, C::BN> BRows;
    typedef OctetSrc<C, DBK, C::BN> BOct;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const TileRef tr = tiles[blockIdx.x];
    if (tr.mat < 0) return;   // padding entry of the XCD-ordered table
    const MatDev& md = mats[tr.mat];
    if ((md.side == NG_SIDE_RIGHT) != RIGHT) return;   // the other instance of the launch pair takes it
    const MatDyn dy = dyn[tr.mat];
    const int i0 = tr.ti * C::BM, j0 = tr.tj * C::BN;
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wv / C::NWN, wn = wv % C::NWN, li = lane & 31, h = lane >> 5;
    const int m = RIGHT ? md.n : md.m, n = RIGHT ? md.m : md.n;   // the weight's rows and columns
    const int nk = (md.roct * 8 + DBK - 1) / DBK;

    floatx16 acc[C::MI][C::NJ];
    zero_acc<C>(acc);

    const NG_AS1 unsigned char* zp = (const NG_AS1 unsigned char*)zero16;
    ARows a_rm;
    AOct a_oc;
    BRows b_rm;
    BOct b_oc;
    if (!RIGHT) {
        a_rm.init(md.Pb, m, md.ldr, i0, lane, wv);
        b_oc.init(md.N, md.ldn, md.roct, j0, lane, wv);
    } else {
        a_oc.init(md.N, md.ldn, md.roct, i0, lane, wv);
        b_rm.init(md.Pb, n, md.ldr, j0, lane, wv);
    }
    auto issue = [&](int kt) {
        unsigned char* stage = smem + (kt % NST) * D::STAGE;
        if (!RIGHT) {
            a_rm.issue(kt, stage, zp, wv);
            b_oc.issue(kt, stage + D::A_BYTES, zp, wv);
        } else {
            a_oc.issue(kt, stage, zp, wv);
            b_rm.issue(kt, stage + D::A_BYTES, zp, wv);
        }
    };

    // fragment addresses inside a stage
    const int a_row = wm * C::WM + li;                       // + 32 mi
    const int b_col = wn * C::WN + li;                       // + 32 nj
    const int a_sw = RIGHT ? 0 : ARows::swz(li), b_sw = RIGHT ? BRows::swz(li) : 0;

    // Ring: stage kt lives in buffer kt % NST.  Before stage kt is multiplied, the loads of the
    // stages up to kt + NST - 2 have been issued; waiting until at most (NST - 2) stages' worth of
    // this lane's loads are in flight means stage kt has landed (loads complete in order).  The
    // barrier that follows also tells everyone that buffer (kt - 1) % NST is free, which is where
    // stage kt + NST - 1 goes.
    constexpr int PER_STAGE = D::A_INSTR + D::B_INSTR;
    static_assert(NST == 2 || NST == 3, "ring depth");
    for (int q = 0; q < NST - 1; ++q)
        if (q < nk) issue(q);
    for (int kt = 0; kt < nk; ++kt) {
        if (NST == 3 && kt + 1 < nk) wait_vmcnt<PER_STAGE>();
        else wait_vmcnt<0>();
        // A bare barrier: __syncthreads() would also fence, i.e. wait for the loads just issued.
        // Each wave's fragment reads of the previous stage were consumed by its MFMAs before it
        // arrives here, so the buffer that is refilled next is no longer being read.
        asm volatile("s_barrier" ::: "memory");
        if (kt + NST - 1 < nk) issue(kt + NST - 1);
        const unsigned char* cur = smem + (kt % NST) * D::STAGE;
        u32x4_t a[KK][C::MI], b[KK][C::NJ];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int ks = 2 * kk + h;
#pragma unroll
            for (int mi = 0; mi < C::MI; ++mi)
                a[kk][mi] = *reinterpret_cast<const u32x4_t*>(
                    cur + (RIGHT ? AOct::frag(a_row + 32 * mi, 0, ks) : ARows::frag(a_row + 32 * mi, a_sw, ks)));
#pragma unroll
            for (int nj = 0; nj < C::NJ; ++nj)
                b[kk][nj] = *reinterpret_cast<const u32x4_t*>(
                    cur + D::A_BYTES +
                    (RIGHT ? BRows::frag(b_col + 32 * nj, b_sw, ks) : BOct::frag(b_col + 32 * nj, 0, ks)));
        }
        // all fragment reads of the stage are issued before the first MFMA (left alone, the
        // scheduler reuses a few registers and alternates 4 reads - full wait - 4 MFMAs)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
                for (int nj = 0; nj < C::NJ; ++nj)
                    acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        *reinterpret_cast<const bf16x8_t*>(&a[kk][mi]), *reinterpret_cast<const bf16x8_t*>(&b[kk][nj]),
                        acc[mi][nj], 0, 0, 0);
    }
    __syncthreads();   // every wave is done with the ring: the epilogue stages C through the same LDS

    NG_AS1 bf16_t* W = (NG_AS1 bf16_t*)dy.w;
    const unsigned ld_w = (unsigned)md.ld_w;
    // vec: the weight tile goes through 16-byte accesses (needs 8 columns to clamp an address into);
    // cols_full: no chunk of this tile straddles column n - 1
    const bool vec = n >= 8;
    const bool cols_full = vec && ((n & 7) == 0 || j0 + C::BN <= n);
    u32x4_t wv4[C::MI][UpdateTile<C>::PER_T];
    if (vec) update_load_w<C>(wv4, W, ld_w, m, n, i0, j0, t);
    update_epilogue<C>(acc, wv4, vec, cols_full, reinterpret_cast<float*>(smem), W, ld_w, m, n, i0, j0, t, wm, wn, li, h,
                       sc);
}

// =================================================================== projection, operands loaded straight into LDS
// Left side, gradients of at least 8 columns.  A = PbT rows (RowMajorSrc, as in the update).  B = the caller's gradient G [k][ld_g]: its 16-byte chunks (8 consecutive columns of one
// contraction row, at any 2-byte alignment) go into LDS as they are,
//   slot(k, jc) = k * JC + (jc ^ ((k & 3) << 2))          (JC = BN / 8 chunks per contraction row)
// and the MFMA fragment (8 consecutive k of one column) is assembled by two transposing reads:
// ds_read_b64_tr_b16 hands lane i of a group of 16 lanes the values M[4e + i/4][i % 4], e = 0..3, where
// M[q] are the 4 bf16 lane q of the group points at.  With lane q pointing at contraction row q / 4,
// columns 4 (q % 4)..+3 of a 16-column block, lane i receives 4 consecutive k of column i.  The XOR
// on the chunk index puts the four contraction rows of one read into different bank quarters.
// The read is issued from inline assembly: as a builtin it makes the compiler wait for every
// direct-to-LDS load in flight (it cannot tell that the ring stage being read is not the one being
// filled), which serialises the ring.  The compiler does not count these reads, so
// lds_read_tr16_done() waits for them and ties the result registers to that wait: nothing may
// touch a result before it has passed through that call.
#define lds_read_tr16(dst, addr, off) \
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off) : "memory")
#define lds_read_b128(dst, addr, off) \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off) : "memory")
__device__ __forceinline__ void lds_read_tr16_done(u32x2_t& x, u32x2_t& y) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x), "+v"(y)::"memory");
}
__device__ __forceinline__ void lds_read_done(u32x4_t& x) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x)::"memory"); }

template <class C, int DBK>
struct GradSrc {
    static constexpr int JC = C::BN / 8, RPI = 64 / JC, INSTR = DBK / (RPI * C::NW);
    static_assert((JC == 16 || JC == 32) && DBK % (RPI * C::NW) == 0 && (RPI * C::NW) % 4 == 0, "chunk mapping");
    const NG_AS1 unsigned char* ptr;   // this lane's chunk in contraction row 0 of the matrix
    long long pitch;                   // bytes per contraction row
    int krow, m;                       // krow: this lane's row within the rows of instruction 0; m: rows to fetch
    const NG_AS1 unsigned char* lastp; // source of this lane's chunk in row m, if it has one there
    bool colok;
    __device__ __forceinline__ void init(const void* G, long long ld_g, int m_, int n, int j0, int lane, int wv,
                                         const void* tail8, const NG_AS1 unsigned char* zp) {
        krow = wv * RPI + lane / JC;
        const int jc = (lane % JC) ^ ((krow & 3) << 2);
        const int col = j0 + 8 * jc;
        colok = col < n;
        // the chunk that straddles the last column is not fetched from the last row (it would end
        // past the matrix) but from its zero-padded copy
        const bool straddle = colok && col + 8 > n;
        m = straddle ? m_ - 1 : m_;
        lastp = straddle ? (const NG_AS1 unsigned char*)tail8 : zp;
        pitch = ld_g * 2;
        ptr = (const NG_AS1 unsigned char*)G + (long long)(colok ? col : 0) * 2;
    }
    __device__ __forceinline__ void issue(int kt, unsigned char* stage, const NG_AS1 unsigned char* zp, int wv) const {
#pragma unroll
        for (int p = 0; p < INSTR; ++p) {
            const int k = kt * DBK + p * C::NW * RPI + krow;   // (p NW RPI) % 4 == 0: the XOR of init holds for every p
            const NG_AS1 unsigned char* g = (colok && k < m) ? ptr + k * pitch : (k == m ? lastp : zp);
            __builtin_amdgcn_global_load_lds((const NG_AS1 void*)g, (NG_AS3 void*)(stage + (p * C::NW + wv) * 1024), 16,
                                             0, 0);
        }
    }
    // byte offset inside the stage that lane (li = lane % 32, h = lane / 32) passes to the first
    // transposing read of column block cb (first column, a multiple of 32) and k-slots 8h..8h+3;
    // the second read (k-slots +4) is 4 rows further, the next 16-deep step 16 rows.
    static constexpr int ROW_BYTES = JC * 16;
    static __device__ __forceinline__ int frag(int cb, int li, int h) {
        const int q = li & 15;
        const int k = 8 * h + (q >> 2);
        const int jc = (cb >> 3) + 2 * (li >> 4) + ((q & 3) >> 1);
        return (k * JC + (jc ^ ((q >> 2) << 2))) * 16 + (q & 1) * 8;
    }
};

template <class C, int DBK, int NST, bool HB>
__global__ __launch_bounds__(C::NT) void k_project_bf16_dl(const MatDev* __restrict__ mats,
                                                           const MatDyn* __restrict__ dyn,
                                                           const TileRef* __restrict__ tiles, const void* zero16) {
    typedef DlCfg<C, DBK, NST> D;
    constexpr int KK = DBK / 16;
    typedef RowMajorSrc<C, DBK, C::BM> ARows;
    typedef GradSrc<C, DBK> BGrad;
    static_assert(BGrad::INSTR == D::B_INSTR, "stage accounting");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const TileRef tr = tiles[blockIdx.x];
    if (tr.mat < 0) return;   // padding entry of the XCD-ordered table
    const MatDev& md = mats[tr.mat];
    if (md.side == NG_SIDE_RIGHT) return;
    const int i0 = tr.ti * C::BM, j0 = tr.tj * C::BN;
    if (!projection_tile_direct(md.n)) return;   // k_project_bf16 takes those
    const MatDyn dy = dyn[tr.mat];
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wv / C::NWN, wn = wv % C::NWN, li = lane & 31, h = lane >> 5;
    const int nk = (md.m + DBK - 1) / DBK;

    floatx16 acc[C::MI][C::NJ];
    zero_acc<C>(acc);

    const NG_AS1 unsigned char* zp = (const NG_AS1 unsigned char*)zero16;
    ARows a_rm;
    BGrad b_g;
    a_rm.init(md.PbT, md.r, md.ldk, i0, lane, wv);
    b_g.init(dy.g, md.ld_g, md.m, md.n, j0, lane, wv,
             md.tail8_off >= 0 ? (const void*)step_scratch<char>(dyn, md.tail8_off) : (const void*)zero16, zp);
    auto issue = [&](int kt) {
        unsigned char* stage = smem + (kt % NST) * D::STAGE;
        a_rm.issue(kt, stage, zp, wv);
        b_g.issue(kt, stage + D::A_BYTES, zp, wv);
    };
    // fragment addresses inside a stage (LDS byte offsets; + 2048 per 32 A rows)
    const unsigned smem_lds = (unsigned)(unsigned long long)(NG_AS3 unsigned char*)smem;
    static_assert(KK == 2, "two 16-deep steps per stage");
    unsigned a_off[KK], b_off[C::NJ];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) a_off[kk] = ARows::frag(wm * C::WM + li, ARows::swz(li), 2 * kk + h);
#pragma unroll
    for (int nj = 0; nj < C::NJ; ++nj) b_off[nj] = D::A_BYTES + BGrad::frag(wn * C::WN + 32 * nj, li, h);

    // One 16-deep step's fragments.  They are read by inline assembly (see lds_read_tr16) and may
    // only be used after done(): the reads of step kk of stage kt + 1 are issued right after the
    // MFMAs of step kk of stage kt, into the registers those MFMAs have just read, and complete
    // while the other step's MFMAs run.
    struct Frag {
        u32x4_t a[C::MI];
        u32x2_t blo[C::NJ], bhi[C::NJ];
    };
    Frag f[KK];
    auto read_frags = [&](int kt) {
        const unsigned cur = smem_lds + (unsigned)(kt % NST) * D::STAGE;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
            for (int mi = 0; mi < C::MI; ++mi) lds_read_b128(f[kk].a[mi], cur + a_off[kk], mi * 32 * ARows::KC * 16);
#pragma unroll
            for (int nj = 0; nj < C::NJ; ++nj) {
                lds_read_tr16(f[kk].blo[nj], cur + b_off[nj], kk * 16 * BGrad::ROW_BYTES);
                lds_read_tr16(f[kk].bhi[nj], cur + b_off[nj], kk * 16 * BGrad::ROW_BYTES + 4 * BGrad::ROW_BYTES);
            }
        }
    };
    auto read_step = [&](int kt, int kk) {   // kk is a literal at every call
        const unsigned cur = smem_lds + (unsigned)(kt % NST) * D::STAGE;
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi) lds_read_b128(f[kk].a[mi], cur + a_off[kk], mi * 32 * ARows::KC * 16);
#pragma unroll
        for (int nj = 0; nj < C::NJ; ++nj) {
            lds_read_tr16(f[kk].blo[nj], cur + b_off[nj], kk * 16 * BGrad::ROW_BYTES);
            lds_read_tr16(f[kk].bhi[nj], cur + b_off[nj], kk * 16 * BGrad::ROW_BYTES + 4 * BGrad::ROW_BYTES);
        }
    };
    // Wait for the fragments of step kk.  LDS reads complete in issue order, so when the reads of the other
    // step were issued after these (LATER of them still allowed in flight) the wait need not cover them.
    constexpr int STEP_READS = C::MI + 2 * C::NJ;
    static_assert(STEP_READS <= 15, "the wait count of one step must fit the counter");
    auto done_step = [&](int kk, bool later_in_flight) {   // kk is a literal at every call
        if (later_in_flight) asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(STEP_READS) : "memory");
        else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi) asm volatile("" : "+v"(f[kk].a[mi])::"memory");
#pragma unroll
        for (int nj = 0; nj < C::NJ; ++nj) asm volatile("" : "+v"(f[kk].blo[nj]), "+v"(f[kk].bhi[nj])::"memory");
    };
    auto mma_step = [&](int kk) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
            for (int nj = 0; nj < C::NJ; ++nj) {
                const u32x4_t b = {f[kk].blo[nj].x, f[kk].blo[nj].y, f[kk].bhi[nj].x, f[kk].bhi[nj].y};
                acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(&f[kk].a[mi]),
                                                                      *reinterpret_cast<const bf16x8_t*>(&b), acc[mi][nj],
                                                                      0, 0, 0);
            }
    };

    // Ring of NST stages, stage kt in buffer kt % NST.  At the top of iteration kt this wave holds the
    // fragments of stage kt (its reads are awaited there), so after the barrier buffer kt % NST is
    // free for stage kt + NST, stage kt + 1 has landed (each wave waited for its own loads of it;
    // loads complete in order) and the stages up to kt + NST - 1 are in flight.
    constexpr int PER_STAGE = D::A_INSTR + D::B_INSTR;
    static_assert(NST >= 2 && NST <= 4 && (NST - 1) * PER_STAGE <= 15, "ring depth / wait counter");
    auto wait_all_but = [&](int stages) {   // at most `stages` stages' worth of this lane's loads in flight
        if (stages <= 0) wait_vmcnt<0>();
        else if (stages == 1) wait_vmcnt<PER_STAGE>();
        else if (stages == 2) wait_vmcnt<(NST > 2 ? 2 : 1) * PER_STAGE>();
        else wait_vmcnt<(NST > 3 ? 3 : 1) * PER_STAGE>();
    };
    for (int q = 0; q < NST; ++q)
        if (q < nk) issue(q);
    wait_all_but((nk < NST ? nk : NST) - 1);
    asm volatile("s_barrier" ::: "memory");
    read_frags(0);
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        done_step(0, true);    // the reads of step 1 were issued after those of step 0
        __builtin_amdgcn_sched_barrier(0);
        mma_step(0);
        __builtin_amdgcn_sched_barrier(0);
        done_step(1, false);   // this wave holds all of stage kt now
        if (more) {
            const int ahead = nk - kt - 2;   // stages issued beyond kt + 1
            wait_all_but(ahead < NST - 2 ? ahead : NST - 2);
            // a bare barrier: __syncthreads() would also wait for the loads in flight.  Behind it every
            // wave has read buffer kt % NST to the end and stage kt + 1 has landed.
            asm volatile("s_barrier" ::: "memory");
            if (kt + NST < nk) issue(kt + NST);
            read_step(kt + 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        mma_step(1);
        __builtin_amdgcn_sched_barrier(0);
        if (more) read_step(kt + 1, 1);
        __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();   // every wave is done with the ring: the bf16 epilogue stages C through the same LDS

    // what the chunk that straddles the last column brought in beyond column n - 1 sits in accumulator
    // columns >= n, which the epilogue zeroes
    project_epilogue<C, HB>(acc, md, dy, smem, i0, j0, t, wm, wn, li, h);
}

// =================================================================== refresh products with a bf16 gradient
// The big products of the projector refresh multiply the bf16 gradient by an fp32 sketch matrix Y.
// On the fp32 MFMA they run at a sixteenth of the bf16 rate, so Y is split on its way into LDS into
// three bf16 planes, Y = Y0 + Y1 + Y2 with Y0 = bf16(Y), Y1 = bf16(Y - Y0), Y2 = bf16(Y - Y0 - Y1)
// (24 mantissa bits: the float itself unless it spans more than three bf16 exponent windows), and the
// product is three bf16 MFMA products accumulated in fp32 -- the arithmetic of an fp32 GEMM whose
// gradient operand is exactly representable, at three sixteenths of its MFMA cost.
//
// YTLoader: Y stored [k][x] with x contiguous (the sketch matrices are [rows][l]).  One 4 (k) x 8 (x)
// block per thread and 64-deep tile, transposed in registers like the gradient tile of the
// register-staged projection, each value split, written as 8-byte LDS words (4 consecutive k).
template <class C>
struct YTLoader {
    static_assert(C::KG * (C::BM / 8) == C::NT && C::BM == C::BN, "one block per thread");
    const NG_AS1 float* base;
    long long ld;
    int k_lim, x_lim, kg4, xcol;
    f32x4_t r[4][2];
    unsigned rowok;

    __device__ __forceinline__ void init(const float* Y, long long ld_, int k_lim_, int x_lim_, int x0, int t) {
        base = (const NG_AS1 float*)Y;
        ld = ld_;
        k_lim = k_lim_;
        x_lim = x_lim_;
        kg4 = (t % C::KG) * 4;
        xcol = x0 + 8 * (t / C::KG);
    }
    __device__ __forceinline__ void load(int k0) {
        rowok = 0;
        const bool whole = xcol + 8 <= x_lim;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = k0 + kg4 + q;
            const bool ok = k < k_lim;
            rowok |= ok ? (1u << q) : 0u;
            const NG_AS1 float* row = base + (long long)(ok ? k : k_lim - 1) * ld;
            if (whole) {
                r[q][0] = *(const NG_AS1 f32x4_a4*)(row + xcol);
                r[q][1] = *(const NG_AS1 f32x4_a4*)(row + xcol + 4);
            } else {
#pragma unroll
                for (int c = 0; c < 8; ++c) r[q][c >> 2][c & 3] = (xcol + c < x_lim) ? row[xcol + c] : 0.f;
            }
        }
    }
    // P0, P1, P2: the plane tiles, [x][LDS_K] bf16 each; only the leading NP planes are written
    template <int NP>
    __device__ __forceinline__ void store(bf16_t* P0, bf16_t* P1, bf16_t* P2, int t) const {
        const int xg = t / C::KG;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            unsigned short h0[4], h1[4], h2[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float v = ((rowok >> q) & 1u) ? r[q][c >> 2][c & 3] : 0.f;
                const unsigned a = f2bf(v);
                const float r1 = v - __uint_as_float(a << 16);
                const unsigned b = f2bf(r1);
                const float r2 = r1 - __uint_as_float(b << 16);
                h0[q] = (unsigned short)a;
                h1[q] = (unsigned short)b;
                h2[q] = (unsigned short)f2bf(r2);
            }
            const int off = (xg * 8 + c) * C::LDS_K + kg4;
            *reinterpret_cast<u32x2_t*>(P0 + off) = (u32x2_t){h0[0] | ((unsigned)h0[1] << 16), h0[2] | ((unsigned)h0[3] << 16)};
            if (NP == 1) continue;
            *reinterpret_cast<u32x2_t*>(P1 + off) = (u32x2_t){h1[0] | ((unsigned)h1[1] << 16), h1[2] | ((unsigned)h1[3] << 16)};
            if (NP == 2) continue;
            *reinterpret_cast<u32x2_t*>(P2 + off) = (u32x2_t){h2[0] | ((unsigned)h2[1] << 16), h2[2] | ((unsigned)h2[3] << 16)};
        }
    }
};

// One BK-deep sweep: the plain operand's fragments against the three planes'.  PA: the planes are the A
// operand (rows of the result), else the B operand.
template <class C, bool PA, int NP>
__device__ __forceinline__ void mma_tile_x3(floatx16 (&acc)[C::MI][C::NJ], const bf16_t* Gs, const bf16_t* P0, int wm,
                                            int wn, int li, int h) {
    constexpr int KK = C::BK / 16, PL = C::BM * C::LDS_K;   // elements per plane tile
    const int prow = (PA ? wm * C::WM : wn * C::WN) + li, grow = (PA ? wn * C::WN : wm * C::WM) + li;
    constexpr int PN = PA ? C::MI : C::NJ, GN = PA ? C::NJ : C::MI;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        u32x4_t g[GN];
#pragma unroll
        for (int x = 0; x < GN; ++x)
            g[x] = *reinterpret_cast<const u32x4_t*>(Gs + (grow + 32 * x) * C::LDS_K + kk * 16 + h * 8);
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) {
            u32x4_t y[PN];
#pragma unroll
            for (int x = 0; x < PN; ++x)
                y[x] = *reinterpret_cast<const u32x4_t*>(P0 + pl * PL + (prow + 32 * x) * C::LDS_K + kk * 16 + h * 8);
#pragma unroll
            for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
                for (int nj = 0; nj < C::NJ; ++nj) {
                    const u32x4_t& a = PA ? y[mi] : g[mi];
                    const u32x4_t& b = PA ? g[nj] : y[nj];
                    acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(&a),
                                                                          *reinterpret_cast<const bf16x8_t*>(&b),
                                                                          acc[mi][nj], 0, 0, 0);
                }
        }
    }
}

// FORM 1: C = Ya [m][l] = G Y        (Y [n][l]; G rows are contraction-contiguous: chunk loader)
// FORM 2: C = Yb [n][l] = G^T Y      (Y [m][l]; G through the transposing loader, as the A operand)
// FORM 3: C = Bm [l][ldn] = Y^T G    (Y [m][l]: planes on the A side; G through the transposing
//                                     loader; columns >= n of C are written as zero)
// ysrc: which sketch buffer Y is (0 Ya, 1 Yb, 2 Yc).  One 128 x 128 tile per workgroup, 64-deep
// k-steps, register-staged loads one step ahead.  NP: planes of Y that enter the product.  1 for the
// first product of a refresh, whose Y is the random test matrix (rounding its entries to bf16
// leaves it as good a test matrix as before); 2 (16 significant bits) for the products inside the
// subspace iteration, whose results are re-orthonormalised and multiplied again; 3 for the last
// basis and for B = Q^T G, which the Rayleigh-Ritz step takes at face value.
template <class C, int FORM, int NP>
__global__ __launch_bounds__(C::NT) void k_refresh_x3(const MatDev* __restrict__ mats, const MatDyn* __restrict__ dyn,
                                                      int ysrc) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    static_assert(FORM >= 1 && FORM <= 3 && NP >= 1 && NP <= 3, "product form");
    const MatDev& md = mats[blockIdx.z];
    if (md.side == NG_SIDE_RIGHT) return;
    const MatDyn dy = dyn[blockIdx.z];
    const int M = FORM == 1 ? md.m : FORM == 2 ? md.n : md.l;
    const int N = FORM == 3 ? md.ldn : md.l;
    const int K = FORM == 1 ? md.n : md.m;
    const int i0 = blockIdx.y * C::BM, j0 = blockIdx.x * C::BN;
    if (i0 >= M || j0 >= N) return;
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv / C::NWN, wn = wv % C::NWN, li = lane & 31, h = lane >> 5;
    bf16_t* Gs = reinterpret_cast<bf16_t*>(smem);
    bf16_t* P0 = Gs + C::BN * C::LDS_K;
    bf16_t* P1 = P0 + C::BM * C::LDS_K;
    bf16_t* P2 = P1 + C::BM * C::LDS_K;
    const float* Y = ysrc == 0 ? md.Ya : ysrc == 1 ? md.Yb : md.Yc;

    floatx16 acc[C::MI][C::NJ];
    zero_acc<C>(acc);

    // the planes' tile index runs over Y's columns (the l sketch columns): result rows in form 3,
    // result columns otherwise
    YTLoader<C> ly;
    ly.init(Y, md.l, K, md.l, FORM == 3 ? i0 : j0, t);
    BTLoader<C> lgt;   // forms 2, 3: tile index = gradient column
    BKLoader<C> lgk;   // form 1: tile index = gradient row
    const int g0 = FORM == 3 ? j0 : i0;
    bool full = true, k8 = true;
    if (FORM == 1) {
        lgk.init(dy.g, md.ld_g, g0, md.m, md.n, t);
        k8 = (md.n & 7) == 0;
    } else {
        lgt.init(dy.g, md.ld_g, md.m, md.n, g0, t);
        full = (md.n >= 8) && ((md.n & 7) == 0 || g0 + C::BN <= md.n);
    }
    const int nk = (K + C::BK - 1) / C::BK;
    auto loads = [&](int k0) {
        ly.load(k0);
        if (FORM == 1) {
            if (k8) lgk.template load<true>(k0);
            else lgk.template load<false>(k0);
        } else {
            if (full) lgt.template load<true>(k0);
            else lgt.template load<false>(k0);
        }
    };
    auto stores = [&]() {
        ly.template store<NP>(P0, P1, P2, t);
        if (FORM == 1) lgk.store(Gs, t);
        else if (full) lgt.template store<true>(Gs, t);
        else lgt.template store<false>(Gs, t);
    };
    loads(0);
    stores();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) loads((kt + 1) * C::BK);
        mma_tile_x3<C, FORM == 3, NP>(acc, Gs, P0, wm, wn, li, h);
        __syncthreads();
        if (kt + 1 < nk) stores();
        __syncthreads();
    }
    float* Cout = FORM == 1 ? md.Ya : FORM == 2 ? md.Yb : md.Bm;
    const int ldc = FORM == 3 ? md.ldn : md.l;
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
                    if (row < M && col < N) Cout[(long long)row * ldc + col] = acc[mi][nj][4 * g + e];
                }
        }
}

// =================================================================== launchers
// Tile configurations (BM x BN workgroup tile, WM x WN per wavefront).  Update: Cfg3 -- the weight tile
// has 512-byte rows and the operand with 64-byte chunks per row (Pb) is the smaller one.  Projection:
// Cfg4 for the direct-to-LDS kernel, Cfg2 for the register-staged one, Cfg0 for both when the rank is at
// most 128 (a 256-row tile would be half empty).
typedef Cfg<128, 128, 64, 64, 64> Cfg0;
typedef Cfg<256, 128, 128, 64, 64> Cfg2;
typedef Cfg<128, 256, 64, 128, 64> Cfg3;
typedef Cfg<256, 256, 128, 64, 64> Cfg4;   // eight wavefronts

static int project_cfg(int max_r) { return max_r > 128 ? 2 : 0; }

// The tile table has three runs: left-side tiles for the direct-to-LDS kernel, the other left-side
// tiles (gradients of fewer than 8 columns) and right-side tiles (register-staged kernel, one
// instance per side).
// CD / NST: tile configuration and ring depth of the direct-to-LDS kernel; CS: of the register-staged one.
template <class CD, int NST, class CS, bool HB>
static hipError_t run_project(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_direct, int n_staged,
                              int n_right, const void* zero16, hipStream_t stream) {
    constexpr int DBK = 32;
    constexpr int lds_dl = DlCfg<CD, DBK, NST>::LDS_BYTES;
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_project_bf16<CS, HB, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, CS::LDS_BYTES);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_project_bf16<CS, HB, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, CS::LDS_BYTES);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_project_bf16_dl<CD, DBK, NST, HB>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds_dl);
        attr = true;
    }
    if (n_direct > 0)
        hipLaunchKernelGGL((k_project_bf16_dl<CD, DBK, NST, HB>), dim3(n_direct), dim3(CD::NT), lds_dl, stream, mats,
                           dyn, tiles, zero16);
    if (n_staged > 0)
        hipLaunchKernelGGL((k_project_bf16<CS, HB, false>), dim3(n_staged), dim3(CS::NT), CS::LDS_BYTES, stream, mats,
                           dyn, tiles + n_direct);
    if (n_right > 0)
        hipLaunchKernelGGL((k_project_bf16<CS, HB, true>), dim3(n_right), dim3(CS::NT), CS::LDS_BYTES, stream, mats, dyn,
                           tiles + n_direct + n_staged);
    return hipGetLastError();
}

hipError_t launch_project_bf16(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_direct, int n_staged,
                               int n_right, int max_r, int hist_bf16, const void* zero16, hipStream_t stream) {
    if (project_cfg(max_r) == 0)
        return hist_bf16
                   ? run_project<Cfg0, 3, Cfg0, true>(mats, dyn, tiles, n_direct, n_staged, n_right, zero16, stream)
                   : run_project<Cfg0, 3, Cfg0, false>(mats, dyn, tiles, n_direct, n_staged, n_right, zero16, stream);
    return hist_bf16 ? run_project<Cfg4, 4, Cfg2, true>(mats, dyn, tiles, n_direct, n_staged, n_right, zero16, stream)
                     : run_project<Cfg4, 4, Cfg2, false>(mats, dyn, tiles, n_direct, n_staged, n_right, zero16, stream);
}

// sides: bit 0 = the layer set has left-side matrices, bit 1 = right-side ones.  Each side has its own
// instance of the kernel over the same tile table; a workgroup whose matrix belongs to the other
// side exits at once.
hipError_t launch_update_bf16(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles,
                              StepScalars sc, const void* zero16, int sides, hipStream_t stream) {
    if (n_tiles == 0) return hipSuccess;
    typedef Cfg3 C;
    constexpr int DBK = 32, NST = 3;   // 72 KiB of LDS: two workgroups per CU
    constexpr int lds = DlCfg<C, DBK, NST>::LDS_BYTES;
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_update_bf16_dl<C, DBK, NST, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_update_bf16_dl<C, DBK, NST, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr = true;
    }
    if (sides & 1)
        hipLaunchKernelGGL((k_update_bf16_dl<C, DBK, NST, false>), dim3(n_tiles), dim3(C::NT), lds, stream, mats, dyn,
                           tiles, sc, zero16);
    if (sides & 2)
        hipLaunchKernelGGL((k_update_bf16_dl<C, DBK, NST, true>), dim3(n_tiles), dim3(C::NT), lds, stream, mats, dyn,
                           tiles, sc, zero16);
    return hipGetLastError();
}

// which: 0 = projection, direct-to-LDS kernel; 1 = update; 2 = projection, register-staged kernel
// (the projection's shapes depend on the largest rank of the layer set)
void bf16_tile_shape(int which, int max_r, int* bm, int* bn) {
    if (which == 1) {
        *bm = Cfg3::BM;
        *bn = Cfg3::BN;
    } else if (project_cfg(max_r) == 0) {
        *bm = Cfg0::BM;
        *bn = Cfg0::BN;
    } else {
        *bm = which == 0 ? Cfg4::BM : Cfg2::BM;
        *bn = which == 0 ? Cfg4::BN : Cfg2::BN;
    }
}

template <int FORM, int NP>
static hipError_t run_refresh_x3(dim3 g, const MatDev* mats, const MatDyn* dyn, int ysrc, hipStream_t stream) {
    typedef Cfg0 C;
    constexpr int lds = (C::BN + NP * C::BM) * C::LDS_K * 2;
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_refresh_x3<C, FORM, NP>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr = true;
    }
    hipLaunchKernelGGL((k_refresh_x3<C, FORM, NP>), g, dim3(C::NT), lds, stream, mats, dyn, ysrc);
    return hipGetLastError();
}

hipError_t launch_refresh_x3(int form, int ysrc, int planes, const MatDev* mats, const MatDyn* dyn, int n_mats,
                             int max_m, int max_n, hipStream_t stream) {
    typedef Cfg0 C;
    const dim3 g((max_n + C::BN - 1) / C::BN, (max_m + C::BM - 1) / C::BM, n_mats);
    if (form == 1 && planes == 1) return run_refresh_x3<1, 1>(g, mats, dyn, ysrc, stream);
    if (form == 1 && planes == 2) return run_refresh_x3<1, 2>(g, mats, dyn, ysrc, stream);
    if (form == 1 && planes == 3) return run_refresh_x3<1, 3>(g, mats, dyn, ysrc, stream);
    if (form == 2 && planes == 2) return run_refresh_x3<2, 2>(g, mats, dyn, ysrc, stream);
    if (form == 2 && planes == 3) return run_refresh_x3<2, 3>(g, mats, dyn, ysrc, stream);
    if (form == 3 && planes == 3) return run_refresh_x3<3, 3>(g, mats, dyn, ysrc, stream);
    return hipErrorInvalidValue;
}

}  // namespace ng

