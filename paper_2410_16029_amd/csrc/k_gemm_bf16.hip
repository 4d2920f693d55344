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
// LDS tiles are [row][BK + 8] bf16: the 16-byte pad makes the 16-byte fragment reads of 16
// consecutive rows hit disjoint banks.
//
// Memory access rules followed here (each was measured to matter):
//   * every pointer read out of a table is cast to the global address space, so loads are
//     global_load (not flat_load, which also ticks the LDS counter);
//   * loads are branch-free: an out-of-range row / k / column is clamped to a valid address and
//     the value is zeroed later, when it is written to LDS -- a guarded load in its own branch,
//     or a select right after the load, makes the compiler wait for the load before the MFMAs
//     of the current tile instead of after them;
//   * offsets are 32-bit (the host checks that every matrix is below 2 GiB).
#include <stdlib.h>

#include "ng_internal.h"

namespace ng {

#define NG_AS1 __attribute__((address_space(1)))

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef u32x4_t __attribute__((aligned(2))) u32x4_a2;   // 16-byte access at 2-byte alignment
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

template <int BM_, int BN_, int WM_, int WN_, int BK_, bool DB_ = false>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_;
    static constexpr bool DB = DB_;                         // two LDS operand buffers, one barrier per k-step
    static constexpr int NWM = BM / WM, NWN = BN / WN, NW = NWM * NWN, NT = NW * 64;
    static constexpr int MI = WM / 32, NJ = WN / 32;
    static constexpr int LDS_K = BK + 8;                    // bf16 elements per LDS row
    static constexpr int KC = BK / 8;                       // 16-byte chunks per row
    static constexpr int KG = BK / 4;                       // 4-row groups of the transposed operand
    static constexpr int A_CHUNKS = BM * KC / NT;           // per thread
    static constexpr int BN8_CHUNKS = BN * KC / NT;         // per thread, octet-layout B
    static constexpr int BT_BLOCKS = KG * (BN / 8) / NT;    // per thread, transposing B: 4k x 8j blocks
    static constexpr int OPER_BYTES = (BM + BN) * LDS_K * 2;
    static constexpr int LDC = BN + 8;                      // floats per staged C row
    static constexpr int STAGE_BYTES = NWM * 32 * LDC * 4;
    static constexpr int OPER_TOTAL = DB ? 2 * OPER_BYTES : OPER_BYTES;
    static constexpr int LDS_BYTES = OPER_TOTAL > STAGE_BYTES ? OPER_TOTAL : STAGE_BYTES;
    static_assert(BM * KC % NT == 0 && BN * KC % NT == 0 && KG * (BN / 8) % NT == 0, "tile/thread mismatch");
    static_assert(NT % KC == 0 && NT % BN == 0 && NT % KG == 0, "per-thread invariants");
};

// ------------------------------------------------------------------ A operand
// bf16 [rows][ld], contraction contiguous.  Chunk c = t + NT*p: row c / KC, k-chunk c % KC
// (the same k-chunk for every p).  Rows >= row_lim and k >= k_lim are zero (k_lim % 8 == 0).
template <class C>
struct ALoader {
    gbf16_cptr base;
    unsigned rowoff[C::A_CHUNKS];
    unsigned rowok;    // bit p
    int kofs, k_lim;
    u32x4_t r[C::A_CHUNKS];
    bool kok;

    __device__ __forceinline__ void init(const bf16_t* A, int ld, int row0, int row_lim, int k_lim_, int t) {
        base = (gbf16_cptr)A;
        kofs = (t % C::KC) * 8;
        k_lim = k_lim_;
        rowok = 0;
#pragma unroll
        for (int p = 0; p < C::A_CHUNKS; ++p) {
            const int row = row0 + (t + C::NT * p) / C::KC;
            const bool ok = row < row_lim;
            rowok |= ok ? (1u << p) : 0u;
            rowoff[p] = (unsigned)(ok ? row : row_lim - 1) * (unsigned)ld;
        }
    }
    __device__ __forceinline__ void load(int k0) {
        const int k = k0 + kofs;
        kok = k < k_lim;
        const unsigned kc = (unsigned)(kok ? k : k_lim - 8);
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

// ------------------------------------------------------------------ B operand, octet layout
// N8 [k/8][ldn][8].  Chunk c = t + NT*p: column c % BN (the same for every p), octet c / BN.
template <class C>
struct B8Loader {
    gbf16_cptr base;
    unsigned joff, ldn8;
    int roct, oct_t;
    bool jok;
    unsigned okmask;
    u32x4_t r[C::BN8_CHUNKS];

    __device__ __forceinline__ void init(const bf16_t* N8, int ldn, int roct_, int j0, int t) {
        base = (gbf16_cptr)N8;
        const int j = j0 + t % C::BN;
        jok = j < ldn;
        joff = (unsigned)(jok ? j : ldn - 1) * 8u;
        ldn8 = (unsigned)ldn * 8u;
        roct = roct_;
        oct_t = t / C::BN;
    }
    __device__ __forceinline__ void load(int k0) {
        okmask = 0;
#pragma unroll
        for (int p = 0; p < C::BN8_CHUNKS; ++p) {
            const int oct = (k0 >> 3) + oct_t + (C::NT / C::BN) * p;
            const bool ok = jok && oct < roct;
            okmask |= ok ? (1u << p) : 0u;
            const unsigned oc = (unsigned)(oct < roct ? oct : roct - 1);
            r[p] = *(const NG_AS1 u32x4_t*)(base + (oc * ldn8 + joff));
        }
    }
    __device__ __forceinline__ void store(bf16_t* Bs, int t) const {
#pragma unroll
        for (int p = 0; p < C::BN8_CHUNKS; ++p) {
            const int c = t + C::NT * p;
            *reinterpret_cast<u32x4_t*>(Bs + (c % C::BN) * C::LDS_K + (c / C::BN) * 8) =
                zero_unless((okmask >> p) & 1u, r[p]);
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
// tile into registers, store(ptr, t) writes them (masked) to LDS.
//   single buffer: loads of tile kt+1 are in flight during the MFMAs of tile kt; two barriers.
//   double buffer: registers hold tile kt+1 (loaded one whole step earlier); they are written to
//   the other LDS buffer while tile kt is multiplied, then the loads of tile kt+2 are issued;
//   one barrier per step.
template <class C, class LA, class LB>
__device__ __forceinline__ void gemm_mainloop(floatx16 (&acc)[C::MI][C::NJ], LA& la, LB& lb, unsigned char* smem,
                                              int nk, int t, int wm, int wn, int li, int h) {
    bf16_t* As0 = reinterpret_cast<bf16_t*>(smem);
    bf16_t* Bs0 = As0 + C::BM * C::LDS_K;
    if (!C::DB) {
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
    } else {
        bf16_t* As1 = reinterpret_cast<bf16_t*>(smem + C::OPER_BYTES);
        bf16_t* Bs1 = As1 + C::BM * C::LDS_K;
        la.load(0);
        lb.load(0);
        la.store(As0, t);
        lb.store(Bs0, t);
        if (nk > 1) {
            la.load(C::BK);
            lb.load(C::BK);
        }
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            bf16_t* Ac = (kt & 1) ? As1 : As0;
            bf16_t* Bc = (kt & 1) ? Bs1 : Bs0;
            bf16_t* An = (kt & 1) ? As0 : As1;
            bf16_t* Bn = (kt & 1) ? Bs0 : Bs1;
            if (kt + 1 < nk) {
                la.store(An, t);
                lb.store(Bn, t);
            }
            if (kt + 2 < nk) {
                la.load((kt + 2) * C::BK);
                lb.load((kt + 2) * C::BK);
            }
            mma_tile<C>(acc, Ac, Bc, wm, wn, li, h);
            __syncthreads();
        }
    }
}

template <class C>
__global__ __launch_bounds__(C::NT) void k_project_bf16(const MatDev* __restrict__ mats,
                                                        const MatDyn* __restrict__ dyn,
                                                        const TileRef* __restrict__ tiles) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const TileRef tr = tiles[blockIdx.x];
    if (tr.mat < 0) return;   // padding entry of the XCD-ordered table
    const MatDev& md = mats[tr.mat];
    const MatDyn dy = dyn[tr.mat];
    const int i0 = tr.ti * C::BM, j0 = tr.tj * C::BN;
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv / C::NWN, wn = wv % C::NWN, li = lane & 31, h = lane >> 5;
    const int m = md.m, n = md.n, r = md.r, ldn = md.ldn;

    floatx16 acc[C::MI][C::NJ];
    zero_acc<C>(acc);

    ALoader<C> la;
    BTLoader<C> lb;
    la.init(md.PbT, md.ldk, i0, r, md.ldk, t);
    lb.init(dy.g, md.ld_g, m, n, j0, t);
    const int nk = (m + C::BK - 1) / C::BK;
    // uniform per workgroup: are all 8-column chunks of this tile whole?
    const bool full = (n >= 8) && ((n & 7) == 0 || j0 + C::BN <= n);
    if (full) {
        BTView<C, true> v{lb};
        gemm_mainloop<C>(acc, la, v, smem, nk, t, wm, wn, li, h);
    } else {
        BTView<C, false> v{lb};
        gemm_mainloop<C>(acc, la, v, smem, nk, t, wm, wn, li, h);
    }

    NG_AS1 float* R = (NG_AS1 float*)(md.H + (long long)dy.head * md.slot_elems);
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
                    if (row < r && col < ldn) R[(unsigned)row * (unsigned)ldn + (unsigned)col] = acc[mi][nj][4 * g + e];
                }
        }
}

// =================================================================== update
template <class C>
__global__ __launch_bounds__(C::NT) void k_update_bf16(const MatDev* __restrict__ mats,
                                                       const MatDyn* __restrict__ dyn,
                                                       const TileRef* __restrict__ tiles, StepScalars sc) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
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

    floatx16 acc[C::MI][C::NJ];
    zero_acc<C>(acc);

    ALoader<C> la;
    B8Loader<C> lb;
    la.init(md.Pb, md.ldr, i0, m, md.ldr, t);
    lb.init(reinterpret_cast<const bf16_t*>(md.N), ldn, md.roct, j0, t);
    const int nk = (kdim + C::BK - 1) / C::BK;
    NG_AS1 bf16_t* W = (NG_AS1 bf16_t*)dy.w;
    const unsigned ld_w = (unsigned)md.ld_w;
    gemm_mainloop<C>(acc, la, lb, smem, nk, t, wm, wn, li, h);
    if (C::DB) __syncthreads();   // (the single-buffer loop already ends on a barrier)

    // Epilogue, one 32-row block of every wave-row at a time: accumulators -> LDS (float),
    // then each thread read-modify-writes 8 consecutive bf16 of one weight row.
    constexpr int ROWS = C::NWM * 32;
    constexpr int CH = C::BN / 8;                         // 8-column chunks per row
    constexpr int PER_T = ROWS * CH / C::NT;
    static_assert(ROWS * CH % C::NT == 0, "epilogue mapping");
    const bool cols_full = (n >= 8) && ((n & 7) == 0 || j0 + C::BN <= n);
    // All weight loads of the tile are issued up front (the main loop's staging registers are
    // free now), so the HBM latency is paid once per tile, not once per pass.
    u32x4_t wv4[C::MI][PER_T];
    if (cols_full) {
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
                wv4[mi][p] = *(const NG_AS1 u32x4_a2*)(W + (rc * ld_w + jc));
            }
    }
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
        if (cols_full) {
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
                if (row < m && col + 8 <= n) *(NG_AS1 u32x4_a2*)(W + ((unsigned)row * ld_w + (unsigned)col)) = ov;
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

// =================================================================== launchers
// Tile configurations: 256 x 128 workgroup tiles (128 x 64 per wavefront); the projection falls
// back to 128 x 128 when the rank is at most 128 (a 256-row tile would be half empty).
typedef Cfg<128, 128, 64, 64, 64> Cfg0;
typedef Cfg<256, 128, 128, 64, 64> Cfg2;

static int project_cfg(int max_r) { return max_r > 128 ? 2 : 0; }

template <class C>
static hipError_t run_project(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles,
                              hipStream_t stream) {
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_project_bf16<C>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        attr = true;
    }
    hipLaunchKernelGGL(k_project_bf16<C>, dim3(n_tiles), dim3(C::NT), C::LDS_BYTES, stream, mats, dyn, tiles);
    return hipGetLastError();
}

template <class C>
static hipError_t run_update(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles,
                             StepScalars sc, hipStream_t stream) {
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_update_bf16<C>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        attr = true;
    }
    hipLaunchKernelGGL(k_update_bf16<C>, dim3(n_tiles), dim3(C::NT), C::LDS_BYTES, stream, mats, dyn, tiles, sc);
    return hipGetLastError();
}

hipError_t launch_project_bf16(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles,
                               int max_r, hipStream_t stream) {
    if (n_tiles == 0) return hipSuccess;
    if (project_cfg(max_r) == 0) return run_project<Cfg0>(mats, dyn, tiles, n_tiles, stream);
    return run_project<Cfg2>(mats, dyn, tiles, n_tiles, stream);
}

hipError_t launch_update_bf16(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles,
                              StepScalars sc, hipStream_t stream) {
    if (n_tiles == 0) return hipSuccess;
    return run_update<Cfg2>(mats, dyn, tiles, n_tiles, sc, stream);
}

// which: 0 = projection (needs the largest rank of the layer set), 1 = update
void bf16_tile_shape(int which, int max_r, int* bm, int* bn) {
    const bool small = which == 0 && project_cfg(max_r) == 0;
    *bm = small ? Cfg0::BM : Cfg2::BM;
    *bn = small ? Cfg0::BN : Cfg2::BN;
}

}  // namespace ng
