// Internal declarations shared by the host scheduler and the kernel files.
// Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "ng.h"

namespace ng {

typedef unsigned short bf16_t;   // raw bfloat16 bits

constexpr int kMaxS = 64;        // history slots
constexpr int kDotPartsMax = 256; // per-matrix partial sums of the Gram-row reduction
constexpr int kAdamPatchCols = 128; // columns of one transform+Adam workgroup patch (32 rows)
constexpr int kDynChunk = 96;    // per-step table entries uploaded per launch (by kernel argument)
constexpr int kSkinnyMaxRank = 16;   // fp32 layer sets with ranks up to this take the vector-ALU projection / update
constexpr int kSkinnyRows = 128;     // rows and columns of the gradient / weight one of their workgroups takes
constexpr int kSkinnyCols = 256;
constexpr int kStatePanelCols = 2048;   // columns per panel of a wide M, V or history slot (see state_panel)
// bits of the device's sticky status word: 1 solve (pivot / non-finite), 2 transform+Adam (non-finite),
// 4 Cholesky pivot of the refresh, 8 non-positive Ritz value among the leading r
constexpr int kStatusNotConverged = 16;   // the Jacobi eigen-solve of a refresh ran out of sweeps
constexpr int kJacobiBlock = 16;  // rows per block of the blocked Jacobi (a visit rotates a pair of blocks)

// Static per-matrix description, lives in the workspace (device) and in the handle (host).
struct MatDev {
    // m, n: dimensions of the problem the kernels see: the weight's for NG_SIDE_LEFT, swapped for
    // NG_SIDE_RIGHT (the transposed problem); ld_w / ld_g always describe the caller's row-major arrays
    int m, n, r, ldn;
    int side;
    int l;            // refresh sketch width
    int ldk;          // contraction length of PbT (m rounded up to 32)
    int ldr;          // contraction length of Pb (r rounded up to 32)
    int roct;         // ceil(r/8): octets of N in the bf16 layout
    long long ld_w, ld_g;
    long long slot_elems;   // elements from one history slot to the next: r * state_cols(ldn, pw)
    int pw;           // columns per panel of M, V and every history slot (== ldn: one panel, plain row-major)
    float* P;
    float* M;
    float* V;
    float* H;         // history ring; bf16 elements when StepScalars::hist_bf16 (same element offsets)
    double* K;        // s*s Gram
    double* w64;      // s
    float* w32;       // s
    void* N;
    bf16_t* Pb;       // [ldr/32][m][32]  bf16 copy of P,   k-blocked: (i, rho) at ((rho/32) m + i) 32 + rho%32
    bf16_t* PbT;      // [ldk/32][r][32]  bf16 copy of P^T, k-blocked: (rho, i) at ((i/32) r + rho) 32 + i%32
                      // (operands of the update / projection GEMMs: the 64 bytes one row gives to a 32-deep
                      // stage lie next to its neighbours', so a tile's stage is one run of whole cache lines)
    // Scratch of one step lies behind the per-step table (MatDyn[n_mats]) in one block: the three
    // offsets below are in bytes from the start of that table (the `dyn` argument of the kernels),
    // -1 where a matrix has none.  The block is the front of the caller's workspace for ng_step and
    // the library's own static device array for ng_step_static.
    long long dot_parts_off;   // double [kDotPartsMax][s]: partial sums of the Gram-row reduction
    int dot_nparts;      // workgroups of the Gram-row reduction for this matrix
    int dot_iters;       // grid-stride iterations per workgroup
    // refresh scratch (all in the workspace)
    float* Ya;        // [max(m,n)][l]
    float* Yb;        // [max(m,n)][l]
    float* Yc;        // [max(m,n)][l]
    float* Bm;        // [l][ldn]   B = Q^T G; later the l x r rotation
    double* T;        // [lp][lp]   Gram / Cholesky factor / Rayleigh-Ritz matrix
    float* Linv;      // [lp][lp]   inverse Cholesky factor (float); during the Rayleigh-Ritz step the rows
                      //            that the Jacobi rotates
    double* ritz;     // [lp]
    int* order;       // [lp]
    int* jflag;       // [0] rotations this sweep, [1] converged
    float* carry;     // [r][ldn] scratch of the history carry-over (null unless enabled)
    long long skinny_parts_off;   // float [ceil(m/kSkinnyRows)][rk][ldn] row-chunk sums of the small-rank projection
    long long tail8_off;   // 8 bf16: the last gradient row's columns from the last multiple of 8 on,
                           // zero-padded (rewritten every step, see launch_upload_dyn)
    int lp;           // l rounded up to a whole number of Jacobi block pairs: order and row pitch of T, Linv
};

// Per-step values: uploaded into the step's scratch block by a tiny kernel that receives them by value.
struct MatDyn {
    const void* g;
    void* w;
    int head;      // slot written by this step
    int count;     // valid slots after the push
    float bc1, bc2;   // Adam bias corrections 1/(1-beta1^t), 1/sqrt(1-beta2^t)
};

struct DynChunk {
    MatDyn e[kDynChunk];
};

constexpr size_t kStaticScratchBytes = NG_STATIC_SCRATCH_BYTES;   // the library's own step scratch (ng_step_static)

// M, V and every history slot hold their r x ldn elements as column panels of pw columns: panel p
// (columns p pw .. p pw + pw - 1) is a row-major r x pw block, and the panels lie one after the other.
// pw == ldn is the plain row-major array.  Otherwise pw = kStatePanelCols, a multiple of every tile and
// patch width (a tile lies in one panel), and the last panel's columns from ldn on are padding: zero,
// never written, and skipped by the kernels that read an array flat.  A 2048-column panel gives 4-byte
// elements a row pitch of 8 KB, at which the streaming kernels run fastest (transform+Adam: 6.6 TB/s on
// 2048-column states against 5.8 TB/s on row-major 5472-column ones and 5.1 TB/s at a 5.5 KB pitch).
struct StatePanel {
    unsigned base;   // element offset of the panel inside the array
    int pitch;       // its row pitch
    int col0;        // its first column
    __host__ __device__ unsigned at(int row, int col) const { return base + (unsigned)row * (unsigned)pitch + (unsigned)(col - col0); }
};
__host__ __device__ inline StatePanel state_panel(int r, int pw, int col) {
    StatePanel sp;
    const int p = col / pw;
    sp.col0 = p * pw;
    sp.pitch = pw;
    sp.base = (unsigned)p * (unsigned)r * (unsigned)pw;
    return sp;
}
// columns an array of ldn columns occupies in panels of pw
__host__ __device__ inline int state_cols(int ldn, int pw) { return (ldn + pw - 1) / pw * pw; }

// The same arrays read flat, V elements per 16-byte vector: the r * ldn / V vectors that hold the
// columns below ldn, numbered in storage order; position q lies at vector at(q) of the array.
struct FlatState {
    unsigned whole;      // vectors before the last panel (stored without gaps)
    unsigned row_valid;  // vectors per row of the last panel that hold columns below ldn
    unsigned row_pitch;  // vectors per stored row of the last panel
    unsigned count;      // r * ldn / V
    __host__ __device__ unsigned at(unsigned q) const {
        if (q < whole || row_valid == row_pitch) return q;
        const unsigned k = q - whole, row = k / row_valid;
        return whole + row * row_pitch + (k - row * row_valid);
    }
};
__host__ __device__ inline FlatState flat_state(int r, int ldn, int pw, int V) {
    FlatState f;
    const int last0 = (ldn - 1) / pw * pw;   // first column of the last panel
    f.whole = (unsigned)last0 / (unsigned)V * (unsigned)r;
    f.row_valid = (unsigned)(ldn - last0) / (unsigned)V;
    f.row_pitch = (unsigned)pw / (unsigned)V;
    f.count = (unsigned)r * (unsigned)ldn / (unsigned)V;
    return f;
}

// address inside the step's scratch block, which starts with the per-step table
template <typename T>
__device__ __forceinline__ T* step_scratch(const MatDyn* dyn, long long off) {
    return reinterpret_cast<T*>(reinterpret_cast<char*>(const_cast<MatDyn*>(dyn)) + off);
}

struct StepScalars {
    float lambda;
    float beta1, beta2, eps;
    float lr_scale, lr_wd;
    int adam_mode;
    int s;               // slots read by the kernels (>= 1; the s = 0 case uses one scratch slot)
    int use_fisher;      // 0 when hparams.s == 0
    int hist_bf16;       // history slots are bf16 (else float)
    int norm_count;      // Fisher normaliser 1/count (valid slots) instead of 1/s
    int slot;            // history slot an OP_CARRY_SLOT product works on
};

// Grouped-launch work item: which matrix and which tile / part of it a workgroup takes.
// mat < 0 marks a padding entry (the workgroup exits).
struct TileRef {
    int mat;
    int ti, tj;
    int pad;
};

// Host side: the order in which a grouped GEMM launch's tile table lists the tiles (ng_api.hip).
void xcd_order(const std::vector<TileRef>& logical, const std::vector<int>& cost, std::vector<TileRef>* out);

// Left-side projection tiles of a gradient with at least 8 columns take the direct-to-LDS kernel.  It
// reads whole 16-byte chunks; the one chunk per row that straddles the last column (n % 8 != 0) reads up
// to 7 elements past the row's end, which is the start of the next row or its padding: inside the
// caller's buffer for every row but the last, whose chunk comes from MatDev::tail8 instead.
__host__ __device__ inline bool projection_tile_direct(int n) { return n >= 8; }

// ---------------------------------------------------------------- launchers
// Every launcher enqueues on `stream` and returns hipGetLastError().

// mats != null: also refresh MatDev::tail8 of the left-side matrices from the bf16 gradients in the chunk
hipError_t launch_upload_dyn(MatDyn* table, const DynChunk& chunk, int first, int n, const MatDev* mats,
                             hipStream_t stream);
hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t stream);   // bytes % 4 == 0
// zero the history ring and the Gram block of every matrix (buffer sizes as ng_query_sizes reports them)
hipError_t launch_clear_history(const MatDev* mats, int n_mats, int s, int h_elem_bytes, size_t k_bytes,
                                hipStream_t stream);

// fp32 MFMA grouped GEMM with selectable operands (k_gemm_f32.hip)
enum GemmOp {
    OP_PROJECT_F32 = 0,   // R(slot head) = P^T G                     (step, NG_F32)
    OP_UPDATE_F32,        // W -= lr*(scale * P N + wd W)             (step, NG_F32)
    OP_G_B2A,             // Ya = G Yb     (m x l)
    OP_G_C2A,             // Ya = G Yc
    OP_GT_C2B,            // Yb = G^T Yc   (n x l)
    OP_GRAM_A,            // T = Ya^T Ya   (rows m) -> double
    OP_GRAM_B,            // T = Yb^T Yb   (rows n)
    OP_GRAM_CA,           // T = Yc^T Yc   (rows m)
    OP_GRAM_CB,           // T = Yc^T Yc   (rows n)
    OP_APPLY_A2C,         // Yc = Ya Linv^T (rows m)
    OP_APPLY_B2C,         // Yc = Yb Linv^T (rows n)
    OP_APPLY_C2A,         // Ya = Yc Linv^T (rows m)
    OP_APPLY_C2B,         // Yb = Yc Linv^T (rows n)
    OP_QT_G,              // Bm = Ya^T G   (l x ldn)
    OP_B_BT,              // T = Bm Bm^T   (l x l) -> double
    OP_ROTATE,            // P = Ya * Urot (m x r), Urot (l x r floats) staged in Bm
    OP_GRAM_P,            // T = P^T P (r x r) -> double
    OP_APPLY_P2A,         // Ya[m][r] = P Linv^T
    OP_T_CARRY,           // Linv (r x r, float) = P^T Yc, Yc holding the previous projector
    OP_CARRY_SLOT,        // carry (r x ldn) = Linv * H[slot]
    OP_COUNT
};
void gemm_f32_dims(int op, const MatDev& md, int* M, int* N, int* K);
// max_m, max_n, max_k: largest dimensions of the product over the layer set (grid and tile choice)
hipError_t launch_gemm_f32(GemmOp op, const MatDev* mats, const MatDyn* dyn, int n_mats,
                           int max_m, int max_n, int max_k, int grad_dtype, StepScalars sc,
                           const void* zero16, hipStream_t stream);

// bf16 MFMA GEMMs of the step (k_gemm_bf16.hip)
// which: 0 projection (direct-to-LDS kernel), 1 update, 2 projection (register-staged kernel)
void bf16_tile_shape(int which, int max_r, int* bm, int* bn);
// zero16: 16 bytes of zeros in device memory (fetched in place of out-of-range operand chunks)
// The projection's tile table has three runs, each with its own kernel: n_direct left-side tiles for
// the direct-to-LDS kernel (see projection_tile_direct), then n_staged other left-side tiles, then
// n_right right-side tiles.
hipError_t launch_project_bf16(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_direct,
                               int n_staged, int n_right, int max_r, int hist_bf16, const void* zero16,
                               hipStream_t stream);
// sides: bit 0 = left-side matrices present, bit 1 = right-side ones (one kernel instance each)
hipError_t launch_update_bf16(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles,
                              StepScalars sc, const void* zero16, int sides, hipStream_t stream);

// Refresh products of a bf16 gradient with an fp32 sketch matrix Y as three bf16 MFMA products (left side).
// form 1: Ya = G Y, form 2: Yb = G^T Y, form 3: Bm = Y^T G; ysrc: Y is 0 Ya, 1 Yb, 2 Yc;
// planes: how many of Y's three bf16 planes enter (1: form 1 only; 2: forms 1 and 2; 3: any form);
// max_m / max_n: largest row / column count of the result over the layer set
hipError_t launch_refresh_x3(int form, int ysrc, int planes, const MatDev* mats, const MatDyn* dyn, int n_mats,
                             int max_m, int max_n, hipStream_t stream);

// Projection and update of fp32 layer sets with ranks <= kSkinnyMaxRank, left side (k_skinny.hip).
// tiles: one entry per kSkinnyRows x kSkinnyCols block of the m x ldn range of every matrix; rk: 4, 8
// or 16, at least the largest rank of the set (the row pitch of MatDev::skinny_parts).
hipError_t launch_project_skinny(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles, int n_mats,
                                 int max_ldn, int rk, hipStream_t stream);
hipError_t launch_update_skinny(const MatDev* mats, const MatDyn* dyn, const TileRef* tiles, int n_tiles, int rk,
                                StepScalars sc, hipStream_t stream);

// Gram row, solve, fused transform + Adam (k_elementwise.hip)
// row_override >= 0: the Gram row of that slot instead of the step's head (history carry-over);
// launch_solve then only stores the row and column of K and skips the solve
hipError_t launch_gram_row(const MatDev* mats, const MatDyn* dyn, const TileRef* chunks, int n_chunks,
                           int s, int hist_bf16, int row_override, hipStream_t stream);
hipError_t launch_solve(const MatDev* mats, const MatDyn* dyn, int first, int n_mats, StepScalars sc,
                        int row_override, int* status, hipStream_t stream);
hipError_t launch_save_projector(const MatDev* mats, int n_mats, hipStream_t stream);   // Yc <- P
hipError_t launch_carry_store(const MatDev* mats, int n_mats, int slot, int hist_bf16, hipStream_t stream);
hipError_t launch_transform_adam(const MatDev* mats, const MatDyn* dyn, const TileRef* patches, int n_patches,
                                 StepScalars sc, int grad_dtype, int* status, hipStream_t stream);
hipError_t launch_make_bf16_copies(const MatDev* mats, int n_mats, int max_m, int max_r, hipStream_t stream);

// refresh helpers (k_refresh.hip)
hipError_t launch_fill_gaussian(const MatDev* mats, int n_mats, int max_rows, unsigned long long seed,
                                unsigned long long call_id, hipStream_t stream);   // fills Yb (n x l)
// which: 0 -> order l (sketch), 1 -> order r (final P)
hipError_t launch_cholesky(const MatDev* mats, int n_mats, int which, int max_order, double shift_rel,
                           int* status, hipStream_t stream);
hipError_t launch_tri_inverse(const MatDev* mats, int n_mats, int which, int max_order, hipStream_t stream);
hipError_t launch_jacobi_prepare(const MatDev* mats, int n_mats, hipStream_t stream);
hipError_t launch_jacobi_round(const MatDev* mats, int n_mats, int max_pairs, int round, hipStream_t stream);
hipError_t launch_jacobi_sweep_end(const MatDev* mats, int n_mats, hipStream_t stream);
hipError_t launch_jacobi_finish(const MatDev* mats, int n_mats, int* status, hipStream_t stream);
hipError_t launch_sign_fix(const MatDev* mats, int n_mats, int max_r, hipStream_t stream);

// micro-benchmarks (k_microbench.hip)
hipError_t launch_mb_copy(const void* src, void* dst, size_t bytes, hipStream_t stream);
hipError_t launch_mb_read(const void* src, size_t bytes, void* sink, hipStream_t stream);
hipError_t launch_mb_mfma(int iters, int waves_per_simd, bool random_operands, void* sink, double* flops,
                          hipStream_t stream);

}  // namespace ng
