// C ABI and host-side scheduler of the Natural GaLore step library.
// Validates arguments, owns the integer bookkeeping (step counter, ring head,
// valid-slot count, refresh count), lays out the caller's workspace and
// enqueues the grouped kernels of every phase.  Allocates no device memory.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "ng_internal.h"

using namespace ng;

// Step scratch of ng_step_static: device memory of the library itself, so that entry point needs
// neither a workspace argument nor an allocation.  Never passed to a kernel by name (in host code
// the name is not a device address): see static_scratch_of_current_device.
static __device__ __align__(256) unsigned char g_ng_static_scratch[ng::kStaticScratchBytes];

// Round-robin workgroup dispatch puts workgroup id w on XCD (w mod 8).  To let one XCD work
// through a contiguous run of the logical tile order (tiles that share operand panels stay in one
// L2), the logical order is cut into 8 runs of about equal cost (cost[i] = contraction length of tile
// i) and hardware id w takes entry w / 8 of run w mod 8.  Inside a run the tiles are taken longest
// first (stable: tiles of one matrix stay together): an XCD's units pick tiles off its run as they
// become free, and a run that ends with its longest tiles leaves most units idle while the last few
// finish (the 5461-deep tiles of a 1.1B-shaped block are 2.7 times as long as the others).
// Runs shorter than the longest are padded with entries whose workgroups exit at once.
void ng::xcd_order(const std::vector<TileRef>& logical, const std::vector<int>& cost, std::vector<TileRef>* out) {
    const size_t T = logical.size();
    out->clear();
    if (T == 0) return;
    double total = 0.0;
    for (size_t i = 0; i < T; ++i) total += (double)cost[i];
    std::vector<std::vector<size_t>> run(8);
    double acc = 0.0;
    for (size_t i = 0; i < T; ++i) {
        // the run in which the tile's midpoint falls
        size_t x = (size_t)((acc + 0.5 * (double)cost[i]) * 8.0 / total);
        run[x < 8 ? x : 7].push_back(i);
        acc += (double)cost[i];
    }
    size_t per = 0;
    for (auto& r : run) {
        std::stable_sort(r.begin(), r.end(), [&](size_t a, size_t b) { return cost[a] > cost[b]; });
        per = r.size() > per ? r.size() : per;
    }
    out->assign(per * 8, TileRef{-1, 0, 0, 0});
    for (size_t x = 0; x < 8; ++x)
        for (size_t k = 0; k < run[x].size(); ++k) (*out)[k * 8 + x] = logical[run[x][k]];
}

namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

struct Sizes {   // per-matrix derived sizes
    int ldn, pw, l, ldk, ldr, roct, lp;
    size_t bytes[NG_NBUF];
    size_t k_gram_off, k_w64_off, k_w32_off;
    size_t aux_pb_off, aux_pbt_off;
    // refresh scratch
    size_t ws_y, ws_bm, ws_t, ws_linv, ws_ritz, ws_order, ws_flag, ws_parts, ws_carry, ws_skinny;
};

int validate(const ng_matrix_desc* d, int n_mats, const ng_hparams* hp) {
    if (!d || !hp || n_mats <= 0) return NG_ERR_INVALID_ARG;
    if (hp->grad_dtype != NG_F32 && hp->grad_dtype != NG_BF16) return NG_ERR_DTYPE;
    if (hp->hist_dtype != NG_F32 && hp->hist_dtype != NG_BF16) return NG_ERR_DTYPE;
    if (hp->hist_dtype == NG_BF16 && hp->grad_dtype != NG_BF16) return NG_ERR_DTYPE;
    if (hp->fisher_norm != NG_NORM_S && hp->fisher_norm != NG_NORM_COUNT) return NG_ERR_HPARAM;
    if (hp->carry_history != 0 && hp->carry_history != 1) return NG_ERR_HPARAM;
    if (hp->proj_dtype != NG_F32 && hp->proj_dtype != NG_BF16) return NG_ERR_DTYPE;
    // the low-memory projector lives in the bf16 copies only: they exist for bf16 gradients, and the
    // history carry-over needs the outgoing float projector
    if (hp->proj_dtype == NG_BF16 && (hp->grad_dtype != NG_BF16 || hp->carry_history != 0)) return NG_ERR_HPARAM;
    if (hp->adam_mode != NG_ADAM_STANDARD && hp->adam_mode != NG_ADAM_PRINTED) return NG_ERR_DTYPE;
    if (hp->s < 0 || hp->s > kMaxS) return NG_ERR_SHAPE;
    if (!(hp->lambda > 0.f) || !isfinite(hp->lambda)) return NG_ERR_HPARAM;
    if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f)) return NG_ERR_HPARAM;
    if (!(hp->eps > 0.f) || !isfinite(hp->eps)) return NG_ERR_HPARAM;
    if (!isfinite(hp->scale) || !isfinite(hp->weight_decay)) return NG_ERR_HPARAM;
    if (hp->refresh_power_iters < 0 || hp->refresh_power_iters > 16) return NG_ERR_HPARAM;
    if (hp->refresh_oversample < 0 || hp->refresh_sweeps < 1 || hp->refresh_sweeps > 64) return NG_ERR_HPARAM;
    for (int i = 0; i < n_mats; ++i) {
        const ng_matrix_desc& x = d[i];
        if (x.m <= 0 || x.n <= 0 || x.r <= 0) return NG_ERR_SHAPE;
        if (x.r > x.m || x.r > x.n) return NG_ERR_SHAPE;
        if (x.ld_w < x.n || x.ld_g < x.n) return NG_ERR_SHAPE;
        if (x.side != NG_SIDE_LEFT && x.side != NG_SIDE_RIGHT) return NG_ERR_INVALID_ARG;
        if ((long long)x.m > (1 << 24) || (long long)x.n > (1 << 24)) return NG_ERR_SHAPE;
        if ((long long)x.r + hp->refresh_oversample > 2048) return NG_ERR_SHAPE;   // widest sketch the refresh is specified for
        // the kernels address one matrix with 32-bit offsets
        const long long ldmax = x.ld_w > x.ld_g ? x.ld_w : x.ld_g;
        if ((long long)x.m * ldmax * 4 >= (1LL << 31)) return NG_ERR_SHAPE;
        if ((long long)x.r * ((x.m > x.n ? x.m : x.n) + 32) * 4 >= (1LL << 31)) return NG_ERR_SHAPE;
    }
    return NG_OK;
}

bool hist_is_bf16(const ng_hparams& hp) { return hp.hist_dtype == NG_BF16; }

// The descriptor of the problem the kernels see: the right-side form is the left-side form of the
// transposed matrix (m and n swapped; the leading dimensions still describe the caller's arrays).
ng_matrix_desc effective(const ng_matrix_desc& u) {
    ng_matrix_desc d = u;
    if (u.side == NG_SIDE_RIGHT) {
        d.m = u.n;
        d.n = u.m;
    }
    return d;
}

// skinny_rk: 0, or the rank class (4, 8, 16) of a layer set that takes the small-rank kernels
void derive(const ng_matrix_desc& user, const ng_hparams& hp, int skinny_rk, Sizes* z) {
    const ng_matrix_desc d = effective(user);
    memset(z, 0, sizeof(*z));
    const int s = hp.s;
    z->ldn = (int)align_up((size_t)d.n, 32);
    // Wide states of bf16 layer sets are stored as column panels (see state_panel).  Only the bf16
    // projection and the transform address them in two dimensions; the fp32 GEMMs that the fp32
    // path and the history carry-over run on the slots want plain row-major.
    // (a last panel narrower than two patches would be all row ends: such rows stay whole)
    z->pw = (hp.grad_dtype == NG_BF16 && !hp.carry_history && z->ldn >= kStatePanelCols + 256) ? kStatePanelCols : z->ldn;
    int l = d.r + hp.refresh_oversample;
    if (l > d.m) l = d.m;
    if (l > d.n) l = d.n;
    // the refresh's products and its eigen-solve work on 32-wide blocks: a sketch width just above a
    // multiple of 32 (r = 512, p = 8) would pay for a whole block to carry a few columns, so the
    // width is trimmed to that multiple when it still holds the r columns wanted
    if (l / 32 * 32 >= d.r) l = l / 32 * 32;
    z->l = l;
    z->ldk = (int)align_up((size_t)d.m, 32);
    z->ldr = (int)align_up((size_t)d.r, 32);
    z->roct = ceil_div(d.r, 8);
    z->lp = (int)align_up((size_t)l, (size_t)2 * kJacobiBlock);
    const size_t rn = (size_t)d.r * z->ldn;
    const size_t state = (size_t)d.r * state_cols(z->ldn, z->pw);   // elements of M, V, a history slot as stored
    z->bytes[NG_BUF_P] = hp.proj_dtype == NG_BF16 ? 0 : align_up((size_t)d.m * d.r * 4, 256);
    z->bytes[NG_BUF_M] = align_up(state * 4, 256);
    z->bytes[NG_BUF_V] = align_up(state * 4, 256);
    z->bytes[NG_BUF_H] = align_up(state * (hist_is_bf16(hp) ? 2 : 4) * (size_t)(s > 0 ? s : 1), 256);
    z->k_gram_off = 0;
    z->k_w64_off = align_up((size_t)s * s * 8, 16);
    z->k_w32_off = z->k_w64_off + align_up((size_t)s * 8, 16);
    z->bytes[NG_BUF_K] = align_up(z->k_w32_off + (size_t)s * 4 + 16, 256);
    if (hp.grad_dtype == NG_BF16) {
        z->bytes[NG_BUF_N] = align_up((size_t)z->roct * z->ldn * 8 * 2, 256);
        z->aux_pb_off = 0;
        z->aux_pbt_off = align_up((size_t)d.m * z->ldr * 2, 256);
        z->bytes[NG_BUF_AUX] = z->aux_pbt_off + align_up((size_t)d.r * z->ldk * 2, 256);
    } else {
        z->bytes[NG_BUF_N] = align_up(rn * 4, 256);
        z->bytes[NG_BUF_AUX] = 0;
    }
    const size_t rows = (size_t)(d.m > d.n ? d.m : d.n);
    z->ws_y = align_up(rows * l * 4, 256);
    z->ws_bm = align_up((size_t)l * z->ldn * 4, 256);
    z->ws_t = align_up((size_t)z->lp * z->lp * 8, 256);
    z->ws_linv = align_up((size_t)z->lp * z->lp * 4, 256);
    z->ws_ritz = align_up((size_t)z->lp * 8, 256);
    z->ws_order = align_up((size_t)z->lp * 4, 256);
    z->ws_flag = 256;
    z->ws_carry = hp.carry_history ? align_up(rn * 4, 256) : 0;
    z->ws_parts = align_up((size_t)kDotPartsMax * (s > 0 ? s : 1) * 8, 256);
    z->ws_skinny = skinny_rk ? align_up((size_t)ceil_div(d.m, kSkinnyRows) * skinny_rk * z->ldn * 4, 256) : 0;
}

// Tables that live at the front of the workspace.
struct Plan {
    std::vector<Sizes> sz;
    std::vector<TileRef> proj, upd, dots, patches, skinny;
    int skinny_rk;                              // 0: the MFMA / fp32-GEMM projection and update
    int proj_direct, proj_staged, proj_right;   // lengths of the three runs of proj
    size_t off_status, off_mats, off_step, off_proj, off_upd, off_dots, off_patches, off_skinny, off_scratch;
    // the scratch block of one step: the per-step table, then what the step's kernels hand to each
    // other (offsets from the start of the block; per matrix)
    size_t step_tail8_off, step_bytes;
    std::vector<size_t> step_parts_off, step_skinny_off;
    size_t total;
};

void make_plan(const ng_matrix_desc* d, int n_mats, const ng_hparams& hp, Plan* p) {
    p->sz.resize(n_mats);
    int max_r = 0;
    for (int i = 0; i < n_mats; ++i) max_r = d[i].r > max_r ? d[i].r : max_r;
    int pbm = 128, pbn = 128, sbm = 128, sbn = 128, ubm = 128, ubn = 128;
    bf16_tile_shape(0, max_r, &pbm, &pbn);
    bf16_tile_shape(2, max_r, &sbm, &sbn);
    bf16_tile_shape(1, max_r, &ubm, &ubn);
    std::vector<TileRef> proj_direct, proj_staged, proj_right, upd;
    std::vector<int> cost_direct, cost_staged, cost_right, cost_upd;   // contraction length per tile
    p->dots.clear();
    p->patches.clear();
    p->skinny.clear();
    // fp32 gradients, ranks far below an MFMA tile, all matrices on the left side: the vector-ALU
    // projection and update
    bool all_left = true;
    for (int i = 0; i < n_mats; ++i) all_left = all_left && d[i].side == NG_SIDE_LEFT;
    p->skinny_rk = (hp.grad_dtype == NG_F32 && all_left && max_r <= kSkinnyMaxRank) ? (max_r <= 4 ? 4 : max_r <= 8 ? 8 : 16) : 0;
    for (int i = 0; i < n_mats; ++i) {
        derive(d[i], hp, p->skinny_rk, &p->sz[i]);
        const Sizes& z = p->sz[i];
        if (p->skinny_rk) {
            for (int ti = 0; ti < ceil_div(d[i].m, kSkinnyRows); ++ti)
                for (int tj = 0; tj < ceil_div(z.ldn, kSkinnyCols); ++tj) p->skinny.push_back(TileRef{i, ti, tj, 0});
        } else if (hp.grad_dtype == NG_BF16) {
            const bool direct = d[i].side != NG_SIDE_RIGHT && projection_tile_direct(effective(d[i]).n);
            std::vector<TileRef>& run = direct ? proj_direct : d[i].side == NG_SIDE_RIGHT ? proj_right : proj_staged;
            std::vector<int>& run_cost = direct ? cost_direct : d[i].side == NG_SIDE_RIGHT ? cost_right : cost_staged;
            const int bm = direct ? pbm : sbm, bn = direct ? pbn : sbn;
            for (int tj = 0; tj < ceil_div(z.ldn, bn); ++tj)
                for (int ti = 0; ti < ceil_div(d[i].r, bm); ++ti) {
                    run.push_back(TileRef{i, ti, tj, 0});
                    run_cost.push_back(effective(d[i]).m);
                }
            // update tiles cover the weight in the caller's orientation on either side.  Consecutive
            // tiles share one operand panel; the other operand is swept whole once per panel, so the
            // loop order keeps the smaller of the two whole operands (rows x r against r x columns) as
            // the one that is swept: it is the one that has to stay in the L2
            if (d[i].m > d[i].n) {
                for (int ti = 0; ti < ceil_div(d[i].m, ubm); ++ti)
                    for (int tj = 0; tj < ceil_div(d[i].n, ubn); ++tj) upd.push_back(TileRef{i, ti, tj, 0});
            } else {
                for (int tj = 0; tj < ceil_div(d[i].n, ubn); ++tj)
                    for (int ti = 0; ti < ceil_div(d[i].m, ubm); ++ti) upd.push_back(TileRef{i, ti, tj, 0});
            }
            cost_upd.resize(upd.size(), d[i].r);
        }
        for (int ti = 0; ti < ceil_div(d[i].r, 32); ++ti)
            for (int tj = 0; tj < ceil_div(z.ldn, kAdamPatchCols); ++tj) p->patches.push_back(TileRef{i, ti, tj, 0});
    }
    {
        std::vector<TileRef> a, b, c;
        xcd_order(proj_direct, cost_direct, &a);
        xcd_order(proj_staged, cost_staged, &b);
        xcd_order(proj_right, cost_right, &c);
        p->proj_direct = (int)a.size();
        p->proj_staged = (int)b.size();
        p->proj_right = (int)c.size();
        p->proj = a;
        p->proj.insert(p->proj.end(), b.begin(), b.end());
        p->proj.insert(p->proj.end(), c.begin(), c.end());
    }
    xcd_order(upd, cost_upd, &p->upd);
    // Gram-row parts are appended in make_mats (they need dot_nparts)
    size_t off = 0;
    p->off_status = off; off += 256;
    p->off_mats = off;   off += align_up(sizeof(MatDev) * (size_t)n_mats, 256);
    {
        size_t so = align_up(sizeof(MatDyn) * (size_t)n_mats, 256);
        p->step_tail8_off = so;
        so += align_up((size_t)16 * (size_t)n_mats, 256);
        p->step_parts_off.resize(n_mats);
        p->step_skinny_off.resize(n_mats);
        for (int i = 0; i < n_mats; ++i) {
            p->step_parts_off[i] = so;
            so += p->sz[i].ws_parts;
            p->step_skinny_off[i] = so;
            so += p->sz[i].ws_skinny;
        }
        p->step_bytes = so;
    }
    p->off_step = off;   off += p->step_bytes;
    p->off_proj = off;   off += align_up(sizeof(TileRef) * p->proj.size(), 256);
    p->off_upd = off;    off += align_up(sizeof(TileRef) * p->upd.size(), 256);
    p->off_dots = off;   off += align_up(sizeof(TileRef) * (size_t)n_mats * kDotPartsMax, 256);
    p->off_patches = off; off += align_up(sizeof(TileRef) * p->patches.size(), 256);
    p->off_skinny = off;  off += align_up(sizeof(TileRef) * p->skinny.size(), 256);
    p->off_scratch = off;
    for (int i = 0; i < n_mats; ++i) {
        const Sizes& z = p->sz[i];
        off += 3 * z.ws_y + z.ws_bm + z.ws_t + z.ws_linv + z.ws_ritz + z.ws_order + z.ws_flag + z.ws_carry;
    }
    p->total = off;
}

constexpr int kProfRing = 64;

}  // namespace

struct ng_state {
    int n_mats;
    ng_hparams hp;
    std::vector<ng_matrix_desc> descs;
    std::vector<ng_matrix_buffers> bufs;
    std::vector<MatDev> mats;
    Plan plan;
    std::vector<int64_t> t, n_refresh;
    std::vector<int32_t> head, count;
    bool projector_valid;
    bool tables_valid;   // the workspace tables are on the device (false for NG_INIT_HOST_ONLY: nothing may launch)
    char* ws;
    MatDev* d_mats;
    MatDyn* d_dyn;
    int* d_status;
    TileRef *d_proj, *d_upd, *d_dots, *d_patches, *d_skinny;
    int n_dots;
    int max_m, max_n, max_r, max_l, max_lp, max_rows, max_ldn;
    int max_ti[OP_COUNT], max_tj[OP_COUNT], max_tk[OP_COUNT];   // largest M, N, K of each fp32 product
    int max_jpairs;
    int sides;       // bit 0: left-side matrices present, bit 1: right-side ones
    // profiling
    bool profiling;
    hipEvent_t ev[kProfRing][NG_NPHASE + 1];
    bool ev_created;
    int ev_head, ev_pending;
    double phase_ms[NG_NPHASE];
    int64_t phase_steps;
};

namespace {

#define NG_HIP(expr)                        \
    do {                                    \
        hipError_t e_ = (expr);             \
        if (e_ != hipSuccess) return NG_ERR_HIP; \
    } while (0)

int upload_dyn(ng_state* st, MatDyn* dyn, const void* const* grads, void* const* weights, bool stepping,
               hipStream_t stream) {
    DynChunk chunk;
    const int s = st->hp.s;
    for (int first = 0; first < st->n_mats; first += kDynChunk) {
        int n = st->n_mats - first;
        if (n > kDynChunk) n = kDynChunk;
        memset(&chunk, 0, sizeof(chunk));
        for (int i = 0; i < n; ++i) {
            const int k = first + i;
            MatDyn& e = chunk.e[i];
            e.g = grads ? grads[k] : nullptr;
            e.w = weights ? weights[k] : nullptr;
            e.head = (s > 0) ? st->head[k] : 0;
            int c = st->count[k] + (stepping ? 1 : 0);
            e.count = c > s ? s : c;
            const double tt = (double)(st->t[k] + 1);
            if (st->hp.adam_mode == NG_ADAM_STANDARD) {
                e.bc1 = (float)(1.0 / (1.0 - pow((double)st->hp.beta1, tt)));
                e.bc2 = (float)(1.0 / sqrt(1.0 - pow((double)st->hp.beta2, tt)));
            } else {
                e.bc1 = 1.f;
                e.bc2 = 1.f;
            }
        }
        NG_HIP(launch_upload_dyn(dyn, chunk, first, n,
                                 (stepping && st->hp.grad_dtype == NG_BF16) ? st->d_mats : nullptr, stream));
    }
    return NG_OK;
}

StepScalars make_scalars(const ng_state* st, float lr) {
    StepScalars sc;
    memset(&sc, 0, sizeof(sc));
    sc.lambda = st->hp.lambda;
    sc.beta1 = st->hp.beta1;
    sc.beta2 = st->hp.beta2;
    sc.eps = st->hp.eps;
    sc.lr_scale = lr * st->hp.scale;
    sc.lr_wd = lr * st->hp.weight_decay;
    sc.adam_mode = st->hp.adam_mode;
    sc.s = st->hp.s > 0 ? st->hp.s : 1;
    sc.use_fisher = st->hp.s > 0 ? 1 : 0;
    sc.hist_bf16 = hist_is_bf16(st->hp) ? 1 : 0;
    sc.norm_count = st->hp.fisher_norm == NG_NORM_COUNT ? 1 : 0;
    return sc;
}

int clear_history(ng_state* st, hipStream_t stream) {
    if (st->n_mats == 0) return NG_OK;
    NG_HIP(launch_clear_history(st->d_mats, st->n_mats, st->hp.s, hist_is_bf16(st->hp) ? 2 : 4,
                                st->plan.sz[0].bytes[NG_BUF_K], stream));
    return NG_OK;
}

// The refresh's products with the gradient: OP_G_B2A / OP_G_C2A (Ya = G Y), OP_GT_C2B (Yb = G^T Y),
// OP_QT_G (Bm = Ya^T G).  bf16 gradients on the left side take three bf16 MFMA
// products (launch_refresh_x3), everything else the fp32 GEMM.
int gemm(ng_state* st, GemmOp op, hipStream_t stream, const StepScalars& sc, const MatDyn* dyn = nullptr);
int gradient_product(ng_state* st, GemmOp op, bool last, hipStream_t stream, const StepScalars& sc) {
    if (st->hp.grad_dtype == NG_BF16 && !(st->sides & 2)) {
        // planes of the sketch that enter: the random test matrix needs one, the last basis and
        // B = Q^T G all three, the products inside the subspace iteration two
        int form = 0, ysrc = 0, planes = last ? 3 : 2;
        switch (op) {
            case OP_G_B2A: form = 1; ysrc = 1; planes = 1; break;
            case OP_G_C2A: form = 1; ysrc = 2; break;
            case OP_GT_C2B: form = 2; ysrc = 2; break;
            case OP_QT_G: form = 3; ysrc = 0; planes = 3; break;
            default: break;
        }
        if (form != 0) {
            NG_HIP(launch_refresh_x3(form, ysrc, planes, st->d_mats, st->d_dyn, st->n_mats, st->max_ti[op], st->max_tj[op], stream));
            return NG_OK;
        }
    }
    return gemm(st, op, stream, sc);
}

int gemm(ng_state* st, GemmOp op, hipStream_t stream, const StepScalars& sc, const MatDyn* dyn) {
    NG_HIP(launch_gemm_f32(op, st->d_mats, dyn ? dyn : st->d_dyn, st->n_mats, st->max_ti[op], st->max_tj[op], st->max_tk[op],
                           st->hp.grad_dtype, sc, (const char*)st->d_status + 64, stream));
    return NG_OK;
}

// CholeskyQR of the sketch X (Ya if is_a, else Yb).
//   twice = false: one pass with a small diagonal shift, result left in Yc -- enough to keep the
//                  power iteration from collapsing;
//   twice = true : a second, unshifted pass repairs the first pass's loss of orthogonality and
//                  puts the result back in X (the basis handed to the Rayleigh-Ritz step).
int orthonormalise(ng_state* st, bool is_a, bool twice, hipStream_t stream, const StepScalars& sc) {
    int rc;
    if ((rc = gemm(st, is_a ? OP_GRAM_A : OP_GRAM_B, stream, sc)) != NG_OK) return rc;
    NG_HIP(launch_cholesky(st->d_mats, st->n_mats, 0, st->max_l, 2e-7, st->d_status, stream));
    NG_HIP(launch_tri_inverse(st->d_mats, st->n_mats, 0, st->max_l, stream));
    if ((rc = gemm(st, is_a ? OP_APPLY_A2C : OP_APPLY_B2C, stream, sc)) != NG_OK) return rc;
    if (!twice) return NG_OK;
    if ((rc = gemm(st, is_a ? OP_GRAM_CA : OP_GRAM_CB, stream, sc)) != NG_OK) return rc;
    NG_HIP(launch_cholesky(st->d_mats, st->n_mats, 0, st->max_l, 0.0, st->d_status, stream));
    NG_HIP(launch_tri_inverse(st->d_mats, st->n_mats, 0, st->max_l, stream));
    if ((rc = gemm(st, is_a ? OP_APPLY_C2A : OP_APPLY_C2B, stream, sc)) != NG_OK) return rc;
    return NG_OK;
}

// copies: build the bf16 copies from the float projector (a commit of a low-memory layer set has none)
int finish_projector(ng_state* st, bool clear, bool copies, hipStream_t stream) {
    copies = copies && st->hp.grad_dtype == NG_BF16;
    if (!st->tables_valid && (clear || copies)) return NG_ERR_HIP;
    if (copies)
        NG_HIP(launch_make_bf16_copies(st->d_mats, st->n_mats, st->max_m, st->max_r, stream));
    if (clear) {
        int rc = clear_history(st, stream);
        if (rc != NG_OK) return rc;
    }
    return NG_OK;
}

void drain_events(ng_state* st, bool all) {
    while (st->ev_pending > 0 && (all || st->ev_pending >= kProfRing)) {
        int slot = (st->ev_head - st->ev_pending + 2 * kProfRing) % kProfRing;
        if (hipEventSynchronize(st->ev[slot][NG_NPHASE]) == hipSuccess) {
            for (int p = 0; p < NG_NPHASE; ++p) {
                float ms = 0.f;
                if (hipEventElapsedTime(&ms, st->ev[slot][p], st->ev[slot][p + 1]) == hipSuccess)
                    st->phase_ms[p] += ms;
            }
            st->phase_steps += 1;
        }
        st->ev_pending -= 1;
    }
}

// One step.  `dyn` is the start of the scratch block the step's kernels use: the per-step table and,
// behind it, what they hand to each other (see MatDev::dot_parts_off).
int step_on_scratch(ng_state* st, const void* const* grads, void* const* weights, float lr, hipStream_t stream,
                    MatDyn* dyn) {
    if (!grads || !weights) return NG_ERR_INVALID_ARG;
    if (!isfinite(lr)) return NG_ERR_HPARAM;
    for (int i = 0; i < st->n_mats; ++i)
        if (!grads[i] || !weights[i]) return NG_ERR_INVALID_ARG;
    if (!st->projector_valid) return NG_ERR_NO_PROJECTOR;
    if (!st->tables_valid) return NG_ERR_HIP;
    const StepScalars sc = make_scalars(st, lr);
    const bool bf = st->hp.grad_dtype == NG_BF16;
    const bool prof = st->profiling && st->ev_created;
    int slot = 0;
    if (prof) {
        drain_events(st, false);
        slot = st->ev_head;
    }
    int rc;
    if ((rc = upload_dyn(st, dyn, grads, weights, true, stream)) != NG_OK) return rc;

    if (prof) NG_HIP(hipEventRecord(st->ev[slot][NG_PHASE_PROJECT], stream));
    const int skinny_rk = st->plan.skinny_rk;
    if (skinny_rk) NG_HIP(launch_project_skinny(st->d_mats, dyn, st->d_skinny, (int)st->plan.skinny.size(), st->n_mats,
                                                st->max_ldn, skinny_rk, stream));
    else if (bf) NG_HIP(launch_project_bf16(st->d_mats, dyn, st->d_proj, st->plan.proj_direct, st->plan.proj_staged,
                                            st->plan.proj_right, st->max_r, sc.hist_bf16, (const char*)st->d_status + 64,
                                            stream));
    else if ((rc = gemm(st, OP_PROJECT_F32, stream, sc, dyn)) != NG_OK) return rc;

    if (prof) NG_HIP(hipEventRecord(st->ev[slot][NG_PHASE_GRAM], stream));
    if (sc.use_fisher) NG_HIP(launch_gram_row(st->d_mats, dyn, st->d_dots, st->n_dots, sc.s, sc.hist_bf16, -1, stream));

    if (prof) NG_HIP(hipEventRecord(st->ev[slot][NG_PHASE_SOLVE], stream));
    if (sc.use_fisher) NG_HIP(launch_solve(st->d_mats, dyn, 0, st->n_mats, sc, -1, st->d_status, stream));

    if (prof) NG_HIP(hipEventRecord(st->ev[slot][NG_PHASE_ADAM], stream));
    NG_HIP(launch_transform_adam(st->d_mats, dyn, st->d_patches, (int)st->plan.patches.size(), sc,
                                 st->hp.grad_dtype, st->d_status, stream));

    if (prof) NG_HIP(hipEventRecord(st->ev[slot][NG_PHASE_UPDATE], stream));
    if (skinny_rk) NG_HIP(launch_update_skinny(st->d_mats, dyn, st->d_skinny, (int)st->plan.skinny.size(), skinny_rk,
                                               sc, stream));
    else if (bf) NG_HIP(launch_update_bf16(st->d_mats, dyn, st->d_upd, (int)st->plan.upd.size(), sc,
                                           (const char*)st->d_status + 64, st->sides, stream));
    else if ((rc = gemm(st, OP_UPDATE_F32, stream, sc, dyn)) != NG_OK) return rc;

    if (prof) {
        NG_HIP(hipEventRecord(st->ev[slot][NG_NPHASE], stream));
        st->ev_head = (st->ev_head + 1) % kProfRing;
        st->ev_pending += 1;
    }

    const int s = st->hp.s;
    for (int i = 0; i < st->n_mats; ++i) {
        st->t[i] += 1;
        if (s > 0) {
            st->head[i] = (st->head[i] + 1) % s;
            if (st->count[i] < s) st->count[i] += 1;
        }
    }
    return NG_OK;
}

// ---------------------------------------------------------------- the library's own step scratch
// One array per GPU (every device that loads this code object holds its own copy at its own
// address).  In host code the array's name is only a handle for hipGetSymbolAddress: the device
// address is looked up once per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
char* g_static_ptr[kMaxDevices] = {nullptr};

int static_scratch_of_current_device(char** out) {
    int dev = -1;
    NG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return NG_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        NG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_ng_static_scratch)));
        if (!p) return NG_ERR_HIP;
        g_static_ptr[dev] = (char*)p;
    }
    *out = g_static_ptr[dev];
    return NG_OK;
}

}  // namespace

extern "C" {

int ng_default_hparams(ng_hparams* hp) {
    if (!hp) return NG_ERR_INVALID_ARG;
    memset(hp, 0, sizeof(*hp));
    hp->s = 4;
    hp->lambda = 1e-3f;
    hp->beta1 = 0.9f;
    hp->beta2 = 0.999f;
    hp->eps = 1e-8f;
    hp->scale = 1.0f;
    hp->weight_decay = 0.0f;
    hp->grad_dtype = NG_F32;
    hp->hist_dtype = NG_F32;
    hp->fisher_norm = NG_NORM_S;
    hp->carry_history = 0;
    hp->proj_dtype = NG_F32;
    hp->adam_mode = NG_ADAM_STANDARD;
    hp->refresh_power_iters = 2;
    hp->refresh_oversample = 8;
    hp->refresh_sweeps = 30;
    hp->seed = 0;
    return NG_OK;
}

int ng_query_sizes(const ng_matrix_desc* descs, int n_mats, const ng_hparams* hp, size_t* bytes,
                   size_t* workspace_bytes) {
    int rc = validate(descs, n_mats, hp);
    if (rc != NG_OK) return rc;
    if (!bytes || !workspace_bytes) return NG_ERR_INVALID_ARG;
    try {
        Plan plan;
        make_plan(descs, n_mats, *hp, &plan);
        for (int i = 0; i < n_mats; ++i)
            for (int b = 0; b < NG_NBUF; ++b) bytes[(size_t)i * NG_NBUF + b] = plan.sz[i].bytes[b];
        *workspace_bytes = plan.total;
    } catch (...) {
        return NG_ERR_INVALID_ARG;
    }
    return NG_OK;
}

int ng_init_state(const ng_matrix_desc* descs, const ng_matrix_buffers* bufs, int n_mats, const ng_hparams* hp,
                  void* workspace, size_t workspace_bytes, uint32_t flags, ng_stream stream_, ng_state** out) {
    hipStream_t stream = (hipStream_t)stream_;
    int rc = validate(descs, n_mats, hp);
    if (rc != NG_OK) return rc;
    if (!bufs || !out || !workspace) return NG_ERR_INVALID_ARG;
    if (((uintptr_t)workspace & 255) != 0) return NG_ERR_WORKSPACE;
    ng_state* st = nullptr;
    try {
        st = new ng_state();
        st->n_mats = n_mats;
        st->hp = *hp;
        st->descs.assign(descs, descs + n_mats);
        st->bufs.assign(bufs, bufs + n_mats);
        make_plan(descs, n_mats, *hp, &st->plan);
        if (workspace_bytes < st->plan.total) {
            delete st;
            return NG_ERR_WORKSPACE;
        }
        for (int i = 0; i < n_mats; ++i)
            for (int b = 0; b < NG_NBUF; ++b) {
                if (st->plan.sz[i].bytes[b] == 0) continue;
                void* p = bufs[i].buf[b];
                if (!p || ((uintptr_t)p & 15) != 0) {
                    delete st;
                    return NG_ERR_INVALID_ARG;
                }
            }
        st->t.assign(n_mats, 0);
        st->n_refresh.assign(n_mats, 0);
        st->head.assign(n_mats, 0);
        st->count.assign(n_mats, 0);
        st->projector_valid = false;
        st->profiling = false;
        st->ev_created = false;
        st->ev_head = st->ev_pending = 0;
        memset(st->phase_ms, 0, sizeof(st->phase_ms));
        st->phase_steps = 0;

        char* ws = (char*)workspace;
        st->ws = ws;
        const Plan& pl = st->plan;
        st->d_status = (int*)(ws + pl.off_status);
        st->d_mats = (MatDev*)(ws + pl.off_mats);
        st->d_dyn = (MatDyn*)(ws + pl.off_step);
        st->d_proj = (TileRef*)(ws + pl.off_proj);
        st->d_upd = (TileRef*)(ws + pl.off_upd);
        st->d_dots = (TileRef*)(ws + pl.off_dots);
        st->d_patches = (TileRef*)(ws + pl.off_patches);
        st->d_skinny = (TileRef*)(ws + pl.off_skinny);

        st->mats.resize(n_mats);
        std::vector<TileRef> dots;
        size_t off = pl.off_scratch;
        st->max_m = st->max_n = st->max_r = st->max_l = st->max_lp = st->max_rows = st->max_ldn = 0;
        st->max_jpairs = 0;
        st->sides = 0;
        for (int op = 0; op < OP_COUNT; ++op) st->max_ti[op] = st->max_tj[op] = st->max_tk[op] = 1;
        for (int i = 0; i < n_mats; ++i) {
            const Sizes& z = pl.sz[i];
            MatDev& md = st->mats[i];
            memset(&md, 0, sizeof(md));
            const ng_matrix_desc ed = effective(descs[i]);
            md.m = ed.m; md.n = ed.n; md.r = ed.r; md.ldn = z.ldn;
            md.side = descs[i].side;
            st->sides |= descs[i].side == NG_SIDE_RIGHT ? 2 : 1;
            md.l = z.l; md.ldk = z.ldk; md.ldr = z.ldr; md.roct = z.roct;
            md.ld_w = descs[i].ld_w; md.ld_g = descs[i].ld_g;
            md.slot_elems = (long long)md.r * state_cols(z.ldn, z.pw);
            md.pw = z.pw;
            md.P = (float*)bufs[i].buf[NG_BUF_P];
            md.M = (float*)bufs[i].buf[NG_BUF_M];
            md.V = (float*)bufs[i].buf[NG_BUF_V];
            md.H = (float*)bufs[i].buf[NG_BUF_H];
            char* kb = (char*)bufs[i].buf[NG_BUF_K];
            md.K = (double*)(kb + z.k_gram_off);
            md.w64 = (double*)(kb + z.k_w64_off);
            md.w32 = (float*)(kb + z.k_w32_off);
            md.N = bufs[i].buf[NG_BUF_N];
            if (hp->grad_dtype == NG_BF16) {
                char* ab = (char*)bufs[i].buf[NG_BUF_AUX];
                md.Pb = (bf16_t*)(ab + z.aux_pb_off);
                md.PbT = (bf16_t*)(ab + z.aux_pbt_off);
            }
            md.tail8_off = hp->grad_dtype == NG_BF16 ? (long long)(pl.step_tail8_off + (size_t)16 * i) : -1;
            md.dot_parts_off = (long long)pl.step_parts_off[i];
            md.skinny_parts_off = z.ws_skinny ? (long long)pl.step_skinny_off[i] : -1;
            md.Ya = (float*)(ws + off); off += z.ws_y;
            md.Yb = (float*)(ws + off); off += z.ws_y;
            // low-memory projector: the float P of a refresh is transient and lives in the sketch buffer
            // Yb ([max(m,n)][l] floats, l >= r), which is free from the Rayleigh-Ritz step on
            if (hp->proj_dtype == NG_BF16) md.P = md.Yb;
            md.Yc = (float*)(ws + off); off += z.ws_y;
            md.Bm = (float*)(ws + off); off += z.ws_bm;
            md.T = (double*)(ws + off); off += z.ws_t;
            md.Linv = (float*)(ws + off); off += z.ws_linv;
            md.ritz = (double*)(ws + off); off += z.ws_ritz;
            md.order = (int*)(ws + off); off += z.ws_order;
            md.jflag = (int*)(ws + off); off += z.ws_flag;
            md.carry = z.ws_carry ? (float*)(ws + off) : nullptr; off += z.ws_carry;
            md.lp = z.lp;
            // units of the Gram-row reduction: 16-byte vectors of a slot
            const long long total4 = (long long)md.r * z.ldn / (hist_is_bf16(*hp) ? 8 : 4);   // positions that hold columns below ldn
            long long iters = (total4 + 256LL * kDotPartsMax - 1) / (256LL * kDotPartsMax);
            if (iters < 1) iters = 1;
            // float slots large enough for several passes: a whole number of 1024-vector passes per
            // workgroup (the kernel then walks the slots one at a time)
            if (!hist_is_bf16(*hp) && iters >= 3) iters = (iters + 3) / 4 * 4;
            md.dot_iters = (int)iters;
            md.dot_nparts = (int)((total4 + iters * 256 - 1) / (iters * 256));
            if (hp->s > 0)
                for (int p = 0; p < md.dot_nparts; ++p) dots.push_back(TileRef{i, p, 0, 0});
            if (md.m > st->max_m) st->max_m = md.m;
            if (md.n > st->max_n) st->max_n = md.n;
            if (md.r > st->max_r) st->max_r = md.r;
            if (md.l > st->max_l) st->max_l = md.l;
            if (md.ldn > st->max_ldn) st->max_ldn = md.ldn;
            if (md.lp > st->max_lp) st->max_lp = md.lp;
            const int rows = md.m > md.n ? md.m : md.n;
            if (rows > st->max_rows) st->max_rows = rows;
            const int pairs = md.lp / kJacobiBlock / 2;
            if (pairs > st->max_jpairs) st->max_jpairs = pairs;
            for (int op = 0; op < OP_COUNT; ++op) {
                int M, N, K;
                gemm_f32_dims(op, md, &M, &N, &K);
                if (M > st->max_ti[op]) st->max_ti[op] = M;
                if (N > st->max_tj[op]) st->max_tj[op] = N;
                if (K > st->max_tk[op]) st->max_tk[op] = K;
            }
        }
        st->n_dots = (int)dots.size();

        st->tables_valid = !(flags & NG_INIT_HOST_ONLY);
        if (!st->tables_valid) {
            *out = st;
            return NG_OK;
        }
        // upload the tables (synchronous copies; init is not a hot path)
        hipError_t e = hipSuccess;
        // the status word, and behind it (bytes 64..127) a block of zeros the update GEMM fetches
        // in place of out-of-range operand chunks
        const char zeros[256] = {0};
        e = hipMemcpy(st->d_status, zeros, sizeof(zeros), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(st->d_mats, st->mats.data(), sizeof(MatDev) * n_mats, hipMemcpyHostToDevice);
        if (e == hipSuccess && !pl.proj.empty())
            e = hipMemcpy(st->d_proj, pl.proj.data(), sizeof(TileRef) * pl.proj.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess && !pl.upd.empty())
            e = hipMemcpy(st->d_upd, pl.upd.data(), sizeof(TileRef) * pl.upd.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess && !dots.empty())
            e = hipMemcpy(st->d_dots, dots.data(), sizeof(TileRef) * dots.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess && !pl.patches.empty())
            e = hipMemcpy(st->d_patches, pl.patches.data(), sizeof(TileRef) * pl.patches.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess && !pl.skinny.empty())
            e = hipMemcpy(st->d_skinny, pl.skinny.data(), sizeof(TileRef) * pl.skinny.size(), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            delete st;
            return NG_ERR_HIP;
        }

        if (!(flags & NG_INIT_NO_CLEAR)) {
            for (int i = 0; i < n_mats; ++i) {
                const int ids[5] = {NG_BUF_M, NG_BUF_V, NG_BUF_H, NG_BUF_K, NG_BUF_N};
                for (int b = 0; b < 5; ++b) {
                    if (launch_fill_zero(bufs[i].buf[ids[b]], pl.sz[i].bytes[ids[b]], stream) != hipSuccess) {
                        delete st;
                        return NG_ERR_HIP;
                    }
                }
            }
        }
    } catch (...) {
        delete st;
        return NG_ERR_INVALID_ARG;
    }
    *out = st;
    return NG_OK;
}

int ng_commit_projector(ng_state* st, int clear, ng_stream stream_) {
    if (!st) return NG_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    int rc = finish_projector(st, clear != 0, st->hp.proj_dtype != NG_BF16, stream);
    if (rc != NG_OK) return rc;
    st->projector_valid = true;
    if (clear) {
        for (int i = 0; i < st->n_mats; ++i) {
            st->head[i] = 0;
            st->count[i] = 0;
            st->n_refresh[i] += 1;
        }
    }
    return NG_OK;
}

int ng_refresh_projector(ng_state* st, const void* const* grads, ng_stream stream_) {
    if (!st || !grads) return NG_ERR_INVALID_ARG;
    for (int i = 0; i < st->n_mats; ++i)
        if (!grads[i]) return NG_ERR_INVALID_ARG;
    if (!st->tables_valid) return NG_ERR_HIP;
    hipStream_t stream = (hipStream_t)stream_;
    const StepScalars sc = make_scalars(st, 0.f);
    int rc;
    if ((rc = upload_dyn(st, st->d_dyn, grads, nullptr, false, stream)) != NG_OK) return rc;

    // randomised subspace iteration: Ya = orth(G Omega); q times { Yb = orth(G^T Ya); Ya = orth(G Yb) }
    NG_HIP(launch_fill_gaussian(st->d_mats, st->n_mats, st->max_n, st->hp.seed,
                                (unsigned long long)st->n_refresh[0], stream));
    const int q = st->hp.refresh_power_iters;
    if ((rc = gradient_product(st, OP_G_B2A, q == 0, stream, sc)) != NG_OK) return rc;
    if ((rc = orthonormalise(st, true, q == 0, stream, sc)) != NG_OK) return rc;
    for (int it = 0; it < q; ++it) {
        // intermediate bases live in Yc (single-pass orthonormalisation)
        if ((rc = gradient_product(st, OP_GT_C2B, false, stream, sc)) != NG_OK) return rc;
        if ((rc = orthonormalise(st, false, false, stream, sc)) != NG_OK) return rc;
        if ((rc = gradient_product(st, OP_G_C2A, it + 1 == q, stream, sc)) != NG_OK) return rc;
        if ((rc = orthonormalise(st, true, it + 1 == q, stream, sc)) != NG_OK) return rc;
    }
    // Rayleigh-Ritz: B = Q^T G, T = B B^T = U diag(ritz^2) U^T, P = Q U[:, top r]
    if ((rc = gradient_product(st, OP_QT_G, true, stream, sc)) != NG_OK) return rc;
    if ((rc = gemm(st, OP_B_BT, stream, sc)) != NG_OK) return rc;
    NG_HIP(launch_jacobi_prepare(st->d_mats, st->n_mats, stream));
    for (int sw = 0; sw < st->hp.refresh_sweeps; ++sw) {
        const int max_rounds = 2 * st->max_jpairs - 1;
        for (int round = 0; round < (max_rounds > 0 ? max_rounds : 1); ++round)
            NG_HIP(launch_jacobi_round(st->d_mats, st->n_mats, st->max_jpairs, round, stream));
        NG_HIP(launch_jacobi_sweep_end(st->d_mats, st->n_mats, stream));
    }
    NG_HIP(launch_jacobi_finish(st->d_mats, st->n_mats, st->d_status, stream));
    // history carry-over needs the outgoing projector: keep it in Yc (free from here on)
    const bool carry = st->hp.carry_history && st->hp.s > 0 && st->projector_valid;
    if (carry) NG_HIP(launch_save_projector(st->d_mats, st->n_mats, stream));
    if ((rc = gemm(st, OP_ROTATE, stream, sc)) != NG_OK) return rc;
    // one CholeskyQR pass on P (m x r) restores orthonormality to rounding level, then fix signs
    if ((rc = gemm(st, OP_GRAM_P, stream, sc)) != NG_OK) return rc;
    NG_HIP(launch_cholesky(st->d_mats, st->n_mats, 1, st->max_r, 0.0, st->d_status, stream));
    NG_HIP(launch_tri_inverse(st->d_mats, st->n_mats, 1, st->max_r, stream));
    if ((rc = gemm(st, OP_APPLY_P2A, stream, sc)) != NG_OK) return rc;
    NG_HIP(launch_sign_fix(st->d_mats, st->n_mats, st->max_r, stream));

    if (carry) {
        // H_j <- (P_new^T P_old) H_j for every slot, then the whole Gram matrix again
        if ((rc = gemm(st, OP_T_CARRY, stream, sc)) != NG_OK) return rc;
        StepScalars scs = sc;
        for (int slot = 0; slot < st->hp.s; ++slot) {
            scs.slot = slot;
            if ((rc = gemm(st, OP_CARRY_SLOT, stream, scs)) != NG_OK) return rc;
            NG_HIP(launch_carry_store(st->d_mats, st->n_mats, slot, sc.hist_bf16, stream));
        }
        for (int row = 0; row < st->hp.s; ++row) {
            NG_HIP(launch_gram_row(st->d_mats, st->d_dyn, st->d_dots, st->n_dots, sc.s, sc.hist_bf16, row, stream));
            NG_HIP(launch_solve(st->d_mats, st->d_dyn, 0, st->n_mats, sc, row, st->d_status, stream));
        }
    }
    if ((rc = finish_projector(st, !carry, true, stream)) != NG_OK) return rc;
    st->projector_valid = true;
    for (int i = 0; i < st->n_mats; ++i) {
        if (!carry) {
            st->head[i] = 0;
            st->count[i] = 0;
        }
        st->n_refresh[i] += 1;
    }
    return NG_OK;
}

int ng_step(ng_state* st, const void* const* grads, void* const* weights, float lr, ng_stream stream_) {
    if (!st) return NG_ERR_INVALID_ARG;
    return step_on_scratch(st, grads, weights, lr, (hipStream_t)stream_, st->d_dyn);
}

int ng_step_static(ng_state* st, const void* const* grads, void* const* weights, float lr, ng_stream stream_) {
    if (!st) return NG_ERR_INVALID_ARG;
    if (st->plan.step_bytes > kStaticScratchBytes) return NG_ERR_WORKSPACE;
    if (!st->tables_valid) return NG_ERR_HIP;
    char* scratch = nullptr;
    int rc = static_scratch_of_current_device(&scratch);
    if (rc != NG_OK) return rc;
    return step_on_scratch(st, grads, weights, lr, (hipStream_t)stream_, (MatDyn*)scratch);
}

int ng_get_counters(const ng_state* st, int mat, int64_t* t, int32_t* head, int32_t* count, int64_t* n_refresh) {
    if (!st || mat < 0 || mat >= st->n_mats) return NG_ERR_INVALID_ARG;
    if (t) *t = st->t[mat];
    if (head) *head = st->head[mat];
    if (count) *count = st->count[mat];
    if (n_refresh) *n_refresh = st->n_refresh[mat];
    return NG_OK;
}

int ng_set_counters(ng_state* st, int mat, int64_t t, int32_t head, int32_t count, int64_t n_refresh) {
    if (!st || mat < 0 || mat >= st->n_mats) return NG_ERR_INVALID_ARG;
    const int s = st->hp.s;
    if (t < 0 || n_refresh < 0) return NG_ERR_INVALID_ARG;
    if (head < 0 || head >= (s > 0 ? s : 1)) return NG_ERR_INVALID_ARG;
    if (count < 0 || count > s) return NG_ERR_INVALID_ARG;
    st->t[mat] = t;
    st->head[mat] = head;
    st->count[mat] = count;
    st->n_refresh[mat] = n_refresh;
    return NG_OK;
}

int ng_get_layout(const ng_state* st, int mat, ng_matrix_layout* out) {
    if (!st || !out || mat < 0 || mat >= st->n_mats) return NG_ERR_INVALID_ARG;
    const Sizes& z = st->plan.sz[mat];
    out->ldn = z.ldn;
    out->l = z.l;
    out->slot_elems = (int64_t)st->descs[mat].r * state_cols(z.ldn, z.pw);
    out->panel_cols = z.pw;
    out->reserved0 = 0;
    out->k_gram_off = (int64_t)z.k_gram_off;
    out->k_w64_off = (int64_t)z.k_w64_off;
    out->k_w32_off = (int64_t)z.k_w32_off;
    out->aux_pb_off = (int64_t)z.aux_pb_off;
    out->aux_pbt_off = (int64_t)z.aux_pbt_off;
    return NG_OK;
}

int ng_get_status(ng_state* st, ng_stream stream_) {
    if (!st) return NG_ERR_INVALID_ARG;
    if (!st->tables_valid) return NG_ERR_HIP;
    hipStream_t stream = (hipStream_t)stream_;
    NG_HIP(hipStreamSynchronize(stream));
    int flag = 0;
    NG_HIP(hipMemcpy(&flag, st->d_status, sizeof(int), hipMemcpyDeviceToHost));
    if (flag != 0) {
        int zero = 0;
        NG_HIP(hipMemcpy(st->d_status, &zero, sizeof(int), hipMemcpyHostToDevice));
        return (flag & ~kStatusNotConverged) ? NG_ERR_NUMERIC : NG_ERR_NOT_CONVERGED;
    }
    return NG_OK;
}

int ng_set_profiling(ng_state* st, int enabled) {
    if (!st) return NG_ERR_INVALID_ARG;
    if (enabled && !st->ev_created) {
        for (int i = 0; i < kProfRing; ++i)
            for (int p = 0; p <= NG_NPHASE; ++p)
                if (hipEventCreate(&st->ev[i][p]) != hipSuccess) return NG_ERR_HIP;
        st->ev_created = true;
    }
    if (!enabled) drain_events(st, true);
    st->profiling = enabled != 0;
    return NG_OK;
}

int ng_get_phase_ms(ng_state* st, double* ms, int64_t* steps, int reset) {
    if (!st || !ms || !steps) return NG_ERR_INVALID_ARG;
    drain_events(st, true);
    for (int p = 0; p < NG_NPHASE; ++p) ms[p] = st->phase_ms[p];
    *steps = st->phase_steps;
    if (reset) {
        memset(st->phase_ms, 0, sizeof(st->phase_ms));
        st->phase_steps = 0;
    }
    return NG_OK;
}

int ng_microbench(int which, const void* a, void* b, size_t bytes, int reps, ng_stream stream_, double* ms,
                  double* work) {
    if (!b || !ms || !work || reps < 1 || reps > 10000) return NG_ERR_INVALID_ARG;
    if (which < NG_MB_COPY || which > NG_MB_MFMA_BF16_RANDOM) return NG_ERR_INVALID_ARG;
    const bool mfma = which == NG_MB_MFMA_BF16 || which == NG_MB_MFMA_BF16_RANDOM;
    if (!mfma && (!a || bytes == 0 || bytes % 16 != 0 || ((uintptr_t)a & 15))) return NG_ERR_INVALID_ARG;
    if (which == NG_MB_COPY && ((uintptr_t)b & 15)) return NG_ERR_INVALID_ARG;
    if (mfma && (bytes == 0 || bytes > (1u << 24))) return NG_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    NG_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return NG_ERR_HIP;
    }
    double w = 0.0;
    hipError_t e = hipSuccess;
    for (int k = -1; k < reps && e == hipSuccess; ++k) {
        if (k == 0) e = hipEventRecord(e0, stream);
        if (e != hipSuccess) break;
        if (which == NG_MB_COPY) {
            e = launch_mb_copy(a, b, bytes, stream);
            w = 2.0 * (double)bytes;
        } else if (which == NG_MB_READ) {
            e = launch_mb_read(a, bytes, b, stream);
            w = (double)bytes;
        } else {
            e = launch_mb_mfma((int)bytes, 2, which == NG_MB_MFMA_BF16_RANDOM, b, &w, stream);
        }
    }
    float t = 0.f;
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return NG_ERR_HIP;
    *ms = (double)t / reps;
    *work = w;
    return NG_OK;
}

const char* ng_strerror(int code) {
    switch (code) {
        case NG_OK: return "ok";
        case NG_ERR_INVALID_ARG: return "invalid argument";
        case NG_ERR_SHAPE: return "invalid shape (m, n, r, ld or s)";
        case NG_ERR_DTYPE: return "unknown dtype or mode";
        case NG_ERR_HPARAM: return "hyper-parameter out of range";
        case NG_ERR_NO_PROJECTOR: return "no projector: call ng_refresh_projector or ng_commit_projector first";
        case NG_ERR_HIP: return "HIP runtime error";
        case NG_ERR_NUMERIC: return "numeric failure on device (non-positive pivot or non-finite value)";
        case NG_ERR_WORKSPACE:
            return "workspace too small or misaligned (ng_step_static: the step's scratch exceeds the library's array)";
        case NG_ERR_NOT_CONVERGED: return "the refresh's eigen-solve used all its sweeps without converging";
        default: return "unknown error code";
    }
}

size_t ng_struct_size(int which) {
    switch (which) {
        case 0: return sizeof(ng_matrix_desc);
        case 1: return sizeof(ng_hparams);
        case 2: return sizeof(ng_matrix_buffers);
        case 3: return sizeof(ng_matrix_layout);
        default: return 0;
    }
}

void ng_destroy(ng_state* st) {
    if (!st) return;
    if (st->ev_created) {
        for (int i = 0; i < kProfRing; ++i)
            for (int p = 0; p <= NG_NPHASE; ++p) (void)hipEventDestroy(st->ev[i][p]);
    }
    delete st;
}

}  // extern "C"
