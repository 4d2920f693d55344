/*
 * ng.h -- C ABI of the Natural GaLore optimizer step for AMD MI355X (gfx950).
 *
 * One handle (ng_state) drives a whole "layer set": n_mats independent weight
 * matrices that are stepped together.  For each matrix W (m x n) with gradient
 * G (m x n) the library keeps
 *     P  m x r   projector with orthonormal columns          (paper Sec. 1, compact SVD)
 *     M,V r x n  Adam moments of the transformed gradient     (paper Sec. 2.2, Adam equations)
 *     H  s x r x n  ring buffer of the last s low-rank gradients  (paper Sec. 2.4, stacked matrix)
 *     K  s x s   Gram matrix of the ring's slots               (paper Sec. 2.4, the s x s system)
 * The paper writes matrices as n x m; here m counts rows and n columns.
 *
 * Conventions
 *   - Every pointer in ng_matrix_buffers, `workspace`, `grads[i]` and
 *     `weights[i]` is a DEVICE pointer; every other pointer (descriptors,
 *     hyper-parameters, the arrays `grads`/`weights` themselves, out-params) is a
 *     HOST pointer.
 *   - All matrices are row-major.  ld_* are in elements.
 *   - All device memory is owned by the caller and must outlive the handle.  The
 *     library allocates no device memory and frees none.  `workspace` is ordinary
 *     (coarse-grained) device memory as hipMalloc returns it: the refresh adds into it
 *     with hardware floating-point atomics.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls
 *     that take a stream only enqueue work on it and do not synchronise, except
 *     where stated.  Calls on one handle must not overlap.
 *   - Every function returns an int: NG_OK (0) or a negative NG_ERR_* code.  No
 *     C++ exception crosses this boundary.  A call that fails leaves the
 *     handle's integer counters unchanged.
 */
#ifndef NG_H_
#define NG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ng_state ng_state;   /* opaque, host-side; created by ng_init_state */
typedef void* ng_stream;            /* a hipStream_t */

/* storage type of gradients AND weights */
enum { NG_F32 = 0, NG_BF16 = 1 };

/* NG_ADAM_STANDARD: bias-corrected moments, eps outside the root (Adam as
 * published; "sent to the Adam optimizer", end of paper Sec. 2.4).
 * NG_ADAM_PRINTED: the three equations exactly as printed in paper Sec. 2.2:
 * no bias correction, u = m / sqrt(v + eps). */
enum { NG_ADAM_STANDARD = 0, NG_ADAM_PRINTED = 1 };

enum {
    NG_OK = 0,
    NG_ERR_INVALID_ARG = -1,   /* null pointer, bad index, bad count                  */
    NG_ERR_SHAPE = -2,         /* m,n,r <= 0, r > min(m,n), ld < n, s out of range,
                                  r + refresh_oversample > 2048, m or n > 2^24, a weight
                                  or gradient of 2 GiB or more (m * ld * 4 bytes)       */
    NG_ERR_DTYPE = -3,         /* unknown grad_dtype / adam_mode                      */
    NG_ERR_HPARAM = -4,        /* lambda <= 0, beta outside [0,1), eps <= 0, ...      */
    NG_ERR_NO_PROJECTOR = -5,  /* ng_step before any refresh / commit                 */
    NG_ERR_HIP = -6,           /* a HIP runtime call or kernel launch failed          */
    NG_ERR_NUMERIC = -7,       /* device flag: non-positive pivot or non-finite value */
    NG_ERR_WORKSPACE = -8,     /* workspace too small or misaligned                   */
    NG_ERR_NOT_CONVERGED = -9  /* device flag: the refresh's eigen-solve used all its
                                  refresh_sweeps without reaching its convergence test  */
};

/* per-matrix caller-owned device buffers, sizes from ng_query_sizes */
enum {
    NG_BUF_P = 0,   /* float  [m][r]                      projector (0 bytes with proj_dtype = NG_BF16) */
    NG_BUF_M,       /* float  [r][ldn]                    first moment                                */
    NG_BUF_V,       /* float  [r][ldn]                    second moment                               */
    NG_BUF_H,       /* float or bf16 (hist_dtype) [max(s,1)][r][ldn]  history ring (one scratch slot when s = 0) */
                    /* (M, V and the slots of H: stored in column panels where
                       ng_matrix_layout::panel_cols < ldn, see there)                                 */
    NG_BUF_K,       /* double [s*s] Gram, double [s] w, then float [s] w  (see ng_matrix_layout)      */
    NG_BUF_N,       /* update direction: float [r][ldn] (NG_F32) or bf16 [ceil(r/8)][ldn][8] (NG_BF16) */
    NG_BUF_AUX,     /* NG_BF16 only: bf16 copies of P; 0 bytes for NG_F32 (pointer may be NULL)       */
    NG_NBUF
};

/* Which factor of the gradient's compact SVD g = P Sigma Q^T (paper Sec. 1) projects.
 * NG_SIDE_LEFT:  R = P^T G (r x n), P is m x r, update W - lr (scale P N + wd W): the form the
 *                paper writes out.
 * NG_SIDE_RIGHT: R = G Q (m x r), Q is n x r, update W - lr (scale N Q^T + wd W): the same method
 *                applied to G^T (the usual choice for m > n: the projector is n x r).  Internally
 *                the state is that of the transposed problem: every "m" in the buffer shapes below
 *                reads n and every "n" reads m (P is [n][r]; M, V, H, N are r x ldm). */
enum { NG_SIDE_LEFT = 0, NG_SIDE_RIGHT = 1 };
enum { NG_NORM_S = 0, NG_NORM_COUNT = 1 };

typedef struct ng_matrix_desc {
    int32_t m, n, r;       /* weight is m x n (row-major), rank r, 1 <= r <= min(m, n) */
    int32_t side;          /* NG_SIDE_LEFT | NG_SIDE_RIGHT                            */
    int64_t ld_w, ld_g;    /* leading dimensions of weight and gradient, >= n         */
} ng_matrix_desc;

typedef struct ng_hparams {
    int32_t s;               /* history length, 0 <= s <= 64; 0 = no Fisher transform (GaLore-Adam) */
    float lambda;            /* Tikhonov damping of the empirical Fisher, > 0 (paper Sec. 2.4)     */
    float beta1, beta2, eps; /* Adam (paper Sec. 2.2)                                              */
    float scale;             /* multiplies P N in the update                                       */
    float weight_decay;      /* decoupled weight decay, multiplies W in the update                 */
    int32_t grad_dtype;      /* NG_F32 | NG_BF16                                                   */
    int32_t adam_mode;       /* NG_ADAM_STANDARD | NG_ADAM_PRINTED                                 */
    int32_t refresh_power_iters;  /* subspace-iteration passes q >= 0 of the refresh               */
    int32_t refresh_oversample;   /* extra sketch columns p >= 0; sketch width l = min(r+p, m, n), trimmed
                                   * to the next lower multiple of 32 when that is still >= r       */
    int32_t refresh_sweeps;       /* maximum Jacobi sweeps of the l x l eigen-solve, >= 1          */
    int32_t hist_dtype;           /* storage type of the history slots: NG_F32 (default) or NG_BF16
                                     (NG_BF16 gradients only).  bf16 slots halve the ring's memory and
                                     the two passes over it that bound the step; M and V are float in
                                     every mode                                                      */
    int32_t fisher_norm;          /* NG_NORM_S (default): F = lambda I + (1/s) sum_j vec(H_j) vec(H_j)^T
                                     always; NG_NORM_COUNT: 1/(number of valid slots) while the ring
                                     fills (the two readings of the paper's 1/h, Sec. 2.2 / 2.4)     */
    int32_t carry_history;        /* 0 (default): ng_refresh_projector clears the history (its slots are
                                     coordinates in the old basis).  1: it re-expresses every slot in
                                     the new basis, H_j <- (P_new^T P_old) H_j, recomputes the Gram
                                     matrix and keeps the ring position                              */
    int32_t proj_dtype;           /* NG_F32 (default): the projector is kept as float [m][r] in NG_BUF_P (plus,
                                     for NG_BF16 gradients, the two bf16 copies in NG_BUF_AUX that the GEMMs
                                     multiply with).  NG_BF16 (NG_BF16 gradients only, not with carry_history):
                                     the low-memory projector -- only the two bf16 copies are kept, NG_BUF_P
                                     has 0 bytes (its pointer may be NULL); a refresh builds the float
                                     projector in the workspace, rounds it into the copies and drops it.
                                     There is then no float P for the caller to read or to commit: a
                                     checkpoint holds NG_BUF_AUX, and ng_commit_projector only marks
                                     restored copies valid                                              */
    uint64_t seed;                /* seed of the refresh's random sketch                            */
} ng_hparams;

typedef struct ng_matrix_buffers {
    void* buf[NG_NBUF];
} ng_matrix_buffers;

typedef struct ng_matrix_layout {
    int32_t ldn;        /* padded row length (elements) of M, V, N and of every H slot; columns >= n are 0 */
    int32_t l;          /* sketch width of the refresh                                                   */
    int64_t slot_elems; /* elements from one history slot to the next (r * ldn unless panelled, see below)    */
    /* M, V and every H slot are stored as column panels of panel_cols columns: element (row, col) lies at
     *   p * r * panel_cols + row * panel_cols + (col - p * panel_cols),  p = col / panel_cols
     * i.e. panel p is a row-major r x panel_cols block and the panels follow each other.  panel_cols ==
     * ldn (one panel) is the plain row-major [r][ldn] array: always so for NG_F32 gradients, with
     * carry_history, and where ldn < 2304.  Otherwise panel_cols = 2048 (the row pitch at which the
     * streaming kernels run fastest); the arrays then hold r * ceil(ldn / 2048) * 2048 elements (the sizes
     * ng_query_sizes reports, and slot_elems above, count them) and the last panel's columns from ldn on
     * are padding that stays 0.  N is not panelled. */
    int32_t panel_cols;
    int32_t reserved0;
    int64_t k_gram_off, k_w64_off, k_w32_off;  /* byte offsets inside the K buffer                       */
    /* NG_BF16 only (else 0): byte offsets inside the AUX buffer of the two bf16 copies of P that the
     * step's GEMMs multiply with, both split into blocks of 32 along the contraction index:
     *   Pb  [ceil(r/32)][m][32]: P[i][rho]   at element ((rho/32) * m + i) * 32 + rho % 32   (update)
     *   PbT [ceil(m/32)][r][32]: P[i][rho]   at element ((i/32) * r + rho) * 32 + i % 32     (projection)
     * positions beyond r (Pb) or m (PbT) inside the last block are 0 */
    int64_t aux_pb_off, aux_pbt_off;
} ng_matrix_layout;

/* Fill hp with the defaults: s=4, lambda=1e-3, betas (0.9, 0.999), eps 1e-8,
 * scale 1, weight_decay 0, NG_F32, NG_ADAM_STANDARD, q=2, p=8, 30 sweeps,
 * hist_dtype NG_F32, fisher_norm NG_NORM_S, carry_history 0, proj_dtype NG_F32, seed 0. */
int ng_default_hparams(ng_hparams* hp);

/* Bytes the caller must allocate.  bytes[i*NG_NBUF + b] = size of buffer b of
 * matrix i (256-byte aligned device memory); *workspace_bytes = size of the one
 * shared workspace (tables, reduction partials, the refresh's scratch).
 * Host-only; touches no device. */
int ng_query_sizes(const ng_matrix_desc* descs, int n_mats, const ng_hparams* hp,
                   size_t* bytes, size_t* workspace_bytes);

/* flags for ng_init_state */
enum { NG_INIT_DEFAULT = 0,
       NG_INIT_NO_CLEAR = 1,  /* caller has already zero-filled (or restored) every buffer */
       NG_INIT_HOST_ONLY = 2  /* touch no device: nothing is uploaded or cleared, and every later call
                                 that would launch a kernel returns NG_ERR_HIP.  For exercising the
                                 host-side bookkeeping (validation, counters, layout) without a GPU;
                                 the buffer and workspace pointers are only checked for alignment */ };

/* Create a handle over caller-owned buffers.  Unless NG_INIT_NO_CLEAR is given,
 * enqueues zero-fills of M, V, H, K, N on `stream`.  Uploads its tables into
 * `workspace` (synchronous copies); a failed upload returns NG_ERR_HIP and no
 * handle.  Counters start at t = head = count = n_refresh = 0 and the projector
 * is marked invalid. */
int ng_init_state(const ng_matrix_desc* descs, const ng_matrix_buffers* bufs, int n_mats,
                  const ng_hparams* hp, void* workspace, size_t workspace_bytes,
                  uint32_t flags, ng_stream stream, ng_state** out);

/* Periodic subspace refresh (paper Sec. 1: P from the compact SVD of the
 * gradient, updated every ~200 iterations; Sec. 2.2).  For every matrix:
 * P <- approximation of the top-r left singular vectors of grads[i] by
 * randomised subspace iteration + Rayleigh-Ritz, columns ordered by descending
 * Ritz value, each column's largest-magnitude entry positive.  Keeps M, V and t;
 * clears H and K; head = count = 0; n_refresh += 1.  grads[i]: m x n, ld_g,
 * grad_dtype; read-only. */
int ng_refresh_projector(ng_state* st, const void* const* grads, ng_stream stream);

/* The caller has written P (float [m][r], orthonormal columns) into every
 * NG_BUF_P itself (resume from a checkpoint, an external SVD).  Builds the
 * internal copies, marks the projector valid.  clear_history != 0 also clears H,
 * K and sets head = count = 0 and n_refresh += 1 (as a refresh does).
 * With proj_dtype = NG_BF16 there is no NG_BUF_P: the caller has restored
 * NG_BUF_AUX (the two bf16 copies) and this call only marks them valid. */
int ng_commit_projector(ng_state* st, int clear_history, ng_stream stream);

/* One optimizer step on every matrix (paper Sec. 2.4 with Sec. 2.2):
 *   R = P^T G                           -> written into ring slot `head`
 *   K[head][:] = <R, H_j>_F             -> (lambda I + K/s) w = e_head   (fp64, Cholesky)
 *   g~ = sum_j w_j H_j                  == (lambda I + (1/s) sum_j vec(H_j)vec(H_j)^T)^{-1} vec(R)
 *   M, V <- Adam moments of g~ ;  N = update direction
 *   W <- W - lr * (scale * P N + weight_decay * W)
 * then t += 1, head = (head+1) mod s, count = min(count+1, s) on the host.
 * grads[i] read-only, weights[i] (m x n, ld_w, grad_dtype) updated in place. */
int ng_step(ng_state* st, const void* const* grads, void* const* weights, float lr,
            ng_stream stream);

/* ng_step for callers that must not allocate and have no workspace to spare for it: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and same results as ng_step, but the scratch the step's kernels hand to each other (the
 * per-step table, the partial sums of the Gram-row reduction, the row-chunk sums of the small-rank
 * projection, the padded gradient tails) lies in a device array of the library itself instead of
 * the caller's workspace.  That array has NG_STATIC_SCRATCH_BYTES bytes per GPU, is held by every
 * GPU the library has run on until the process ends, and is shared by every handle and every call
 * on that GPU: calls of ng_step_static that overlap on one GPU (two streams, two threads) race;
 * calls ordered on one stream, also from different handles, are fine (each call rewrites all it
 * reads; nothing in the array has to start at zero).  A layer set whose step scratch exceeds the
 * array returns NG_ERR_WORKSPACE (the per-matrix share is 2 KiB * s for the reduction plus, for
 * fp32 sets of rank <= 16, ceil(m/128) * rank class * ldn * 4 bytes); nothing is launched then.
 * Calls no hipMalloc / hipFree.  The first call on a GPU looks the array's address up
 * (hipGetSymbolAddress, once per device and process): make that call outside a graph capture.
 * A captured call holds this step's ring position, bias corrections, learning rate and the
 * gradient / weight pointers as launch arguments: replaying the graph repeats that step (the host
 * counters advance at capture, not at replay), so capture each step anew or use the graph for one.
 * The handle still comes from ng_init_state (its workspace keeps the static tables and the
 * refresh's scratch). */
#define NG_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int ng_step_static(ng_state* st, const void* const* grads, void* const* weights, float lr,
                   ng_stream stream);

int ng_get_counters(const ng_state* st, int mat, int64_t* t, int32_t* head, int32_t* count,
                    int64_t* n_refresh);
/* Resume: requires 0 <= head < max(s,1), 0 <= count <= s, t >= 0. */
int ng_set_counters(ng_state* st, int mat, int64_t t, int32_t head, int32_t count,
                    int64_t n_refresh);

int ng_get_layout(const ng_state* st, int mat, ng_matrix_layout* out);

/* Synchronises `stream`, reads and clears the device's sticky flag.  Returns
 * NG_OK, NG_ERR_NUMERIC (non-positive pivot, non-finite value; takes precedence),
 * NG_ERR_NOT_CONVERGED (a refresh whose eigen-solve ran out of sweeps; P is still
 * orthonormal, its columns may mix neighbouring Ritz vectors) or NG_ERR_HIP. */
int ng_get_status(ng_state* st, ng_stream stream);

/* Phase timing with HIP events on the stream of the call.  When enabled, ng_step
 * records an event before each phase (project, gram, solve, adam, update) and
 * one after the last.  ng_get_phase_ms synchronises on the last event and adds
 * the elapsed milliseconds of every profiled step since the last reset into
 * ms[0..4]; *steps = number of steps accumulated.  reset != 0 clears the sums. */
enum { NG_PHASE_PROJECT = 0, NG_PHASE_GRAM, NG_PHASE_SOLVE, NG_PHASE_ADAM, NG_PHASE_UPDATE,
       NG_NPHASE };
int ng_set_profiling(ng_state* st, int enabled);
int ng_get_phase_ms(ng_state* st, double* ms, int64_t* steps, int reset);

/* Measured ceilings of the GPU the library runs on, to read the step's roofline fractions against:
 * NG_MB_COPY      plain streaming copy a -> b of `bytes` bytes (device pointers, 16-byte aligned,
 *                 bytes % 16 == 0); *work = 2 * bytes (read + written);
 * NG_MB_READ      streaming read of a; b: >= 4 bytes of device memory (never written in practice);
 *                 *work = bytes;
 * NG_MB_MFMA_BF16 a bare loop of v_mfma_f32_32x32x16_bf16 on register operands, two wavefronts per
 *                 SIMD on all 256 units; a ignored, b as for NG_MB_READ, `bytes` = loop trips per
 *                 wavefront (8 MFMAs each); *work = floating-point operations.  The operands are small
 *                 integers that never change: the nominal rate at the full clock;
 * NG_MB_MFMA_BF16_RANDOM the same loop on pseudo-random operands that change from one MFMA to the next:
 *                 the switching activity of real data, under which the chip lowers its clock.
 * One untimed launch, then `reps` launches timed with HIP events on `stream` (synchronises).
 * *ms = mean milliseconds per launch, *work = bytes or flops per launch.  No handle needed;
 * allocates nothing. */
enum { NG_MB_COPY = 0, NG_MB_READ = 1, NG_MB_MFMA_BF16 = 2, NG_MB_MFMA_BF16_RANDOM = 3 };
int ng_microbench(int which, const void* a, void* b, size_t bytes, int reps, ng_stream stream,
                  double* ms, double* work);

const char* ng_strerror(int code);

/* sizeof of a structure of this header as the library was compiled: which = 0 ng_matrix_desc,
 * 1 ng_hparams, 2 ng_matrix_buffers, 3 ng_matrix_layout; 0 for any other value.  Lets a binding
 * written in another language check its own declarations.  Host only. */
size_t ng_struct_size(int which);

void ng_destroy(ng_state* st);

#ifdef __cplusplus
}
#endif
#endif /* NG_H_ */
