"""GPU parity on the degenerate and extreme cases of the step: strided operands, full rank,
ranks and widths that are not multiples of the tile or vector sizes, the largest history, and
the full 1.1B layer set in the launch configuration the benchmark times (sampled matrices)."""
import numpy as np
import pytest
import torch

from paper_2410_16029_amd import binding as B
from paper_2410_16029_amd import workloads
from parity_harness import Lockstep, summarize, worst
from test_gpu_parity import DEV, TOL_BF16, TOL_F32, _assert_all

pytestmark = pytest.mark.gpu


def _run(shapes, r, s, dtype, steps, seed, k=8, check=None, lr=1e-3, pad_w=0, pad_g=0, gscale=1.0,
         energy_tol=2e-3, orth_tol=5e-6, **kw):
    """Free-running lockstep; with pad_w / pad_g the weights / gradients are column slices of
    wider tensors (leading dimension larger than n) whose remaining columns must stay untouched."""
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    stream = workloads.TorchGradientStream(shapes, k, 0.01, seed, dtype, DEV)
    W0 = workloads.torch_weights(shapes, seed, dtype, DEV)
    ld_w = ld_g = None
    Wfull = None
    if pad_w:
        Wfull = [torch.full((m, n + pad_w), 7.0, dtype=w.dtype, device=DEV) for (m, n), w in zip(shapes, W0)]
        for wf, w, (m, n) in zip(Wfull, W0, shapes):
            wf[:, :n] = w
        W = [wf[:, :n] for wf, (m, n) in zip(Wfull, shapes)]
        ld_w = [n + pad_w for (m, n) in shapes]
    else:
        W = W0
    if pad_g:
        ld_g = [n + pad_g for (m, n) in shapes]
    ls = B.LayerSet(shapes, r, s=s, dtype=dtype, device=DEV, ld_w=ld_w, ld_g=ld_g, **kw)
    lk = Lockstep(ls, check=check, tol=tol, k_signal=k, energy_tol=energy_tol, orth_tol=orth_tol)
    lk.set_weights(W)
    errs = []
    for step in range(steps):
        G = stream.next_set()
        if gscale != 1.0:
            G = [(g.float() * gscale).to(g.dtype) for g in G]
        if pad_g:
            Gfull = [torch.full((m, n + pad_g), float("nan"), dtype=g.dtype, device=DEV)
                     for (m, n), g in zip(shapes, G)]
            for gf, g, (m, n) in zip(Gfull, G, shapes):
                gf[:, :n] = g
            G = [gf[:, :n] for gf, (m, n) in zip(Gfull, shapes)]
        if step == 0:
            lk.refresh(G)
            assert ls.status() == B.NG_OK
        errs.append(lk.step(G, W, lr))
    assert ls.status() == B.NG_OK
    if lk.refresh_stats:
        print("refresh", {k_: float("%.3g" % max(st[k_] for st in lk.refresh_stats if k_ in st))
                          for k_ in ("orth", "energy_deficit", "angle") if any(k_ in st for st in lk.refresh_stats)})
    if Wfull is not None:
        for wf, (m, n) in zip(Wfull, shapes):
            assert bool((wf[:, n:] == 7.0).all()), "columns beyond n of a strided weight were written"
    return ls, errs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_strided_weights_and_gradients(dtype):
    # leading dimensions larger than n; the gradient's extra columns hold NaN and must not be read
    shapes = [(130, 75), (64, 200), (300, 257)]
    ls, errs = _run(shapes, 16, 3, dtype, 5, seed=41, pad_w=5, pad_g=3)
    _assert_all(errs, TOL_F32 if dtype == "f32" else TOL_BF16, "strided " + dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_full_rank_projector(dtype):
    # r = min(m, n): the projector is a full orthogonal basis of the shorter side.  The synthetic
    # gradient has full rank too, so that no row of R is pure noise (the direction N of such rows
    # is a sign, which no tolerance covers).
    shapes = [(48, 80), (72, 40)]
    descs_r = [48, 40]
    ls, errs = _run(shapes, descs_r, 2, dtype, 4, seed=43, k=48)
    _assert_all(errs, TOL_F32 if dtype == "f32" else TOL_BF16, "full rank " + dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_odd_ranks_and_narrow_matrices(dtype):
    # ranks that are not multiples of 8, fewer columns than one vector, a single row block
    # (gradient rank above every r: no pure-noise rows in R, see test_full_rank_projector)
    shapes = [(40, 5), (33, 7), (200, 9), (9, 120), (257, 31)]
    ranks = [3, 5, 7, 4, 20]
    ls, errs = _run(shapes, ranks, 3, dtype, 5, seed=47, k=24)
    _assert_all(errs, TOL_F32 if dtype == "f32" else TOL_BF16, "odd ranks " + dtype)


def test_rank_one():
    ls, errs = _run([(64, 96), (17, 33)], 1, 4, "f32", 6, seed=53, k=2)
    _assert_all(errs, TOL_F32, "rank one")


def test_largest_history_wraps_around():
    # s = 64 is the largest history the library accepts; 67 steps wrap the ring
    ls, errs = _run([(64, 96)], 8, 64, "f32", 67, seed=59, k=8)
    _assert_all(errs, TOL_F32, "s=64")
    assert ls.counters(0) == (67, 3, 64, 1)


def test_mixed_ranks_in_one_layer_set_bf16():
    # per-matrix ranks across the 128 threshold that selects the projection tile shape
    shapes = [(384, 520), (256, 300), (520, 384)]
    ranks = [160, 24, 128]
    ls, errs = _run(shapes, ranks, 4, "bf16", 6, seed=61, k=16)
    _assert_all(errs, TOL_BF16, "mixed ranks")


def test_bf16_history_slots_ragged_shapes():
    # opt-in bf16 storage of the history ring: same tolerances; ring wrap-around (steps > s)
    shapes = [(384, 520), (200, 333), (520, 384), (128, 128)]
    ls, errs = _run(shapes, 64, 4, "bf16", 7, seed=23, k=16, hist_dtype="bf16")
    assert ls.H(0).dtype == torch.bfloat16
    _assert_all(errs, TOL_BF16, "bf16 history, ragged")


def test_bf16_history_slots_1b_shapes_and_no_fisher():
    cfg = workloads.CONFIGS["c5"]
    shapes = cfg.matrices()[:7]
    ls, errs = _run(shapes, cfg.r, cfg.s, "bf16", 3, seed=cfg.seed, k=cfg.k, check=[0, 4, 6], hist_dtype="bf16")
    _assert_all(errs, TOL_BF16, "bf16 history, c5 block")
    # s = 0: the single scratch slot is bf16 too
    ls, errs = _run([(200, 333), (130, 64)], 24, 0, "bf16", 3, seed=29, k=24, hist_dtype="bf16")
    _assert_all(errs, TOL_BF16, "bf16 history, s=0")


def test_f32_mid_size_layer_set_many_tiles():
    # fp32 gradients at sizes where the fp32 MFMA GEMMs run many tiles per matrix and the Gram-row
    # reduction many workgroups (the small fp32 configuration is a single 256 x 512 matrix)
    shapes = [(1024, 1536), (1536, 1024), (777, 1290)]
    ls, errs = _run(shapes, 128, 8, "f32", 10, seed=111, k=32)
    _assert_all(errs, TOL_F32, "f32 mid size")
    assert ls.counters(2) == (10, 2, 8, 1)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_long_free_run_with_refreshes(dtype):
    # 40 free-running steps, the projector refreshed every 16: errors must not accumulate past the tolerance
    shapes = [(384, 520), (333, 200)]
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    stream = workloads.TorchGradientStream(shapes, 16, 0.01, 113, dtype, DEV)
    W = workloads.torch_weights(shapes, 113, dtype, DEV)
    ls = B.LayerSet(shapes, 32, s=8, dtype=dtype, device=DEV)
    lk = Lockstep(ls, tol=tol, k_signal=16)
    lk.set_weights(W)
    errs = []
    for step in range(40):
        G = stream.next_set()
        if step % 16 == 0:
            lk.refresh(G)
            assert ls.status() == B.NG_OK
        errs.append(lk.step(G, W, 1e-3))
    assert ls.status() == B.NG_OK
    _assert_all(errs, tol, "40 steps " + dtype)
    assert ls.counters(0) == (40, 0, 8, 3)


@pytest.mark.parametrize("dtype,shape,r", [("bf16", (16384, 32000), 1024), ("f32", (8192, 40000), 256),
                                           ("bf16", (32000, 16384), 512)])
def test_near_the_largest_matrix_the_library_accepts(dtype, shape, r):
    """One matrix just below the size limit (rows x leading dimension x 4 bytes < 2 GiB: the kernels address
    a matrix with 32-bit offsets), two steps, every tensor against the oracle.  The refresh invariants
    are not evaluated here (a full SVD of such a matrix takes minutes on the host): orthonormality and the
    captured energy of the signal part are checked directly."""
    m, n = shape
    assert 0.6 * 2 ** 31 < m * n * 4 < 2 ** 31
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    stream = workloads.TorchGradientStream([shape], 64, 0.01, 131, dtype, DEV)
    W = workloads.torch_weights([shape], 131, dtype, DEV)
    ls = B.LayerSet([shape], r, s=2, dtype=dtype, device=DEV)
    lk = Lockstep(ls, tol=tol, check_refresh=False)
    lk.set_weights(W)
    errs = []
    for step in range(2):
        G = stream.next_set()
        if step == 0:
            lk.refresh(G)
            assert ls.status() == B.NG_OK
            P = ls.P(0).double()
            eye = torch.eye(r, dtype=torch.float64, device=DEV)
            orth = float((P.T @ P - eye).abs().max())
            print("orthonormality", orth)
            # the last orthonormalisation accumulates its Gram matrix over the rows in float: the bound
            # grows with the square root of the row count (5e-6 holds up to about 8000 rows)
            assert orth <= max(5e-6, 1e-7 * ls.eff_shape(0)[0] ** 0.5)
            # G = A B^T + 0.01 E with A, B ~ N(0, 1/k), k = 64: the rank-64 signal carries m n / k of the
            # energy against 1e-4 m n of the noise, i.e. a share of 1 / (1 + 1e-4 k) = 0.99364 in
            # expectation; a projector that holds the signal subspace keeps at least that share (plus
            # r / min(m, n) of the noise)
            Gd = G[0].double()
            kept = float(((P.T @ Gd) ** 2).sum() / (Gd ** 2).sum())
            print("kept energy", kept)
            assert kept >= (1.0 / (1.0 + 1e-4 * 64)) * (1.0 - 1e-3)
            del P, Gd, eye
        errs.append(lk.step(G, W, 1e-3))
    assert ls.status() == B.NG_OK
    _assert_all(errs, tol, "near-maximum %s %s" % (dtype, shape))


def test_low_memory_projector_bf16_copies_only():
    """proj_dtype = bf16: no float projector is kept (NG_BUF_P has 0 bytes); a refresh builds it in the
    workspace, rounds it into the two bf16 copies the GEMMs multiply with and drops it.  The oracle steps
    with that bf16 projector, which is orthonormal to the rounding of bf16 only (orth_tol).  Ragged
    shapes, both sides, a second refresh in the middle of the run, then one block of the 1.1B shapes."""
    shapes = [(384, 520), (200, 333), (520, 384), (333, 200)]
    sides = [B.NG_SIDE_LEFT, B.NG_SIDE_LEFT, B.NG_SIDE_RIGHT, B.NG_SIDE_RIGHT]
    stream = workloads.TorchGradientStream(shapes, 16, 0.01, 97, "bf16", DEV)
    W = workloads.torch_weights(shapes, 97, "bf16", DEV)
    ls = B.LayerSet(shapes, 64, s=4, dtype="bf16", device=DEV, sides=sides, proj_dtype="bf16")
    assert all(ls.sizes[i][B.NG_BUF_P] == 0 for i in range(len(shapes)))
    lk = Lockstep(ls, tol=TOL_BF16, k_signal=16, orth_tol=2e-3)
    lk.set_weights(W)
    errs = []
    for step in range(8):
        G = stream.next_set()
        if step in (0, 5):
            lk.refresh(G)
            assert ls.status() == B.NG_OK
        errs.append(lk.step(G, W, 1e-3))
    assert ls.status() == B.NG_OK
    _assert_all(errs, TOL_BF16, "low-memory projector")
    assert ls.counters(0) == (8, 3, 3, 2)
    # a checkpoint is the buffers as they are (the copies live in NG_BUF_AUX): restore into a fresh layer
    # set, mark the copies valid, and the next step gives the same bits
    G = stream.next_set()
    ls2 = B.LayerSet(shapes, 64, s=4, dtype="bf16", device=DEV, sides=sides, proj_dtype="bf16")
    torch.cuda.synchronize()
    for row, row2 in zip(ls.buffers, ls2.buffers):
        for b, b2 in zip(row, row2):
            b2.copy_(b)
    for i in range(len(shapes)):
        B.ng_set_counters(ls2.st, i, *ls.counters(i))
    ls2.commit_projector(clear_history=False)
    W2 = [w.clone() for w in W]
    ls.step(G, W, 1e-3)
    ls2.step(G, W2, 1e-3)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(W, W2))
    # 1.1B shapes
    cfg = workloads.CONFIGS["c5"]
    ls, errs = _run(cfg.matrices()[:7], cfg.r, cfg.s, "bf16", 3, seed=cfg.seed, k=cfg.k, check=[0, 4, 6],
                    energy_tol=1e-3, orth_tol=2e-3, proj_dtype="bf16")
    _assert_all(errs, TOL_BF16, "low-memory projector, c5 block")


@pytest.mark.parametrize("name,dtype", [("ft4", "f32"), ("ft4", "bf16"), ("ft8", "f32"), ("ft8", "bf16")])
def test_fine_tuning_shaped_block(name, dtype):
    # one block of the RoBERTa-Base-shaped sets: rank 4 / 8, far below a GEMM tile
    cfg = workloads.CONFIGS[name]
    shapes = cfg.matrices()[:6]
    ls, errs = _run(shapes, cfg.r, cfg.s, dtype, cfg.s + 2, seed=cfg.seed, k=cfg.k, check=[0, 4, 5], lr=cfg.lr)
    # lr = 2e-5 and rank 4: the update is ~1e-6, a few hundred fp32 steps of a weight, so "dW"
    # (relative to the update) is bounded by the weights' rounding, not by the GEMM; the
    # rounding-interval check still applies to every element
    _assert_all(errs, TOL_F32 if dtype == "f32" else TOL_BF16, "%s %s" % (name, dtype), skip=("dW",))


@pytest.mark.parametrize("ranks,s", [([3, 4, 2, 1], 4), ([5, 8, 7, 6], 3), ([13, 16, 9, 11], 0)])
def test_small_rank_f32_ragged_strided(ranks, s):
    # fp32 layer sets with every rank <= 16 take the vector-ALU projection / update: ranks that are
    # not the kernel's 4 / 8 / 16 classes, row counts that are not multiples of a 128-row chunk,
    # column counts that are not multiples of 4, strided weights (rest untouched) and gradients
    # (NaN beyond column n), with and without the Fisher history
    shapes = [(300, 517), (129, 66), (1000, 30), (64, 1030)]
    ls, errs = _run(shapes, ranks, s, "f32", 6, seed=83, k=12, pad_w=3, pad_g=5)
    _assert_all(errs, TOL_F32, "small ranks %s" % ranks)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_right_side_projection(dtype):
    # R = G Q with the n x r factor (the usual choice for m > n), mixed with left-side matrices in
    # one layer set; ragged sizes, strided operands, GPU refresh of both kinds
    shapes = [(520, 384), (200, 333), (333, 200), (384, 520), (130, 64)]
    sides = [B.NG_SIDE_RIGHT, B.NG_SIDE_RIGHT, B.NG_SIDE_RIGHT, B.NG_SIDE_LEFT, B.NG_SIDE_RIGHT]
    ls, errs = _run(shapes, [64, 24, 40, 64, 20], 4, dtype, 7, seed=67, k=64, sides=sides, pad_w=3, pad_g=5)
    _assert_all(errs, TOL_F32 if dtype == "f32" else TOL_BF16, "right side " + dtype)
    assert ls.P(0).shape == (384, 64) and ls.M(0).shape[0] == 64


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_count_normaliser_while_the_ring_fills(dtype):
    # 1/count instead of 1/s: differs from the default on the first s - 1 steps
    ls, errs = _run([(200, 333), (130, 64)], 24, 6, dtype, 9, seed=71, k=24, fisher_norm="count")
    _assert_all(errs, TOL_F32 if dtype == "f32" else TOL_BF16, "count normaliser " + dtype)


@pytest.mark.parametrize("dtype,hist", [("f32", "f32"), ("bf16", "f32"), ("bf16", "bf16")])
def test_history_carry_over_across_refresh(dtype, hist):
    # carry_history: a refresh in the middle of a run re-expresses the slots in the new basis, rebuilds
    # the Gram matrix and keeps the ring position; left- and right-side matrices
    shapes = [(200, 333), (333, 200), (130, 64)]
    sides = [B.NG_SIDE_LEFT, B.NG_SIDE_RIGHT, B.NG_SIDE_LEFT]
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    stream = workloads.TorchGradientStream(shapes, 24, 0.01, 73, dtype, DEV)
    W = workloads.torch_weights(shapes, 73, dtype, DEV)
    ls = B.LayerSet(shapes, 24, s=4, dtype=dtype, device=DEV, sides=sides, carry_history=True,
                    hist_dtype=hist if dtype == "bf16" else None)
    lk = Lockstep(ls, tol=tol, k_signal=24)
    lk.set_weights(W)
    errs = []
    for step in range(9):
        G = stream.next_set()
        if step in (0, 3, 6):
            lk.refresh(G)
            assert ls.status() == B.NG_OK
            if step > 0:    # the whole Gram matrix was rebuilt from the carried slots
                for i in range(len(shapes)):
                    Hm = lk.states[i].H.reshape(4, -1)
                    err = np.abs(ls.K(i).cpu().numpy() - Hm @ Hm.T).max() / np.abs(Hm @ Hm.T).max()
                    assert err <= tol, ("K after carry", i, err)
        errs.append(lk.step(G, W, 1e-3))
    assert ls.status() == B.NG_OK
    _assert_all(errs, tol, "carry-over %s/%s" % (dtype, hist))
    assert ls.counters(0) == (9, 9 % 4, 4, 3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("gscale", [1e-4, 1e2])
def test_gradient_scale_extremes(dtype, gscale):
    # ||R||^2 far below and far above s * lambda: the damping-dominated and the history-dominated
    # regimes of the s x s system (lambda = 1e-3).  The upper scale is bounded by the oracle, not by
    # the library: the printed form g/lambda - U z/lambda^2, which the oracle evaluates literally in
    # float64, cancels about log10(||R||^2 / (s lambda)) digits (9.4 here; at a scale of 1e3 it is
    # left with fewer digits than the 1e-4 tolerance).
    ls, errs = _run([(200, 333), (130, 64)], 24, 4, dtype, 6, seed=79, k=24, gscale=gscale)
    _assert_all(errs, TOL_F32 if dtype == "f32" else TOL_BF16, "gradient scale %g %s" % (gscale, dtype))


def test_right_side_1b_shapes_sampled():
    # one block of the 1.1B shapes with the usual side rule (right where m > n: the 5461 x 2048 matrix)
    cfg = workloads.CONFIGS["c5"]
    shapes = cfg.matrices()[:7]
    ls, errs = _run(shapes, cfg.r, cfg.s, "bf16", 3, seed=cfg.seed, k=cfg.k, check=[0, 6], sides="auto",
                    energy_tol=1e-3)
    assert ls.side(6) == B.NG_SIDE_RIGHT and ls.side(0) == B.NG_SIDE_LEFT
    _assert_all(errs, TOL_BF16, "c5 block, auto sides")


def test_full_1b_layer_set_sampled():
    """All 168 matrices of the 1.1B configuration in one layer set (the grouped launches, tile
    tables and history size the benchmark times); the oracle follows one matrix of each shape
    from the first and the last transformer block."""
    cfg = workloads.CONFIGS["c5"]
    shapes = cfg.matrices()
    assert len(shapes) == 168
    check = [0, 4, 6, 161, 165, 167]
    assert {shapes[i] for i in check} == set(shapes)
    ls, errs = _run(shapes, cfg.r, cfg.s, cfg.dtype, 2, seed=cfg.seed, k=cfg.k, check=check, lr=cfg.lr,
                    energy_tol=1e-3)
    _assert_all(errs, TOL_BF16, "c5 full")
    for i in (0, 83, 167):
        assert ls.counters(i) == (2, 2, 2, 1)


@pytest.mark.parametrize("rank_cap", [None, 16, 8])
@pytest.mark.parametrize("pad_g", [0, 3])
@pytest.mark.parametrize("hist", ["f32", "bf16"])
def test_bf16_projection_slot_small_and_ragged(hist, pad_g, rank_cap):
    """The bf16 projection alone, against the oracle's R = P^T G on the projector the library holds
    (rounded to bf16, as the kernel's operand is), at shapes where single rows and columns matter:
    few contraction rows (the last row's share of the columns beyond the last whole 8-column chunk is
    taken from a padded copy), column counts that are not multiples of 8, and gradients that are column
    slices of wider tensors whose other columns hold NaN.  The slot's columns n..ldn-1 must be zero."""
    import oracle.natural_galore as ONG

    shapes = [(9, 13), (24, 45), (40, 8), (16, 7), (33, 300), (70, 261), (2, 9), (1, 12)]
    ranks = [4, 8, 8, 5, 16, 33, 2, 1]
    if rank_cap:   # every rank at most 16 / 8: the fine-tuning regime (row tiles almost empty)
        ranks = [min(r, rank_cap) for r in ranks]
    gen = torch.Generator(device="cpu").manual_seed(77)
    G, Gfull = [], []
    for (m, n) in shapes:
        g = torch.randn(m, n, generator=gen).to(torch.bfloat16).to(DEV)
        if pad_g:
            gf = torch.full((m, n + pad_g), float("nan"), dtype=torch.bfloat16, device=DEV)
            gf[:, :n] = g
            Gfull.append(gf)
            g = gf[:, :n]
        G.append(g)
    W = [torch.zeros(m, n, dtype=torch.bfloat16, device=DEV) for (m, n) in shapes]
    ls = B.LayerSet(shapes, ranks, s=2, dtype="bf16", device=DEV, hist_dtype=hist,
                    ld_g=[n + pad_g for (m, n) in shapes] if pad_g else None)
    ls.refresh(G)
    ls.step(G, W, 1e-3)
    assert ls.status() == B.NG_OK
    torch.cuda.synchronize()
    for i, (m, n) in enumerate(shapes):
        _, head, count, _ = ls.counters(i)
        slot = (head - 1) % 2
        Hs = ls.H(i)[slot].double().cpu().numpy()
        Pb = ls.P(i).to(torch.bfloat16).double().cpu().numpy()
        R = ONG.project(Pb, G[i].double().cpu().numpy())
        scale = np.abs(R).max()
        tol = 1e-5 if hist == "f32" else 2.0 ** -8
        assert np.abs(Hs[:, :n] - R).max() <= tol * scale, (i, shapes[i], np.abs(Hs[:, :n] - R).max() / scale)
        assert not Hs[:, n:].any(), (i, shapes[i], "padding columns of the slot are not zero")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_large_rank_refresh_and_step(dtype):
    # sketch width 608: more Jacobi block pairs and more block rows of the triangular inverse than at
    # the ranks of the benchmark layer sets
    ls, errs = _run([(700, 900), (640, 1000)], 600, 2, dtype, 3, seed=91, k=640)
    _assert_all(errs, TOL_F32 if dtype == "f32" else TOL_BF16, "large rank " + dtype)


def test_rank_beyond_the_lds_resident_triangular_inverse():
    # sketch width 1208 (38 blocks of 32): a block column of the inverse Cholesky factor no longer
    # fits in LDS, so the solved blocks are read back from global memory
    ls, errs = _run([(1300, 1400)], 1200, 2, "f32", 2, seed=92, k=1250)
    _assert_all(errs, TOL_F32, "rank 1200")


@pytest.mark.parametrize("hist", [None, "bf16"])
def test_wide_states_in_column_panels(hist):
    """Rows of 2304 padded elements or more: M, V and the history slots are stored as 2048-column panels
    (two whole panels and a ragged third one, on both sides, two exact panels, the narrowest second panel,
    beside one-panel matrices)."""
    shapes = [(96, 4200), (4131, 72), (80, 4096), (64, 520), (72, 2300), (72, 2270)]
    ls, errs = _run(shapes, 32, 3, "bf16", 6, seed=61, hist_dtype=hist, sides=[0, 1, 0, 0, 0, 0])
    assert [B.ng_get_layout(ls.st, i).panel_cols for i in range(6)] == [2048, 2048, 2048, 544, 2048, 2272]
    assert [B.ng_get_layout(ls.st, i).ldn for i in range(6)] == [4224, 4160, 4096, 544, 2304, 2272]
    _assert_all(errs, TOL_BF16, "panels hist=%s" % hist)


def test_microbench_copy_is_exact_and_reports_its_work():
    """The streaming copy behind the measured ceilings moves every byte (whole chunks, a ragged last chunk,
    fewer vectors than one workgroup), the read leaves its sink alone, the MFMA loop reports its flops."""
    cur = torch.cuda.current_stream().cuda_stream
    for n16 in (1, 255, 4096, 3 * 4096 + 777, 256 * 16 * 4096 + 5):
        src = torch.randint(-2**31, 2**31 - 1, (n16 * 4,), dtype=torch.int32, device=DEV)
        dst = torch.zeros(n16 * 4 + 4, dtype=torch.int32, device=DEV)
        ms, work = B.ng_microbench(B.NG_MB_COPY, src.data_ptr(), dst.data_ptr(), n16 * 16, 1, cur)
        torch.cuda.synchronize()
        assert work == 2 * n16 * 16 and ms > 0
        assert torch.equal(dst[:-4], src), n16
        assert int(dst[-4:].abs().sum()) == 0, "copy wrote past its size"
        sink = torch.full((4,), 7, dtype=torch.int32, device=DEV)
        ms, work = B.ng_microbench(B.NG_MB_READ, src.data_ptr(), sink.data_ptr(), n16 * 16, 2, cur)
        torch.cuda.synchronize()
        assert work == n16 * 16 and sink.tolist() == [7, 7, 7, 7]
    sink = torch.zeros(4, dtype=torch.float32, device=DEV)
    for which in (B.NG_MB_MFMA_BF16, B.NG_MB_MFMA_BF16_RANDOM):
        ms, work = B.ng_microbench(which, 0, sink.data_ptr(), 64, 1, cur)
        # 256 units x 4 SIMDs x 2 resident wavefronts, four workgroups deep; 64 trips of 8 MFMAs of 2*32*32*16 flop
        assert work == 256 * 4 * 2 * 4 * 64 * 8 * 2 * 32 * 32 * 16 and ms > 0
    torch.cuda.synchronize()
    assert sink.tolist() == [0.0] * 4
