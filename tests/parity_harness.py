"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle on
the same bytes and report per-tensor errors  max|x - x_oracle| / max|x_oracle|."""
from __future__ import annotations

import dataclasses

import numpy as np
import torch

import oracle
from paper_2410_16029_amd import binding as B


def rel_err(x, ref) -> float:
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    denom = np.max(np.abs(ref))
    if denom == 0.0:
        return float(np.max(np.abs(x)))
    return float(np.max(np.abs(x - ref)) / denom)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def oracle_hparams(ls: B.LayerSet) -> oracle.HParams:
    hp = ls.hp
    return oracle.HParams(s=hp.s, lam=float(hp.lambda_), beta1=float(hp.beta1), beta2=float(hp.beta2),
                          eps=float(hp.eps), scale=float(hp.scale), weight_decay=float(hp.weight_decay),
                          adam_mode="standard" if hp.adam_mode == B.NG_ADAM_STANDARD else "printed",
                          fisher_norm="count" if hp.fisher_norm == B.NG_NORM_COUNT else "s",
                          weight_dtype=ls.dtype)


# N = M^/(sqrt(V^)+eps) divides by the element's own root-mean-square gradient, so an absolute error e
# in the transformed gradients (small against the tensor's maximum) becomes about 2 e / sqrt(V^_ij) in
# N_ij: |dM^| <= e and, by Cauchy-Schwarz on the moving averages, |dV^| <= 2 e sqrt(V^) and |M^| <= about
# sqrt(V^).  N is therefore asserted at the tolerance on every element whose root second moment is at
# least max(sqrt(V^)) / KAPPA; below that the bound grows as 1 / sqrt(V^_ij) (the same e, amplified), and
# the fraction of elements that miss the plain tolerance is capped.  fp32 layer sets: KAPPA = 100 (an
# element with a hundredth of the largest root second moment still meets 1e-4; measured: 1.2e-5 at 50,
# 7.7e-5 at 500; far fraction at most 3.4e-3, where three quarters of the rows of R carry no signal: the
# cap says that 99 % of all elements meet the plain tolerance).  bf16 layer sets: no weighting at all -- once the oracle
# multiplies with the bf16 projector the kernels use, every element of N meets 2e-2 (measured 4e-3, the
# rounding of N to bf16; far fraction 0).
KAPPA = {"f32": 100.0, "bf16": float("inf")}
N_FAR_CAP = 1e-2
KAPPA_REPORT = (50.0, 500.0)


def direction_errors(Ng, N0, V_hat_root, tol, kappa):
    """Errors of the update direction Ng against the oracle's N0.  V_hat_root: the oracle's
    denominator sqrt(V^)+eps (or sqrt(V+eps)) per element."""
    nmax = np.max(np.abs(N0))
    diff = np.abs(Ng - N0)
    dmax = np.max(V_hat_root)
    out = {"N_raw": float(np.max(diff) / nmax), "N_far_frac": float(np.mean(diff > tol * nmax))}
    for kp in sorted(set(KAPPA_REPORT + (kappa,))):
        weight = np.maximum(1.0, (dmax / kp) / V_hat_root)
        val = float(np.max(diff / weight) / nmax)
        if kp == kappa:
            out["N"] = val
            out["N_illcond_frac"] = float(np.mean(weight > 1.0))
        else:
            out["N_k%g" % kp] = val
    return out


def refresh_invariants(P, G, r, k_signal=None, energy_tol=2e-3, orth_tol=5e-6, angle_tol=1e-4, label=""):
    """What a refresh must deliver whichever basis it picks (Sec. 1: P = the leading r left
    singular vectors of G): orthonormal columns, the energy of the best rank-r subspace up to
    energy_tol, the leading k_signal singular vectors inside range(P) where the spectrum has a gap
    after them, columns ordered by descending Ritz value, each column's largest entry positive.
    Returns the measured numbers."""
    P = np.asarray(P, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    orth = float(np.max(np.abs(P.T @ P - np.eye(r))))
    assert orth <= orth_tol, (label, "orthonormality", orth)
    if k_signal is not None and k_signal < min(G.shape):
        U, sig, _ = np.linalg.svd(G, full_matrices=False)
    else:
        U, sig = None, np.linalg.svd(G, compute_uv=False)
    best = float(np.sum(sig[:r] ** 2))
    B_ = P.T @ G
    captured = float(np.sum(B_ ** 2))
    deficit = 1.0 - captured / best
    assert deficit <= energy_tol, (label, "captured energy deficit", deficit)
    # (columns that are orthonormal only to orth_tol can "capture" that much more)
    assert captured <= best * (1.0 + max(1e-6, 4.0 * orth_tol)), (label, "captured more than the best rank-r subspace", deficit)
    out = {"orth": orth, "energy_deficit": deficit}
    if U is not None and k_signal <= r:
        # principal angles between range(P) and the signal subspace (an orthonormal basis of range(P):
        # P itself up to its orthonormality error)
        cosines = np.linalg.svd(U[:, :k_signal].T @ np.linalg.qr(P)[0], compute_uv=False)
        out["angle"] = float(1.0 - cosines.min())
        assert out["angle"] <= angle_tol, (label, "principal angle to the signal subspace", out["angle"])
    # sign rule: the entry of largest magnitude of every column is positive (up to ties: entries whose
    # magnitudes agree to the precision P is stored in)
    tie = max(1e-6, 4.0 * orth_tol)
    assert np.all(P.max(axis=0) >= np.abs(P).max(axis=0) * (1.0 - tie)), (label, "sign rule")
    ritz = np.sum(B_ ** 2, axis=1)
    assert np.all(ritz[:-1] >= ritz[1:] * (1.0 - 1e-3)), (label, "Ritz order")
    return out


class Lockstep:
    """GPU layer set + one oracle state per checked matrix, advanced together (free-running).

    projector="kernel" (default): the oracle steps with the projector the step's kernels multiply
    with -- for bf16 layer sets the bf16 copy of P the library makes at refresh / commit (both of
    its copies are checked to be exactly P rounded to bf16), for fp32 ones P itself.
    projector="stored": the oracle keeps the float P also for bf16 layer sets.
    k_signal: rank of the synthetic gradient's low-rank part (for the refresh's angle check)."""

    def __init__(self, ls: B.LayerSet, check=None, tol=1e-4, projector="kernel", k_signal=None,
                 check_refresh=True, energy_tol=2e-3, energy_tol_flat=2e-2, orth_tol=5e-6):
        self.ls = ls
        self.tol = tol
        self.check = list(range(len(ls.shapes))) if check is None else list(check)
        self.ohp = oracle_hparams(ls)
        self.projector = projector
        self.k_signal = k_signal
        self.check_refresh = check_refresh
        self.energy_tol = energy_tol
        self.orth_tol = orth_tol
        # rank below the gradient's signal rank: sigma_r and sigma_(r+1) are signal values of similar size,
        # where two power passes separate the wanted from the unwanted directions only slowly (the energy
        # given up is that of swapping nearly equal singular values; more passes shrink it, which
        # test_refresh_flat_spectrum_converges_with_more_power_passes checks)
        self.energy_tol_flat = energy_tol_flat
        self.kappa = KAPPA[ls.dtype]
        self.states = {}
        for i in self.check:
            m, n = ls.shapes[i]
            side = "right" if ls.side(i) == B.NG_SIDE_RIGHT else "left"
            self.states[i] = oracle.init_state(m, n, ls.descs[i].r, ls.hp.s, side)
        self.Wo = {}
        self.W0 = {}
        self.refresh_stats = []
        self._refreshed = False

    def adopt_gpu_projector(self):
        """The oracle steps with the very projector the GPU multiplies with (its basis is not unique)."""
        torch.cuda.synchronize()
        for i in self.check:
            if self.ls.dtype == "bf16":
                rounded = self.ls.P(i).to(torch.bfloat16).float()
                assert torch.equal(self.ls.Pb(i), rounded), "Pb is not P rounded to bf16"
                assert torch.equal(self.ls.PbT(i), rounded), "PbT is not P rounded to bf16"
            if self.ls.dtype == "bf16" and self.projector == "kernel":
                self.states[i].P = to_f64(self.ls.Pb(i))
            else:
                self.states[i].P = to_f64(self.ls.P(i))

    def set_weights(self, weights):
        for i in self.check:
            self.Wo[i] = to_f64(weights[i])
            self.W0[i] = self.Wo[i].copy()

    def refresh(self, grads):
        """GPU refresh; the oracle takes over the GPU's new basis (a refresh result is not unique)
        and clears its history or, with carry_history, re-expresses it in that basis.  The new
        basis itself is checked through refresh_invariants on every followed matrix."""
        carry = bool(self.ls.hp.carry_history) and self.ls.hp.s > 0 and self._refreshed
        self.ls.refresh(grads)
        torch.cuda.synchronize()
        for i in self.check:
            st = self.states[i]
            Pf = to_f64(self.ls.P(i))
            if self.check_refresh:
                G = to_f64(grads[i])
                r = self.ls.descs[i].r
                flat = self.k_signal is not None and r < min(self.k_signal, min(G.shape))
                self.refresh_stats.append(refresh_invariants(
                    Pf, G.T if st.side == "right" else G, r, self.k_signal,
                    energy_tol=self.energy_tol_flat if flat else self.energy_tol, orth_tol=self.orth_tol,
                    label="matrix %d %s r=%d" % (i, self.ls.shapes[i], r)))
            if carry:
                # the slots are re-expressed with the stored float projectors on both sides
                P_kernel = st.P
                st.P = self._P_float_prev[i]
                oracle.carry_history(st, Pf)
                st.P = P_kernel
            else:
                st.H[...] = 0.0
                st.head = 0
                st.count = 0
            st.n_refresh += 1
        self._refreshed = True
        self.adopt_gpu_projector()
        self._P_float_prev = {i: to_f64(self.ls.P(i)) for i in self.check}

    def step(self, grads, weights, lr):
        """One step on both sides.  Returns {matrix: {tensor name: rel err}}.

        R, K, w, M, V and W are compared free-running (relative to each tensor's maximum).
        "N": the update direction against the oracle's, free-running, weighted by the element's
        conditioning (see KAPPA above); "N_far_frac": the fraction of elements that miss the plain
        tolerance (capped by the callers; all of them lie below the conditioning threshold, or "N"
        would exceed the tolerance); "N_raw" (unweighted) and "N_formula" (the GPU's N
        against the oracle's direction formula applied to the GPU's own M and V) are reported.
        The weight update is pinned by "W" free-running, by "dW_total" (the accumulated update
        W - W_0 against the oracle's, relative; asserted by the callers where the update is large
        against the weights' rounding step) and by the oracle's update formula fed with the GPU's
        own N, "W_round_viol_frac": with x the unrounded fp64 update and d = tol * max|dW|, the
        stored weight (bf16 or fp32) must lie between round(x - d) and round(x + d) in its
        storage type, i.e. be the correct rounding of a value within the GEMM tolerance of x; the
        fraction of elements outside must be 0.  "dW" (fp32 weights: the applied update against
        the expected one, relative) is asserted by the callers only where the update is large
        against the weights' own rounding step; "W_upd_excess" and "W_mismatch_frac" (bf16) are
        reported."""
        ls = self.ls
        slot = {i: ls.counters(i)[1] for i in self.check}
        prev = {i: (self.states[i].M.copy(), self.states[i].V.copy(), to_f64(weights[i])) for i in self.check}
        ls.step(grads, weights, lr)
        torch.cuda.synchronize()
        out = {}
        for i in self.check:
            st = self.states[i]
            # The library holds the r x n state of the problem it works on; on the right side that
            # is the transposed problem, so the oracle's m x r tensors are compared transposed.
            right = st.side == "right"
            n = ls.eff_shape(i)[1]
            T = (lambda x: x.T) if right else (lambda x: x)
            self.Wo[i] = oracle.step(st, to_f64(grads[i]), self.Wo[i], lr, self.ohp)
            tr = st.trace
            e = {}
            H = ls.H(i)
            e["R"] = rel_err(to_f64(H[slot[i] if ls.hp.s > 0 else 0][:, :n]), T(tr["R"]))
            if ls.hp.s > 0:
                assert tr["slot"] == slot[i]
                e["K_row"] = rel_err(to_f64(ls.K(i)[slot[i]]), tr["K"][slot[i]])
                e["K"] = rel_err(to_f64(ls.K(i)), tr["K"])
                # w = (lambda I + K/s)^{-1} e_slot, from the oracle's own K
                s = ls.hp.s
                w_ref = np.linalg.solve(self.ohp.lam * np.eye(s) + tr["K"] / tr["h"], np.eye(s)[slot[i]])
                e["w"] = rel_err(to_f64(ls.w(i)), w_ref)
                e["pad"] = float(H[:, :, n:].abs().max().item()) if H.shape[2] > n else 0.0
            e["M"] = rel_err(to_f64(ls.M(i)[:, :n]), T(st.M))
            e["V"] = rel_err(to_f64(ls.V(i)[:, :n]), T(st.V))
            Ng = to_f64(ls.N(i))
            N0 = T(tr["N"])
            if self.ohp.adam_mode == "standard":
                root = np.sqrt(T(st.V) / (1.0 - self.ohp.beta2 ** st.t)) + self.ohp.eps
            else:
                root = np.sqrt(T(st.V) + self.ohp.eps)
            e.update(direction_errors(Ng, N0, root, self.tol, self.kappa))
            Nf = oracle.adam_direction(to_f64(ls.M(i)[:, :n]), to_f64(ls.V(i)[:, :n]), st.t, self.ohp)
            e["N_formula"] = float(np.max(np.abs(Ng - Nf)) / np.max(np.abs(Nf)))
            Wp = prev[i][2]
            Wg = to_f64(weights[i])
            e["W"] = rel_err(Wg, self.Wo[i])
            e["dW_total"] = rel_err(Wg - self.W0[i], self.Wo[i] - self.W0[i])
            # the accumulated update in units of the bf16 spacing at the largest weight
            e["dW_total_steps"] = float(np.max(np.abs(self.Wo[i] - self.W0[i]))
                                        / 2.0 ** (np.floor(np.log2(np.max(np.abs(self.Wo[i])))) - 7))
            upd = (lambda hp_: oracle.back_project_update_right(Wp, st.P, Ng.T, lr, hp_)) if right else \
                  (lambda hp_: oracle.back_project_update(Wp, st.P, Ng, lr, hp_))
            W_expect = upd(self.ohp)
            dmax = np.max(np.abs(W_expect - Wp))
            x = upd(dataclasses.replace(self.ohp, weight_dtype="f32"))
            d = self.tol * dmax
            if ls.dtype == "bf16":
                big = np.maximum(np.maximum(np.abs(W_expect), np.abs(Wg)), 1e-30)
                step_bf16 = 2.0 ** (np.floor(np.log2(big)) - 7)
                e["W_upd_excess"] = float(np.max(np.abs(Wg - W_expect) / (step_bf16 + self.tol * dmax)))
                e["W_mismatch_frac"] = float(np.mean(Wg != W_expect))
                lo, hi = oracle.round_to_bf16(x - d), oracle.round_to_bf16(x + d)
            else:
                e["dW"] = rel_err(Wg - Wp, W_expect - Wp)
                lo = (x - d).astype(np.float32).astype(np.float64)   # IEEE round-to-nearest-even
                hi = (x + d).astype(np.float32).astype(np.float64)
            e["W_round_viol_frac"] = float(np.mean((Wg < lo) | (Wg > hi)))
            t, head, count, nref = ls.counters(i)
            assert (t, head, count, nref) == (st.t, st.head if ls.hp.s > 0 else 0, st.count, st.n_refresh), \
                ((t, head, count, nref), (st.t, st.head, st.count, st.n_refresh))
            out[i] = e
        return out


def summarize(errs_list):
    keys = sorted({k for step in errs_list for e in step.values() for k in e})
    return {k: max(e[k] for step in errs_list for e in step.values() if k in e) for k in keys}


def worst(errs_list, key):
    return max(e[key] for step in errs_list for e in step.values() if key in e)
