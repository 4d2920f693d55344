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


class Lockstep:
    """GPU layer set + one oracle state per checked matrix, advanced together (free-running)."""

    def __init__(self, ls: B.LayerSet, check=None, tol=1e-4):
        self.ls = ls
        self.tol = tol
        self.check = list(range(len(ls.shapes))) if check is None else list(check)
        self.ohp = oracle_hparams(ls)
        self.states = {}
        for i in self.check:
            m, n = ls.shapes[i]
            side = "right" if ls.side(i) == B.NG_SIDE_RIGHT else "left"
            self.states[i] = oracle.init_state(m, n, ls.descs[i].r, ls.hp.s, side)
        self.Wo = {}
        self._refreshed = False

    def adopt_gpu_projector(self):
        """The oracle steps with the very projector the GPU holds (its basis is not unique)."""
        torch.cuda.synchronize()
        for i in self.check:
            self.states[i].P = to_f64(self.ls.P(i))

    def set_weights(self, weights):
        for i in self.check:
            self.Wo[i] = to_f64(weights[i])

    def refresh(self, grads):
        """GPU refresh; the oracle takes over the GPU's new basis (a refresh result is not unique)
        and clears its history or, with carry_history, re-expresses it in that basis."""
        carry = bool(self.ls.hp.carry_history) and self.ls.hp.s > 0 and self._refreshed
        self.ls.refresh(grads)
        torch.cuda.synchronize()
        for i in self.check:
            st = self.states[i]
            if carry:
                oracle.carry_history(st, to_f64(self.ls.P(i)))
            else:
                st.H[...] = 0.0
                st.head = 0
                st.count = 0
            st.n_refresh += 1
        self._refreshed = True
        self.adopt_gpu_projector()

    def step(self, grads, weights, lr):
        """One step on both sides.  Returns {matrix: {tensor name: rel err}}.

        R, K, w, M, V and W are compared free-running (relative to each tensor's maximum).
        The update direction N = M^/(sqrt(V^)+eps) is normalised element by element, so an
        element whose moments are tiny compared with the tensor's maximum amplifies an error
        that is small by that yardstick to O(1) (on the first step N is sign(g~)).  N is
        therefore pinned in two parts: M and V free-running as above, and "N_formula": the
        GPU's N against the oracle's direction formula applied to the GPU's own M and V.
        "N" and "N_far_frac" (elements off by more than tol) are reported, not asserted.
        The weight update is pinned by "W" free-running and by the oracle's update formula fed
        with the GPU's own N, "W_round_viol_frac": with x the unrounded fp64 update and
        d = tol * max|dW|, the stored weight (bf16 or fp32) must lie between round(x - d) and
        round(x + d) in its storage type, i.e. be the correct rounding of a value within the GEMM
        tolerance of x; the fraction of elements outside must be 0.  "dW" (fp32 weights: the
        applied update against the expected one, relative) is asserted by the callers only
        where the update is large against the weights' own rounding step; "W_upd_excess" and
        "W_mismatch_frac" (bf16) are reported."""
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
            e["N"] = rel_err(Ng, N0)
            nmax = np.max(np.abs(N0))
            Nf = oracle.adam_direction(to_f64(ls.M(i)[:, :n]), to_f64(ls.V(i)[:, :n]), st.t, self.ohp)
            e["N_formula"] = float(np.max(np.abs(Ng - Nf)) / np.max(np.abs(Nf)))
            e["N_far_frac"] = float(np.mean(np.abs(Ng - N0) > self.tol * nmax))
            Wp = prev[i][2]
            Wg = to_f64(weights[i])
            e["W"] = rel_err(Wg, self.Wo[i])
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
