"""Plain float64 definition of one Natural GaLore optimizer step (numpy only).

TEST INFRASTRUCTURE: imported only by tests, the smoke check and the
benchmark's CPU-baseline leg.  It is deliberately slow and literal -- every
function follows one passage of the paper, in the paper's order, with no
blocking, fusion or reordering -- and it shares no code with the HIP library.

Letters.  The paper writes the weight/gradient as n x m and the projector as
n x r; here (as in the rest of this repository) the weight W and gradient G are
m x n, the projector P is m x r with orthonormal columns, the low-rank gradient
R = P^T G is r x n, the Adam moments M, V are r x n and the history H keeps the
last s low-rank gradients (s x r x n).  The paper's stacked matrix "G" of
vectorised low-rank gradients is called ``Hmat`` (rn x s) here to keep it apart
from the full gradient.

Readings of the paper taken here (the paper is silent or inconsistent):
  * the empirical Fisher carries the 1/h normaliser of Sec. 2.2's empirical-FIM
    equation, with h = s fixed:  F = lambda*I + (1/s) * sum_i vec(H_i) vec(H_i)^T,
    i.e. Woodbury's U is Hmat / sqrt(s);  empty slots are zero;
  * the history holds exactly s slots and the current low-rank gradient is
    pushed into it before the transform (Sec. 2.4 lists vec(g_k) first);
  * s = 0 bypasses the transform: the step is then GaLore with Adam (Sec. 2.2,
    the sentence after the Adam equations);
  * "sent to the Adam optimizer" (end of Sec. 2.4) means Adam as published by
    Kingma & Ba: bias-corrected moments, epsilon outside the root
    (``adam_mode="standard"``).  The three equations exactly as printed in
    Sec. 2.2 -- no bias correction, epsilon inside the root -- are
    ``adam_mode="printed"``;
  * update  W <- W - lr * (scale * P N + weight_decay * W)  (Sec. 2.2, update
    equation; scale and weight_decay default to 1 and 0);
  * a refresh keeps M, V and the step counter and clears the history (its slots
    are coordinates in the old basis);
  * ``side="right"`` projects with the other factor of the compact SVD
    g = P Sigma Q^T of Sec. 1: R = G Q (m x r) with Q n x r, moments and history
    m x r, update W - lr * (scale * N Q^T + weight_decay * W).  The paper writes only
    the left form; the right form is the same method applied to G^T.

Pins (tests/test_oracle_pins.py): the Woodbury route against the explicit
rn x rn damped-Fisher solve, closed forms for one slot and for orthogonal
slots, the large-lambda limit, GaLore-Adam against torch.optim.Adam when s = 0,
the first-step Adam closed form, orthonormality / lossless projection /
Eckart-Young for the projector, exact integer bookkeeping, and bf16 rounding
against torch's conversion.  Parity unpinned: the individual trailing singular
vectors returned by ``top_r_left_singular_vectors`` when the r-th and (r+1)-th
singular values are not separated (only subspace invariants are pinned there).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import scipy.linalg


@dataclass
class HParams:
    s: int = 4
    lam: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    scale: float = 1.0
    weight_decay: float = 0.0
    adam_mode: str = "standard"      # "standard" | "printed"
    fisher_norm: str = "s"           # "s": 1/s always | "count": 1/(valid slots) while the ring fills
    weight_dtype: str = "f32"        # "f32" | "bf16": storage type of W


@dataclass
class OracleState:
    P: np.ndarray                    # m x r (side "left") or n x r (side "right": the Q factor)
    M: np.ndarray                    # r x n
    V: np.ndarray                    # r x n
    H: np.ndarray                    # s x r x n ring buffer
    t: int = 0                       # steps taken (1-based after the first step)
    head: int = 0                    # slot the next push writes
    count: int = 0                   # valid slots, min(pushes since clear, s)
    n_refresh: int = 0
    trace: dict = field(default_factory=dict)   # intermediates of the last step
    side: str = "left"


def init_state(m: int, n: int, r: int, s: int, side: str = "left") -> OracleState:
    if side == "left":
        return OracleState(
            P=np.zeros((m, r)), M=np.zeros((r, n)), V=np.zeros((r, n)),
            H=np.zeros((max(s, 0), r, n)))
    if side == "right":
        return OracleState(
            P=np.zeros((n, r)), M=np.zeros((m, r)), V=np.zeros((m, r)),
            H=np.zeros((max(s, 0), m, r)), side="right")
    raise ValueError(side)


# --------------------------------------------------------------------------
# Sec. 1, "Gradient Low-Rank Projection (GaLore)": compact SVD and projection
# --------------------------------------------------------------------------
def top_r_left_singular_vectors(G: np.ndarray, r: int) -> np.ndarray:
    """P of the compact SVD G = P Sigma Q^T, first r columns (Sec. 1; Sec. 2.2).

    LAPACK via numpy.  Each column's sign is fixed so that its entry of largest
    magnitude is positive (an SVD leaves the sign free).
    """
    U, _, _ = np.linalg.svd(np.asarray(G, dtype=np.float64), full_matrices=False)
    P = U[:, :r].copy()
    rows = np.argmax(np.abs(P), axis=0)
    signs = np.sign(P[rows, np.arange(P.shape[1])])
    signs[signs == 0] = 1.0
    return P * signs


def top_r_right_singular_vectors(G: np.ndarray, r: int) -> np.ndarray:
    """Q of the compact SVD G = P Sigma Q^T, first r columns (Sec. 1), same sign rule."""
    _, _, Vt = np.linalg.svd(np.asarray(G, dtype=np.float64), full_matrices=False)
    Q = Vt[:r].T.copy()
    rows = np.argmax(np.abs(Q), axis=0)
    signs = np.sign(Q[rows, np.arange(Q.shape[1])])
    signs[signs == 0] = 1.0
    return Q * signs


def project(P: np.ndarray, G: np.ndarray) -> np.ndarray:
    """Low-rank gradient R = P^T G (Sec. 1, projection equation)."""
    return P.T @ np.asarray(G, dtype=np.float64)


def project_right(Q: np.ndarray, G: np.ndarray) -> np.ndarray:
    """Low-rank gradient from the right factor: R = G Q (m x r)."""
    return np.asarray(G, dtype=np.float64) @ Q


# --------------------------------------------------------------------------
# Sec. 2.4: history of the last s low-rank gradients
# --------------------------------------------------------------------------
def push_history(state: OracleState, R: np.ndarray) -> int:
    """Store R in slot ``head`` and advance the ring.  Returns the slot used."""
    s = state.H.shape[0]
    slot = state.head
    state.H[slot] = R
    state.head = (state.head + 1) % s
    state.count = min(state.count + 1, s)
    return slot


def fisher_history_matrix(H: np.ndarray) -> np.ndarray:
    """rn x s matrix whose columns are the vectorised history slots (Sec. 2.4)."""
    s = H.shape[0]
    return H.reshape(s, -1).T.copy()


def natural_gradient_transform(H: np.ndarray, R: np.ndarray, lam: float, h: int = None) -> tuple:
    """Inverse damped empirical Fisher applied to R through Woodbury (Sec. 2.4).

    F = lam*I + U U^T with U = Hmat / sqrt(h), h = s unless given (the normaliser of Sec. 2.2's
    empirical FIM; h = number of valid slots is the other reading while the ring fills).
    Following the section's steps: S = I + U^T U / lam,  y = U^T vec(R),  Cholesky solve S z = y,
    g~ = vec(R)/lam - U z / lam^2.  Returns (g~ as r x n, dict of K, S, y, z).
    """
    s = H.shape[0]
    Hmat = fisher_history_matrix(H)
    U = Hmat / np.sqrt(s if h is None else h)
    g = R.reshape(-1)
    K = Hmat.T @ Hmat                       # s x s Gram of the stored slots
    S = np.eye(s) + (U.T @ U) / lam
    y = U.T @ g
    z = scipy.linalg.cho_solve(scipy.linalg.cho_factor(S, lower=True), y)
    g_nat = g / lam - (U @ z) / lam ** 2
    return g_nat.reshape(R.shape), {"K": K, "S": S, "y": y, "z": z}


# --------------------------------------------------------------------------
# Sec. 2.2: Adam moments in the r x n space, and the weight update
# --------------------------------------------------------------------------
def adam_direction(M, V, t: int, hp: HParams):
    """Update direction N from the moments after step t (Sec. 2.2, third Adam equation)."""
    if hp.adam_mode == "standard":
        m_hat = M / (1.0 - hp.beta1 ** t)
        v_hat = V / (1.0 - hp.beta2 ** t)
        return m_hat / (np.sqrt(v_hat) + hp.eps)
    if hp.adam_mode == "printed":
        return M / np.sqrt(V + hp.eps)
    raise ValueError(hp.adam_mode)


def adam_moments(M, V, g, t: int, hp: HParams):
    """Moment recursion and update direction N (Sec. 2.2, Adam equations)."""
    M_new = hp.beta1 * M + (1.0 - hp.beta1) * g
    V_new = hp.beta2 * V + (1.0 - hp.beta2) * g * g
    return M_new, V_new, adam_direction(M_new, V_new, t, hp)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (ties to even), as float64.

    bfloat16 keeps 1 sign, 8 exponent and 7 mantissa bits.  Works on the
    float64 bit pattern directly (one rounding, not two); valid for finite
    values inside bfloat16's normal range, which is asserted.
    """
    x = np.ascontiguousarray(x, dtype=np.float64)
    a = np.abs(x)
    nz = a[a > 0]
    if nz.size:
        assert nz.min() >= 2.0 ** -126 and nz.max() < 2.0 ** 127, "outside bf16 normal range"
    bits = x.view(np.uint64)
    drop = np.uint64(52 - 7)
    lsb = (bits >> drop) & np.uint64(1)
    rounded = bits + ((np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1)) + lsb
    rounded &= ~((np.uint64(1) << drop) - np.uint64(1))
    return rounded.view(np.float64).reshape(x.shape)


def back_project_update(W, P, N, lr: float, hp: HParams):
    """W <- W - lr * (scale * P N + weight_decay * W) (Sec. 2.2, update equation)."""
    W = np.asarray(W, dtype=np.float64)
    W_new = W - lr * (hp.scale * (P @ N) + hp.weight_decay * W)
    if hp.weight_dtype == "bf16":
        W_new = round_to_bf16(W_new)
    return W_new


def back_project_update_right(W, Q, N, lr: float, hp: HParams):
    """W <- W - lr * (scale * N Q^T + weight_decay * W): the update of the right-side form."""
    W = np.asarray(W, dtype=np.float64)
    W_new = W - lr * (hp.scale * (N @ Q.T) + hp.weight_decay * W)
    if hp.weight_dtype == "bf16":
        W_new = round_to_bf16(W_new)
    return W_new


# --------------------------------------------------------------------------
# The step and the refresh
# --------------------------------------------------------------------------
def carry_history(state: OracleState, P_new: np.ndarray) -> None:
    """Re-express the stored slots in a new basis: H_j <- (P_new^T P_old) H_j.

    A slot holds the coordinates, in the old basis, of the part of an old gradient inside the old
    subspace (P_old H_j); its coordinates in the new basis are P_new^T (P_old H_j).  On the right
    side the slots are m x r and the r x r change of basis multiplies from the right, transposed.
    """
    T = P_new.T @ state.P
    for j in range(state.H.shape[0]):
        state.H[j] = state.H[j] @ T.T if state.side == "right" else T @ state.H[j]


def refresh_projector(state: OracleState, G: np.ndarray, carry: bool = False) -> None:
    """P <- top-r left (right, for side "right") singular vectors of the current gradient.

    The history is cleared (default: its slots are coordinates in the old basis), or, with
    ``carry``, re-expressed in the new basis and kept together with head and count.
    """
    r = state.P.shape[1]
    if state.side == "right":
        P_new = top_r_right_singular_vectors(G, r)
    else:
        P_new = top_r_left_singular_vectors(G, r)
    if carry:
        carry_history(state, P_new)
    else:
        state.H[...] = 0.0
        state.head = 0
        state.count = 0
    state.P = P_new
    state.n_refresh += 1


def step(state: OracleState, G: np.ndarray, W: np.ndarray, lr: float, hp: HParams) -> np.ndarray:
    """One Natural GaLore step on one weight matrix.  Returns the new W.

    Order (Sec. 2.4, first and last paragraphs): project, push into the
    history, natural-gradient transform, Adam, back-project and update.
    """
    state.t += 1
    right = state.side == "right"
    R = project_right(state.P, G) if right else project(state.P, G)
    tr = {"R": R}
    if hp.s > 0:
        slot = push_history(state, R)
        h = state.count if hp.fisher_norm == "count" else None
        g_nat, parts = natural_gradient_transform(state.H, R, hp.lam, h)
        parts["h"] = hp.s if h is None else h
        tr.update(parts)
        tr["slot"] = slot
    else:
        g_nat = R
    tr["g_nat"] = g_nat
    state.M, state.V, N = adam_moments(state.M, state.V, g_nat, state.t, hp)
    tr["N"] = N
    state.trace = tr
    if right:
        return back_project_update_right(W, state.P, N, lr, hp)
    return back_project_update(W, state.P, N, lr, hp)
