"""CPU oracle for the Fira optimizer step ("Fira with Adam", Algorithm 1, Appendix A.1).

TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute and is used by
`tests/`, by `__graft_entry__.smoke()` and by the `cpu_baseline` leg of `bench.py`; nothing in
the product path may import it.  It shares no code with the HIP path and does not import it.

It is Algorithm 1's loop body below the SVD branch, executed step by step in fp64 with numpy,
in the paper's order and notation.  A dense matrix product (`@`) is the only library primitive
used as a step; there is no blocking, fusion or re-association beyond what the algorithm states.

Readings taken where the paper is silent or inconsistent (each is listed in the design notes):

* step index: bias correction uses the 1-based step count (Eq. 4 needs t >= 1, while
  Algorithm 1 starts t at 0 and increments after the update);
* the limiter's ||S_{t-1}|| does not exist at a matrix's first step: that step is not limited
  and only records its norm;
* the remembered norm is the norm *after* limiting (Eq. 12 assigns S_t);
* epsilon appears in the denominators of the column factors and of the limiter as in
  Algorithm 1 (Eqs. 11-12 omit it);
* Adam's epsilon sits where Eq. 4 puts it (added to sqrt(V_t) before the bias factor);
* norms are l2 (columns) and Frobenius (S), consistent with Appendix C writing phi^2 as a ratio
  of sums of squares;
* m > n: the footnote of Sec. 3.3 gives R = G Q with Q n x r; the rest of the algorithm is read
  as the m <= n algorithm applied to the transposed problem, so there is one factor per *row*
  of G and the reduction always runs over the rank axis; m == n is the m <= n case;
* bf16 storage: W is re-rounded to bf16 (round to nearest even) after each update when the
  caller asks for it; all arithmetic stays fp64.

Parity pins live in tests/test_oracle_pins.py.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np


@dataclasses.dataclass
class OracleHparams:
    """Input line of Algorithm 1: eta, {beta1, beta2}, eps (Eq. 4), alpha, gamma."""

    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    alpha: float = 1.0
    gamma: float = 1.01


@dataclasses.dataclass
class OracleState:
    """Optimizer state of one weight matrix (Table "Comparison": mr + 2nr + 1 numbers):
    M, V (r x n when m <= n, m x r when m > n), the scalar ||S_{t-1}||, and the step count.
    P is held by the caller and passed to every step."""

    M: np.ndarray
    V: np.ndarray
    s_prev: Optional[float] = None  # None = no previous step yet
    t: int = 0

    @staticmethod
    def zeros(m: int, n: int, r: int) -> "OracleState":
        shape = (r, n) if m <= n else (m, r)
        return OracleState(np.zeros(shape), np.zeros(shape))

    def copy(self) -> "OracleState":
        return OracleState(self.M.copy(), self.V.copy(), self.s_prev, self.t)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bf16 value (8 significant bits, ties to even) of fp64 numbers, as fp64.
    Models the storage format of W; subnormal/overflow ranges are never reached here."""
    x = np.asarray(x, dtype=np.float64)
    mant, expo = np.frexp(x)  # x = mant * 2**expo, 0.5 <= |mant| < 1
    return np.ldexp(np.rint(mant * 256.0) / 256.0, expo)


def adam_correction(M, V, R, t, beta1, beta2, eps):
    """psi_t(R_t): Eqs. 2-4 applied to the low-rank gradient (Algorithm 1, Adam block).
    t is the 1-based step count.  Returns (M_t, V_t, N_t)."""
    M = beta1 * M + (1.0 - beta1) * R
    V = beta2 * V + (1.0 - beta2) * (R * R)
    N = (np.sqrt(1.0 - beta2 ** t) / (1.0 - beta1 ** t)) * (M / (np.sqrt(V) + eps))
    return M, V, N


def column_factors(N, R, eps):
    """K of Algorithm 1 ("Norm-Based Scaling"): k_i = ||N[:, i]|| / (||R[:, i]|| + eps)."""
    return np.sqrt(np.sum(N * N, axis=0)) / (np.sqrt(np.sum(R * R, axis=0)) + eps)


def matrix_factor(N, R, eps):
    """Eq. 9, the matrix-level factor of the "Fira-matrix" variant, with the same epsilon
    placement as the column form."""
    return np.sqrt(np.sum(N * N)) / (np.sqrt(np.sum(R * R)) + eps)


def limiter_factor(s, s_prev, gamma, eps):
    """Algorithm 1 ("Norm-Growth Limiter"): the scalar multiplying S_t,
    gamma / max(||S_t|| / (||S_{t-1}|| + eps), gamma).  No previous norm, or gamma = inf
    (the "w.o.-limiter" variant): factor 1."""
    if s_prev is None or np.isinf(gamma):
        return 1.0
    if s == 0.0:            # 0 / (0 + 0) only arises with eps = 0: a zero S stays zero, factor 1
        return 1.0
    den = s_prev + eps
    ratio = s / den if den > 0.0 else float("inf")
    return gamma / max(ratio, gamma)


def _step_short_rows(W, G, P, st: OracleState, hp: OracleHparams, scaling: str, variant: str = "full") -> Dict:
    """Algorithm 1's loop body for m <= n.  W, G: m x n.  P: m x r.  Mutates st; returns the new
    W and every intermediate."""
    t = st.t + 1
    R = P.T @ G                                  # R_t = P^T G_t                        (r x n)
    E = G - P @ R                                # (I - P P^T) G_t = G_t - P R_t        (m x n)
    M, V, N = adam_correction(st.M, st.V, R, t, hp.beta1, hp.beta2, hp.eps)
    if scaling == "column":
        k = column_factors(N, R, hp.eps)         # one factor per column
    elif scaling == "matrix":
        k = np.full(G.shape[1], matrix_factor(N, R, hp.eps))
    elif scaling == "none":                      # phi == 1: the "GaLore-add" update, Eq. 8
        k = np.ones(G.shape[1])
    else:
        raise ValueError(scaling)
    S = E * k[None, :]                           # S_t[:, i] = k_i S_t[:, i]
    if variant == "only_scaling":                # Appendix "Fira-only-scaling": the factors on the full gradient,
        S = G * k[None, :]                       # W_{t+1} = W_t - eta phi_t(R_t) G_t (limiter as in Algorithm 1)
    elif variant != "full":
        raise ValueError(variant)
    s_pre = float(np.sqrt(np.sum(S * S)))
    c = limiter_factor(s_pre, st.s_prev, hp.gamma, hp.eps)
    S = c * S
    s_post = c * s_pre
    G_tilde = hp.alpha * (P @ N + S)             # project back, complete the gradient
    if variant == "only_scaling":
        G_tilde = hp.alpha * S                   # no Adam term P psi(R)
    W_new = W - hp.lr * G_tilde
    st.M, st.V, st.s_prev, st.t = M, V, s_post, t
    return dict(W=W_new, R=R, E=E, N=N, k=k, S=S, s_pre=s_pre, c=c, s_post=s_post,
                update=G_tilde)


def fira_step(W, G, P, st: OracleState, hp: OracleHparams, *, scaling: str = "column",
              store_bf16: bool = False, variant: str = "full") -> Dict:
    """One Fira step for one weight matrix.

    W, G: m x n.  P: min(m, n) x r (P of Eq. 7 when m <= n, Q of the Sec. 3.3 footnote when
    m > n).  Returns a dict with the updated W (a new array) and the intermediates in the
    orientation of the inputs (R is r x n for m <= n and m x r for m > n; k has one entry per
    column for m <= n and per row for m > n)."""
    W = np.asarray(W, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    m, n = G.shape
    if W.shape != G.shape or P.shape[0] != min(m, n) or P.shape[1] > min(m, n):
        raise ValueError("shape mismatch")
    if m <= n:
        out = _step_short_rows(W, G, P, st, hp, scaling, variant)
    else:
        # transposed problem: (G^T, W^T) is n x m with n < m; state arrays are kept as m x r
        tst = OracleState(st.M.T, st.V.T, st.s_prev, st.t)
        out = _step_short_rows(W.T, G.T, P, tst, hp, scaling, variant)
        st.M, st.V, st.s_prev, st.t = tst.M.T, tst.V.T, tst.s_prev, tst.t
        for key in ("W", "R", "E", "N", "S", "update"):
            out[key] = out[key].T
    if store_bf16:
        out["W_unrounded"] = out["W"]
        out["W"] = round_to_bf16(out["W"])
    return out


def run(W0, grads, P_for_step, hp: OracleHparams, r: int, *, scaling: str = "column",
        store_bf16: bool = False, state: Optional[OracleState] = None):
    """Convenience loop: apply fira_step for every gradient in `grads`.  `P_for_step(i)` returns
    the projector to use at 0-based step i (the caller decides when it is refreshed; M, V, t and
    the remembered norm are kept across a switch, Sec. 4.2 "Loss spike analysis")."""
    m, n = np.asarray(W0).shape
    st = state if state is not None else OracleState.zeros(m, n, r)
    W = np.asarray(W0, dtype=np.float64)
    trace = []
    for i, G in enumerate(grads):
        out = fira_step(W, G, P_for_step(i), st, hp, scaling=scaling, store_bf16=store_bf16)
        W = out["W"]
        trace.append(out)
    return W, st, trace


# --------------------------------------------------------------------------------------------------
# Projector refresh (Sec. 3.3, Eq. 7; the "if t mod T = 0" branch of Algorithm 1)
# --------------------------------------------------------------------------------------------------

def top_r_projector(G: np.ndarray, r: int) -> np.ndarray:
    """Eq. 7: the first r left singular vectors of G (m <= n), or the first r right singular vectors
    (m > n, footnote of Sec. 3.3), from LAPACK's SVD.  Returns min(m, n) x r."""
    G = np.asarray(G, dtype=np.float64)
    U, _, Vt = np.linalg.svd(G, full_matrices=False)
    return U[:, :r] if G.shape[0] <= G.shape[1] else Vt[:r, :].T


def subspace_sines(P: np.ndarray, Q: np.ndarray) -> np.ndarray:
    """Sines of the principal angles between span(P) and span(Q) (both S x r, any bases): the
    singular values of (I - Pq Pq^T) Qq with orthonormalised Pq, Qq.  All zero iff the spans agree."""
    Pq, _ = np.linalg.qr(np.asarray(P, dtype=np.float64))
    Qq, _ = np.linalg.qr(np.asarray(Q, dtype=np.float64))
    return np.linalg.svd(Qq - Pq @ (Pq.T @ Qq), compute_uv=False)


def captured_energy(G: np.ndarray, P: np.ndarray) -> float:
    """||R||_F^2 / ||G||_F^2 for R = P^T G (or G P when m > n), with P orthonormalised first: the share
    of the gradient that the projection keeps.  Maximal, over all r-dimensional P, for Eq. 7's choice."""
    G = np.asarray(G, dtype=np.float64)
    Pq, _ = np.linalg.qr(np.asarray(P, dtype=np.float64))
    R = Pq.T @ G if G.shape[0] <= G.shape[1] else G @ Pq
    return float(np.sum(R * R) / np.sum(G * G))
