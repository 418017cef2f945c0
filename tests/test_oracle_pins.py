"""Pins for the CPU oracle: things the paper and the mathematics fix, independent of the oracle's
own code.  Each pin is a function of an oracle *module*, so that test_mutants_are_caught can run
the same pins on deliberately broken copies of the oracle and check that every planted mistake
is caught by at least one of them.

Citations are to the paper's sections/equations/algorithm (Fira, arXiv 2410.01623).
"""
import importlib.util
import math
import os
import sys
import types

import numpy as np
import pytest

from oracle import fira_oracle as ORC

HERE = os.path.dirname(os.path.abspath(__file__))


# ------------------------------------------------------------------------------------------
# helpers (no method arithmetic here beyond what each pin states explicitly)
# ------------------------------------------------------------------------------------------

def _orth(rng, m, r):
    q, _ = np.linalg.qr(rng.standard_normal((m, r)))
    return q


def _hp(o, **kw):
    return o.OracleHparams(**kw)


# ------------------------------------------------------------------------------------------
# brute force: a second, independent, loop-level statement of Algorithm 1 for tiny inputs.
# Written separately for both orientations (no transposition trick), scalars only.
# ------------------------------------------------------------------------------------------

def brute_force_steps(W, Gs, P, hp, left):
    W = [list(map(float, row)) for row in W]
    m, n = len(W), len(W[0])
    r = len(P[0])
    L = n if left else m
    M = [[0.0] * r for _ in range(L)]   # indexed [long index][rank index]
    V = [[0.0] * r for _ in range(L)]
    s_prev = None
    out = []
    for t, G in enumerate(Gs, start=1):
        # low-rank gradient, one length-r vector per long index
        R = [[0.0] * r for _ in range(L)]
        for j in range(L):
            for a in range(r):
                acc = 0.0
                if left:       # R[a, j] = sum_i P[i, a] G[i, j]
                    for i in range(m):
                        acc += P[i][a] * G[i][j]
                else:          # R[j, a] = sum_i G[j, i] Q[i, a]
                    for i in range(n):
                        acc += G[j][i] * P[i][a]
                R[j][a] = acc
        N = [[0.0] * r for _ in range(L)]
        bias = math.sqrt(1.0 - hp.beta2 ** t) / (1.0 - hp.beta1 ** t)
        for j in range(L):
            for a in range(r):
                M[j][a] = hp.beta1 * M[j][a] + (1.0 - hp.beta1) * R[j][a]
                V[j][a] = hp.beta2 * V[j][a] + (1.0 - hp.beta2) * R[j][a] ** 2
                N[j][a] = bias * M[j][a] / (math.sqrt(V[j][a]) + hp.eps)
        k = []
        for j in range(L):
            nn = math.sqrt(sum(x * x for x in N[j]))
            rr = math.sqrt(sum(x * x for x in R[j]))
            k.append(nn / (rr + hp.eps))
        # residual, scaled; and the back-projection of N
        S = [[0.0] * n for _ in range(m)]
        B = [[0.0] * n for _ in range(m)]
        for i in range(m):
            for j in range(n):
                if left:
                    pr = sum(P[i][a] * R[j][a] for a in range(r))
                    pn = sum(P[i][a] * N[j][a] for a in range(r))
                    S[i][j] = k[j] * (G[i][j] - pr)
                else:
                    pr = sum(R[i][a] * P[j][a] for a in range(r))
                    pn = sum(N[i][a] * P[j][a] for a in range(r))
                    S[i][j] = k[i] * (G[i][j] - pr)
                B[i][j] = pn
        s = math.sqrt(sum(x * x for row in S for x in row))
        if s_prev is None:
            c = 1.0
        else:
            c = hp.gamma / max(s / (s_prev + hp.eps), hp.gamma)
        s_prev = c * s
        for i in range(m):
            for j in range(n):
                W[i][j] -= hp.lr * hp.alpha * (B[i][j] + c * S[i][j])
        out.append(dict(W=[row[:] for row in W], c=c, s_pre=s, s_post=s_prev, k=k[:]))
    return out


# ------------------------------------------------------------------------------------------
# the pins
# ------------------------------------------------------------------------------------------

def pin_hand_case(o):
    """Hand-derived 2x2 example (tests/golden/hand_case_2x2.txt)."""
    rows = {}
    with open(os.path.join(HERE, "golden", "hand_case_2x2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            rows[(int(p[0]), p[1])] = [float(x) for x in p[2:]]
    hp = _hp(o, lr=0.1, eps=0.0)
    P = np.array([[1.0], [0.0]])
    Gs = [np.array([[3.0, 4.0], [1.0, -2.0]]), np.array([[3.0, 4.0], [5.0, -10.0]]),
          np.array([[3.0, 4.0], [1.0, -2.0]])]
    st = o.OracleState.zeros(2, 2, 1)
    W = np.zeros((2, 2))
    for t, G in enumerate(Gs, start=1):
        out = o.fira_step(W, G, P, st, hp)
        W = out["W"]
        np.testing.assert_allclose(out["s_pre"], rows[(t, "s_pre")][0], rtol=1e-13)
        np.testing.assert_allclose(out["c"], rows[(t, "c")][0], rtol=1e-13)
        np.testing.assert_allclose(st.s_prev, rows[(t, "s_post")][0], rtol=1e-13)
        np.testing.assert_allclose(W.ravel(), rows[(t, "W")], rtol=1e-13, atol=1e-16)
    # with the usual eps = 1e-8 everything moves by <~ 1e-6 relative
    st = o.OracleState.zeros(2, 2, 1)
    W = np.zeros((2, 2))
    hp = _hp(o, lr=0.1)
    for t, G in enumerate(Gs, start=1):
        W = o.fira_step(W, G, P, st, hp)["W"]
        np.testing.assert_allclose(W.ravel(), rows[(t, "W")], rtol=2e-6)


def pin_brute_force(o):
    """Loop-level restatement of Algorithm 1 on tiny random inputs, both orientations."""
    rng = np.random.default_rng(11)
    for (m, n, r) in [(5, 7, 2), (7, 5, 2), (4, 4, 3), (4, 6, 3)]:
        left = m <= n
        P = _orth(rng, min(m, n), r)
        W0 = rng.standard_normal((m, n))
        Gs = [rng.standard_normal((m, n)) * (1.0 + 3.0 * (i % 4 == 3)) for i in range(12)]
        hp = _hp(o, lr=0.05, alpha=0.25)
        ref = brute_force_steps(W0.tolist(), [g.tolist() for g in Gs], P.tolist(), hp, left)
        st = o.OracleState.zeros(m, n, r)
        W = W0
        fired = 0
        for i, G in enumerate(Gs):
            out = o.fira_step(W, G, P, st, hp)
            W = out["W"]
            np.testing.assert_allclose(W, np.array(ref[i]["W"]), rtol=1e-12, atol=1e-14)
            np.testing.assert_allclose(out["c"], ref[i]["c"], rtol=1e-12)
            np.testing.assert_allclose(out["s_pre"], ref[i]["s_pre"], rtol=1e-12)
            np.testing.assert_allclose(out["k"], ref[i]["k"], rtol=1e-12)
            fired += out["c"] < 1.0
        assert fired >= 1, "the spike steps must exercise the limiter"


def pin_full_rank_identity_is_adam(o):
    """r = m, P = I: the residual vanishes exactly and W follows element-wise Adam (Eqs. 2-4).
    Checked against torch.optim.Adam (library routine), whose eps is set each step to
    eps / sqrt(1 - beta2^t) so that it equals Eq. 4's placement of epsilon."""
    import torch
    rng = np.random.default_rng(3)
    m, n = 6, 9
    W0 = rng.standard_normal((m, n))
    Gs = [rng.standard_normal((m, n)) for _ in range(8)]
    for eps in (0.0, 1e-8, 1e-3):
        hp = _hp(o, lr=1e-2, eps=eps)
        st = o.OracleState.zeros(m, n, m)
        W = W0
        p = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
        opt = torch.optim.Adam([p], lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=eps)
        for t, G in enumerate(Gs, start=1):
            out = o.fira_step(W, G, np.eye(m), st, hp)
            W = out["W"]
            assert np.all(out["E"] == 0.0) and out["s_pre"] == 0.0 and np.all(out["S"] == 0.0)
            for g in opt.param_groups:
                g["eps"] = eps / math.sqrt(1.0 - hp.beta2 ** t)
            p.grad = torch.tensor(G, dtype=torch.float64)
            opt.step()
            np.testing.assert_allclose(W, p.detach().numpy(), rtol=1e-11, atol=1e-13)


def pin_full_rank_rotation(o):
    """r = m with a random orthogonal P: residual ~ 0 and W_{t+1} = W_t - eta alpha P Adam(P^T G)
    (Adam in rotated coordinates, Eq. 6)."""
    import torch
    rng = np.random.default_rng(4)
    m, n = 5, 8
    P = _orth(rng, m, m)
    W0 = rng.standard_normal((m, n))
    hp = _hp(o, lr=1e-2, eps=0.0, alpha=0.5)
    st = o.OracleState.zeros(m, n, m)
    W = W0
    q = torch.zeros((m, n), dtype=torch.float64, requires_grad=True)   # rotated-coordinate weights
    opt = torch.optim.Adam([q], lr=hp.lr * hp.alpha, betas=(hp.beta1, hp.beta2), eps=0.0)
    for _ in range(6):
        G = rng.standard_normal((m, n))
        out = o.fira_step(W, G, P, st, hp)
        W = out["W"]
        assert np.linalg.norm(out["E"]) <= 1e-14 * np.linalg.norm(G)
        q.grad = torch.tensor(P.T @ G)
        opt.step()
        np.testing.assert_allclose(W, W0 + P @ q.detach().numpy(), rtol=1e-10, atol=1e-12)


def pin_orthonormal_split(o):
    """Orthonormal P: P^T (G - P R) = 0, so projecting the weight delta recovers both halves of
    the update: P^T dW/(eta alpha) = -N and (I - P P^T) dW/(eta alpha) = -S (Alg. 1, last lines)."""
    rng = np.random.default_rng(5)
    for (m, n, r) in [(8, 12, 3), (12, 8, 3)]:
        left = m <= n
        P = _orth(rng, min(m, n), r)
        assert np.max(np.abs(P.T @ P - np.eye(r))) < 1e-12
        hp = _hp(o, lr=3e-3, alpha=0.25)
        st = o.OracleState.zeros(m, n, r)
        W = rng.standard_normal((m, n))
        for _ in range(5):
            G = rng.standard_normal((m, n))
            out = o.fira_step(W, G, P, st, hp)
            d = (out["W"] - W) / (hp.lr * hp.alpha)
            if left:
                np.testing.assert_allclose(P.T @ d, -out["N"], atol=1e-10)
                np.testing.assert_allclose(d - P @ (P.T @ d), -out["S"], atol=1e-10)
                np.testing.assert_allclose(out["R"], P.T @ G, atol=1e-13)
            else:
                np.testing.assert_allclose(d @ P, -out["N"], atol=1e-10)
                np.testing.assert_allclose(d - (d @ P) @ P.T, -out["S"], atol=1e-10)
                np.testing.assert_allclose(out["R"], G @ P, atol=1e-13)   # Sec. 3.3 footnote
            W = out["W"]


def pin_limiter_bound(o):
    """Norm-growth limiter (Eq. 12 / Alg. 1): after the first step the kept norm never exceeds
    gamma (||S_{t-1}|| + eps); it equals it when the raw ratio exceeds gamma; S is untouched
    (factor exactly 1) otherwise; the norm may fall freely."""
    rng = np.random.default_rng(6)
    m, n, r = 10, 14, 3
    P = _orth(rng, m, r)
    hp = _hp(o)
    st = o.OracleState.zeros(m, n, r)
    W = rng.standard_normal((m, n))
    scales = [1, 1, 30, 1, 1, 0.01, 1, 1, 5, 5, 5, 5]
    saw_limit = saw_free = saw_fall = False
    for i, sc in enumerate(scales):
        G = sc * rng.standard_normal((m, n))
        prev = st.s_prev
        out = o.fira_step(W, G, P, st, hp)
        W = out["W"]
        s_kept = float(np.linalg.norm(out["S"]))
        np.testing.assert_allclose(s_kept, out["s_post"], rtol=1e-12)
        np.testing.assert_allclose(st.s_prev, out["s_post"], rtol=0)
        if i == 0:
            assert out["c"] == 1.0
            continue
        bound = hp.gamma * (prev + hp.eps)
        assert s_kept <= bound * (1 + 1e-12)
        if out["s_pre"] / (prev + hp.eps) > hp.gamma:
            np.testing.assert_allclose(s_kept, bound, rtol=1e-12)
            saw_limit = True
        else:
            assert out["c"] == 1.0
            saw_free = True
            saw_fall |= s_kept < 0.5 * prev
    assert saw_limit and saw_free and saw_fall


def pin_first_step_and_constant_gradient(o):
    """Closed forms of Eqs. 2-4: at t = 1, N = R / (|R| + eps / sqrt(1 - beta2)); if R is the same
    for steps 1..t then M_t = (1 - beta1^t) R, V_t = (1 - beta2^t) R^2 and
    N_t = R / (|R| + eps / sqrt(1 - beta2^t))."""
    rng = np.random.default_rng(7)
    m, n, r = 9, 11, 4
    P = _orth(rng, m, r)
    G = rng.standard_normal((m, n))
    R = P.T @ G
    hp = _hp(o, eps=1e-3)   # large eps so that its placement matters
    st = o.OracleState.zeros(m, n, r)
    W = np.zeros((m, n))
    for t in range(1, 8):
        out = o.fira_step(W, G, P, st, hp)
        W = out["W"]
        np.testing.assert_allclose(st.M, (1 - hp.beta1 ** t) * R, rtol=1e-12)
        np.testing.assert_allclose(st.V, (1 - hp.beta2 ** t) * R * R, rtol=1e-12)
        np.testing.assert_allclose(
            out["N"], R / (np.abs(R) + hp.eps / math.sqrt(1 - hp.beta2 ** t)), rtol=1e-11)
        assert st.t == t
    # eps -> 0: N = sign(R), ||N[:, i]|| = sqrt(r), k_i = sqrt(r) / ||R[:, i]||
    st = o.OracleState.zeros(m, n, r)
    out = o.fira_step(np.zeros((m, n)), G, P, st, _hp(o, eps=0.0))
    np.testing.assert_allclose(out["N"], np.sign(R), rtol=1e-12)
    np.testing.assert_allclose(out["k"], math.sqrt(r) / np.linalg.norm(R, axis=0), rtol=1e-12)


def pin_scale_invariance(o):
    """eps = 0: multiplying every gradient by 2^k leaves the W trajectory bit-identical
    (M and sqrt(V) scale exactly, N is unchanged, k_i scales by 2^-k, the residual by 2^k)."""
    rng = np.random.default_rng(8)
    m, n, r = 7, 10, 3
    P = _orth(rng, m, r)
    W0 = rng.standard_normal((m, n))
    Gs = [rng.standard_normal((m, n)) for _ in range(6)]
    hp = _hp(o, eps=0.0)
    res = []
    for k in (0, 5, -7):
        W, _, _ = o.run(W0, [g * 2.0 ** k for g in Gs], lambda i: P, hp, r)
        res.append(W)
    assert np.array_equal(res[0], res[1]) and np.array_equal(res[0], res[2])


def pin_permutation_equivariance(o):
    """Permuting the columns of (W, G) (m <= n) permutes the result's columns."""
    rng = np.random.default_rng(9)
    m, n, r = 6, 9, 2
    P = _orth(rng, m, r)
    W0 = rng.standard_normal((m, n))
    Gs = [rng.standard_normal((m, n)) for _ in range(5)]
    perm = rng.permutation(n)
    hp = _hp(o)
    Wa, _, _ = o.run(W0, Gs, lambda i: P, hp, r)
    Wb, _, _ = o.run(W0[:, perm], [g[:, perm] for g in Gs], lambda i: P, hp, r)
    np.testing.assert_allclose(Wa[:, perm], Wb, rtol=1e-12, atol=1e-14)


def pin_norm_identity(o):
    """sum_i k_i^2 (||R[:, i]|| + eps)^2 = ||N||_F^2: ties the column factors (Eq. 11) to the
    matrix-level factor (Eq. 9)."""
    rng = np.random.default_rng(10)
    m, n, r = 8, 13, 4
    P = _orth(rng, m, r)
    hp = _hp(o)
    st = o.OracleState.zeros(m, n, r)
    W = np.zeros((m, n))
    for _ in range(4):
        G = rng.standard_normal((m, n))
        out = o.fira_step(W, G, P, st, hp)
        W = out["W"]
        lhs = np.sum(out["k"] ** 2 * (np.linalg.norm(out["R"], axis=0) + hp.eps) ** 2)
        np.testing.assert_allclose(lhs, np.sum(out["N"] ** 2), rtol=1e-12)
        # matrix-level variant: a single factor ||N|| / (||R|| + eps) for every column
        st2 = o.OracleState.zeros(m, n, r)
        out2 = o.fira_step(np.zeros((m, n)), G, P, st2, hp, scaling="matrix")
        np.testing.assert_allclose(
            out2["k"], np.linalg.norm(P.T @ G / (np.abs(P.T @ G) + hp.eps / math.sqrt(1 - hp.beta2)))
            / (np.linalg.norm(P.T @ G) + hp.eps), rtol=1e-10)


def pin_transpose(o):
    """m > n is the m <= n algorithm on the transposed problem: step(G, W, Q) == step(G^T, W^T, Q)^T,
    with one factor per row of G."""
    rng = np.random.default_rng(12)
    m, n, r = 11, 6, 2
    Q = _orth(rng, n, r)
    W0 = rng.standard_normal((m, n))
    Gs = [rng.standard_normal((m, n)) * (1 + 4 * (i == 3)) for i in range(6)]
    hp = _hp(o)
    Wa, sta, tra = o.run(W0, Gs, lambda i: Q, hp, r)
    Wb, stb, trb = o.run(W0.T, [g.T for g in Gs], lambda i: Q, hp, r)
    np.testing.assert_allclose(Wa, Wb.T, rtol=1e-13, atol=1e-15)
    assert sta.M.shape == (m, r) and stb.M.shape == (r, m)
    np.testing.assert_allclose(sta.M, stb.M.T, rtol=1e-13)
    assert tra[0]["k"].shape == (m,)
    np.testing.assert_allclose(
        tra[0]["k"], np.linalg.norm(tra[0]["N"], axis=1) / (np.linalg.norm(Gs[0] @ Q, axis=1) + hp.eps),
        rtol=1e-12)
    # square matrices take the m <= n branch (P multiplies from the left)
    Pq = _orth(rng, 5, 2)
    G = rng.standard_normal((5, 5))
    out = o.fira_step(np.zeros((5, 5)), G, Pq, o.OracleState.zeros(5, 5, 2), hp)
    np.testing.assert_allclose(out["R"], Pq.T @ G, atol=1e-14)


def pin_gradient_in_subspace_and_switches(o):
    """G = P A lies in the subspace: the residual vanishes and the step is GaLore's (Eq. 6).
    gamma = inf removes the limiter (the "w.o.-limiter" variant); scaling "none" gives the
    GaLore-add update (Eq. 8)."""
    rng = np.random.default_rng(13)
    m, n, r = 8, 10, 3
    P = _orth(rng, m, r)
    hp = _hp(o, alpha=0.25)
    A = rng.standard_normal((r, n))
    st = o.OracleState.zeros(m, n, r)
    W0 = rng.standard_normal((m, n))
    out = o.fira_step(W0, P @ A, P, st, hp)
    assert np.linalg.norm(out["E"]) < 1e-14 * np.linalg.norm(A)
    np.testing.assert_allclose(out["W"], W0 - hp.lr * hp.alpha * (P @ out["N"]), atol=1e-15)
    np.testing.assert_allclose(out["N"], A / (np.abs(A) + hp.eps / math.sqrt(1 - hp.beta2)), rtol=1e-9)
    # switches
    Gs = [rng.standard_normal((m, n)) * (1 + 9 * (i == 2)) for i in range(4)]
    hp_inf = _hp(o, gamma=float("inf"))
    W, st, tr = o.run(W0, Gs, lambda i: P, hp_inf, r)
    assert all(t["c"] == 1.0 for t in tr)
    np.testing.assert_allclose(tr[2]["s_post"], tr[2]["s_pre"])
    W, st, tr = o.run(W0, Gs[:1], lambda i: P, hp_inf, r, scaling="none")
    R = P.T @ Gs[0]
    np.testing.assert_allclose(
        W, W0 - hp_inf.lr * (P @ tr[0]["N"] + (Gs[0] - P @ R)), rtol=1e-12, atol=1e-15)


def pin_degenerate_columns(o):
    """Zero columns follow the formulas literally (no NaN): an all-zero column history gives
    N = 0/(0+eps) = 0 and k = 0; a zero column of R with non-zero moments gives k = ||N||/eps."""
    m, n, r = 4, 5, 2
    P = np.eye(m)[:, :r]
    rng = np.random.default_rng(14)
    hp = _hp(o)
    G1 = rng.standard_normal((m, n))
    G1[:, 0] = 0.0
    st = o.OracleState.zeros(m, n, r)
    out = o.fira_step(np.zeros((m, n)), G1, P, st, hp)
    assert np.all(np.isfinite(out["W"])) and out["k"][0] == 0.0 and np.all(out["N"][:, 0] == 0.0)
    G2 = rng.standard_normal((m, n))
    G2[:r, 1] = 0.0   # column 1 of R is zero now, but its moments are not
    out = o.fira_step(out["W"], G2, P, st, hp)
    assert np.all(np.isfinite(out["W"]))
    np.testing.assert_allclose(out["k"][1], np.linalg.norm(out["N"][:, 1]) / hp.eps, rtol=1e-12)
    assert out["k"][1] > 1e6
    # P = I_m: the residual is exactly zero, s = 0, and later steps stay finite
    st = o.OracleState.zeros(m, n, m)
    W = np.zeros((m, n))
    for _ in range(3):
        out = o.fira_step(W, rng.standard_normal((m, n)), np.eye(m), st, hp)
        W = out["W"]
        assert out["s_pre"] == 0.0 and out["c"] == 1.0 and st.s_prev == 0.0


def pin_projector_switch_keeps_state(o):
    """Switching P keeps M, V, t and the remembered norm (Sec. 4.2, loss-spike analysis): a run
    with a switch at step 3 equals continuing the first run's state with the new projector."""
    rng = np.random.default_rng(15)
    m, n, r = 7, 9, 3
    P1, P2 = _orth(rng, m, r), _orth(rng, m, r)
    W0 = rng.standard_normal((m, n))
    Gs = [rng.standard_normal((m, n)) for _ in range(6)]
    hp = _hp(o)
    Wa, sta, _ = o.run(W0, Gs, lambda i: P1 if i < 3 else P2, hp, r)
    Wm, stm, _ = o.run(W0, Gs[:3], lambda i: P1, hp, r)
    M3 = stm.M.copy()
    Wb, stb, trb = o.run(Wm, Gs[3:], lambda i: P2, hp, r, state=stm)
    assert np.array_equal(Wa, Wb) and stb.t == 6
    # first step after the switch uses the old moments: M_4 = beta1 M_3 + (1-beta1) P2^T G_4
    st_chk = o.OracleState.zeros(m, n, r)
    o.run(W0, Gs[:4], lambda i: P1 if i < 3 else P2, hp, r, state=st_chk)
    np.testing.assert_allclose(st_chk.M, hp.beta1 * M3 + (1 - hp.beta1) * (P2.T @ Gs[3]), rtol=1e-12)


def pin_bf16_rounding(o):
    """Storage-format model: round_to_bf16 keeps 8 significant bits with ties to even, and agrees
    with torch's float32 -> bfloat16 conversion (library routine) on float32 inputs."""
    import torch
    f = o.round_to_bf16
    assert f(np.array([1.0 + 2.0 ** -8]))[0] == 1.0            # tie -> even (1.0)
    assert f(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6   # tie -> even (1.015625)
    assert f(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]))[0] == 1.0 + 2.0 ** -7
    x = np.random.default_rng(16).standard_normal(4096).astype(np.float32) * 0.02
    ref = torch.tensor(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(f(x.astype(np.float64)), ref)
    # a step with store_bf16 returns representable weights and the unrounded ones beside them
    rng = np.random.default_rng(17)
    P = _orth(rng, 4, 2)
    out = o.fira_step(f(rng.standard_normal((4, 6))), rng.standard_normal((4, 6)), P,
                      o.OracleState.zeros(4, 6, 2), _hp(o), store_bf16=True)
    assert np.array_equal(f(out["W"]), out["W"])
    assert np.max(np.abs(out["W"] - out["W_unrounded"])) <= 2.0 ** -8 * np.max(np.abs(out["W"]))


def pin_only_scaling_variant(o):
    """Appendix variant "Fira-only-scaling": W_{t+1} = W_t - eta phi_t(R_t) G_t.  With the limiter off
    and alpha = 1 the weight delta of one step is exactly -lr * G * k (k from the same R, N as the
    full method), column by column; the Adam state advances as in the full method; and the variant
    differs from the full method by lr * (P N - k (P R)) when P is orthonormal."""
    rng = np.random.default_rng(41)
    m, n, r = 5, 8, 2
    P = _orth(rng, m, r)
    hp = _hp(o, gamma=float("inf"), alpha=1.0)
    W0 = rng.standard_normal((m, n))
    st_a, st_b = o.OracleState.zeros(m, n, r), o.OracleState.zeros(m, n, r)
    for t in range(3):
        G = rng.standard_normal((m, n))
        full = o.fira_step(W0, G, P, st_a, hp)
        only = o.fira_step(W0, G, P, st_b, hp, variant="only_scaling")
        np.testing.assert_allclose(only["k"], full["k"], rtol=1e-13)
        np.testing.assert_allclose(W0 - only["W"], hp.lr * G * full["k"][None, :], rtol=1e-9, atol=1e-15)
        np.testing.assert_allclose(only["W"] - full["W"],
                                   hp.lr * (P @ full["N"] - (P @ full["R"]) * full["k"][None, :]), rtol=1e-9, atol=1e-15)
        np.testing.assert_allclose(st_a.M, st_b.M, rtol=0, atol=0)
    # transposed problem and the limiter: the norm that is limited is ||k G||
    hp2 = _hp(o, alpha=1.0)
    Gt = rng.standard_normal((n, m))
    st_c = o.OracleState.zeros(n, m, r)
    o1 = o.fira_step(np.zeros((n, m)), Gt, P, st_c, hp2, variant="only_scaling")
    np.testing.assert_allclose(o1["s_pre"], np.linalg.norm(Gt * o1["k"][:, None]), rtol=1e-13)
    o2 = o.fira_step(np.zeros((n, m)), 7.0 * Gt + rng.standard_normal((n, m)), P, st_c, hp2, variant="only_scaling")
    assert o2["c"] <= 1.0 and o2["s_post"] <= hp2.gamma * (o1["s_post"] + hp2.eps) * (1 + 1e-12)


def pin_projector_refresh_helpers(o):
    """Eq. 7 and the subspace measures used to judge a refreshed projector.
    * a matrix of exact rank r: the projector spans its column (row) space and keeps all its energy;
    * known singular vectors: G = U diag(s) V^T with a decreasing s gives back U[:, :r] (V[:, :r] for
      m > n) up to sign, and the kept energy is sum(s[:r]^2) / sum(s^2) (Eckart-Young);
    * principal angles: equal spans -> 0 whatever the bases; orthogonal spans -> 1; a plane rotated
      by theta against another about a common axis -> (sin theta, 0)."""
    rng = np.random.default_rng(31)
    for (m, n) in ((9, 14), (14, 9)):
        r = 3
        S = min(m, n)
        U = _orth(rng, m, S); V = _orth(rng, n, S)
        s = np.array([5.0, 4.0, 3.0, 0.5, 0.4, 0.3, 0.2, 0.1, 0.05])[:S]
        G = (U * s) @ V.T
        P = o.top_r_projector(G, r)
        assert P.shape == (S, r)
        ref = U[:, :r] if m <= n else V[:, :r]
        np.testing.assert_allclose(np.abs(ref.T @ P), np.eye(r), atol=1e-10)      # same vectors up to sign
        assert np.max(o.subspace_sines(P, ref)) < 1e-10
        np.testing.assert_allclose(o.captured_energy(G, P), np.sum(s[:r] ** 2) / np.sum(s ** 2), rtol=1e-12)
        # any other r-dimensional subspace keeps less
        other = _orth(rng, S, r)
        assert o.captured_energy(G, other) < o.captured_energy(G, P)
        # exact rank r: all the energy, and the span is the column/row space
        G0 = (U[:, :r] * s[:r]) @ V[:, :r].T
        P0 = o.top_r_projector(G0, r)
        np.testing.assert_allclose(o.captured_energy(G0, P0), 1.0, rtol=1e-12)
        assert np.max(o.subspace_sines(P0, ref)) < 1e-9
    # principal angles
    B = _orth(rng, 7, 7)
    A1 = B[:, :2]
    Rm = np.array([[2.0, 1.0], [-1.0, 3.0]])
    assert np.max(o.subspace_sines(A1, A1 @ Rm)) < 1e-12                      # basis change
    np.testing.assert_allclose(o.subspace_sines(A1, B[:, 2:4]), [1.0, 1.0], atol=1e-12)
    th = 0.3
    A2 = np.stack([B[:, 0], np.cos(th) * B[:, 1] + np.sin(th) * B[:, 2]], axis=1)
    np.testing.assert_allclose(np.sort(o.subspace_sines(A1, A2)), [0.0, np.sin(th)], atol=1e-12)


PINS = [pin_hand_case, pin_brute_force, pin_full_rank_identity_is_adam, pin_full_rank_rotation,
        pin_orthonormal_split, pin_limiter_bound, pin_first_step_and_constant_gradient,
        pin_scale_invariance, pin_permutation_equivariance, pin_norm_identity, pin_transpose,
        pin_gradient_in_subspace_and_switches, pin_degenerate_columns,
        pin_projector_switch_keeps_state, pin_bf16_rounding, pin_projector_refresh_helpers,
        pin_only_scaling_variant]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(ORC)


# ------------------------------------------------------------------------------------------
# planted mistakes: every mutant of the oracle source must be caught by at least one pin
# ------------------------------------------------------------------------------------------

MUTANTS = [
    ("residual sign", "E = G - P @ R", "E = G + P @ R"),
    ("first-moment weight dropped", "(1.0 - beta1) * R", "R"),
    ("second-moment uses R not R^2", "(1.0 - beta2) * (R * R)", "(1.0 - beta2) * R"),
    ("bias correction one step late", "1.0 - beta2 ** t) / (1.0 - beta1 ** t)",
     "1.0 - beta2 ** (t - 1)) / (1.0 - beta1 ** t)"),
    ("bias correction inverted", "np.sqrt(1.0 - beta2 ** t) / (1.0 - beta1 ** t)",
     "(1.0 - beta1 ** t) / np.sqrt(1.0 - beta2 ** t)"),
    ("eps inside the square root", "(np.sqrt(V) + eps)", "np.sqrt(V + eps)"),
    ("column factor inverted", "np.sqrt(np.sum(N * N, axis=0)) / (np.sqrt(np.sum(R * R, axis=0)) + eps)",
     "np.sqrt(np.sum(R * R, axis=0)) / (np.sqrt(np.sum(N * N, axis=0)) + eps)"),
    ("column factor without eps", "(np.sqrt(np.sum(R * R, axis=0)) + eps)", "np.sqrt(np.sum(R * R, axis=0))"),
    ("column factor along the wrong axis", "np.sum(N * N, axis=0)", "np.sum(N * N, axis=1)"),
    ("squared norms in the factor", "return np.sqrt(np.sum(N * N, axis=0)) / (np.sqrt(np.sum(R * R, axis=0)) + eps)",
     "return np.sum(N * N, axis=0) / (np.sum(R * R, axis=0) + eps)"),
    ("limiter compares with 1 instead of gamma", "max(ratio, gamma)", "max(ratio, 1.0)"),
    ("limiter without eps", "den = s_prev + eps", "den = s_prev"),
    ("limiter remembers the raw norm", "s_post = c * s_pre", "s_post = s_pre"),
    ("limiter applied on the first step", "if s_prev is None or np.isinf(gamma):", "if np.isinf(gamma):"),
    ("scaled residual not limited", "S = c * S", "S = 1.0 * S"),
    ("residual subtracted", "(P @ N + S)", "(P @ N - S)"),
    ("low-rank part not projected back", "(P @ N + S)", "(P @ R + S)"),
    ("alpha dropped", "G_tilde = hp.alpha * (", "G_tilde = ("),
    ("ascent instead of descent", "W_new = W - hp.lr * G_tilde", "W_new = W + hp.lr * G_tilde"),
    ("projection not transposed", "R = P.T @ G ", "R = P[:G.shape[0], :].T[:, :G.shape[0]] @ G * 0 + (P.T @ G)[::-1] "),
    ("step counter not advanced", "st.M, st.V, st.s_prev, st.t = M, V, s_post, t", "st.M, st.V, st.s_prev, st.t = M, V, s_post, st.t"),
    ("moments not stored", "st.M, st.V, st.s_prev, st.t = M, V, s_post, t", "st.s_prev, st.t = s_post, t"),
    ("m > n handled as m <= n", "    if m <= n:\n        out = _step_short_rows", "    if True:\n        out = _step_short_rows"),
    ("bf16 rounding truncates", "np.rint(mant * 256.0)", "np.trunc(mant * 256.0)"),
    ("bf16 keeps 9 bits", "np.rint(mant * 256.0) / 256.0", "np.rint(mant * 512.0) / 512.0"),
    ("only-scaling keeps the residual", "        S = G * k[None, :]                       # W_{t+1}", "        S = E * k[None, :]                       # W_{t+1}"),
    ("only-scaling keeps the Adam term", "        G_tilde = hp.alpha * S                   # no Adam term", "        G_tilde = hp.alpha * (P @ N + S)         # no Adam term"),
    ("refresh takes the trailing vectors", "return U[:, :r] if G.shape[0] <= G.shape[1] else Vt[:r, :].T",
     "return U[:, -r:] if G.shape[0] <= G.shape[1] else Vt[-r:, :].T"),
    ("refresh takes the wrong side", "return U[:, :r] if G.shape[0] <= G.shape[1] else Vt[:r, :].T",
     "return U[:, :r] if G.shape[0] > G.shape[1] else Vt[:r, :].T"),
    ("principal angles return cosines", "return np.linalg.svd(Qq - Pq @ (Pq.T @ Qq), compute_uv=False)",
     "return np.linalg.svd(Pq.T @ Qq, compute_uv=False)"),
    ("kept energy not normalised", "return float(np.sum(R * R) / np.sum(G * G))", "return float(np.sum(R * R))"),
]


def _load_mutant(old, new):
    path = ORC.__file__
    src = open(path).read()
    assert src.count(old) >= 1, f"mutation target not found: {old!r}"
    mod = types.ModuleType("oracle_mutant")
    mod.__file__ = path
    sys.modules["oracle_mutant"] = mod   # dataclasses look the module up by name
    exec(compile(src.replace(old, new), path, "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutants_are_caught(name, old, new):
    mod = _load_mutant(old, new)
    caught = []
    with np.errstate(all="ignore"):
        for pin in PINS:
            try:
                pin(mod)
            except Exception as e:   # assertion or any crash both count as detection
                caught.append(pin.__name__)
    assert caught, f"planted mistake '{name}' passed every pin"
