"""Why long bf16 runs drift from the oracle by more than one step's rounding, shown on the CPU.

The library computes the update as W -= lr alpha (P Z + c k G) with Z = N - c k R rounded to bf16 as an MFMA
operand, and stores W in bf16 (nearest even).  This file emulates exactly that arithmetic in numpy (fp32 where
the kernels use fp32, exact products accumulated in fp32, bf16 roundings where the kernels round) next to the
fp64 oracle, for three forms of the operand: one bf16 plane, two planes (hi + lo, fira_set_z_planes(2)) and the
unrounded fp32 Z.  An element of W whose per-step update sits next to half an ulp of its bf16 value moves or
stays depending on the last bits of the update, so a 2^-9 perturbation of P Z lets single elements walk away
from the oracle by one ulp per step; with 16 mantissa bits in Z they do not.  The GPU tests hold long runs to
3x the gate with one plane and to the gate itself with two; this is the arithmetic behind those two numbers."""
import numpy as np

from oracle import fira_oracle as orc
from paper_2410_01623_amd import synth


def _bf(x):
    return synth.as_bf16_values(np.asarray(x, dtype=np.float32)).astype(np.float32)


def _emulate(mode, m, n, r, steps, seed):
    rng = np.random.default_rng(seed)
    hp = orc.OracleHparams()
    W0 = _bf(0.02 * rng.standard_normal((m, n)))
    scale = 10.0 ** rng.uniform(-1.0, 1.0, n)          # per-column gradient scales, as in the 60M-shaped workload
    M = np.zeros((r, n), np.float32)
    V = np.zeros((r, n), np.float32)
    s_prev = None
    Wg = W0.copy()
    st = orc.OracleState.zeros(m, n, r)
    Wr = W0.astype(np.float64)
    worst = 0.0
    for s in range(steps):
        G = _bf(1e-3 * rng.standard_normal((m, n)) * scale[None, :])
        if s == 0:
            P = synth.store_projector(synth.projector_from_gradient(G, r), "bf16")
        Pd, Gd = P.astype(np.float64), G.astype(np.float64)
        Wr = orc.fira_step(Wr, Gd, Pd, st, hp, store_bf16=True)["W"]
        t = s + 1
        R = (Pd.T @ Gd).astype(np.float32)               # exact products, fp32 accumulators
        M = np.float32(hp.beta1) * M + np.float32(1.0 - hp.beta1) * R
        V = np.float32(hp.beta2) * V + np.float32(1.0 - hp.beta2) * (R * R)
        bias = np.float32(np.sqrt(1.0 - hp.beta2 ** t) / (1.0 - hp.beta1 ** t))
        N = bias * (M / (np.sqrt(V) + np.float32(hp.eps)))
        k = np.sqrt((N * N).sum(0)) / (np.sqrt((R * R).sum(0)) + np.float32(hp.eps))
        E = Gd - Pd @ _bf(R).astype(np.float64)          # residual route: R as a bf16 operand
        sn = float(np.sqrt(((E * k[None, :]) ** 2).sum()))
        c = 1.0 if s_prev is None else hp.gamma / max(sn / (s_prev + hp.eps), hp.gamma)
        s_prev = c * sn
        Z = N - np.float32(c) * k[None, :] * R           # fp32, from the unrounded N and R
        if mode == "one_plane":
            Zop = _bf(Z).astype(np.float64)
        elif mode == "two_planes":
            hi = _bf(Z)
            Zop = hi.astype(np.float64) + _bf(Z - hi).astype(np.float64)
        else:
            Zop = Z.astype(np.float64)
        U = (Pd @ Zop).astype(np.float32)
        Wg = _bf(Wg - np.float32(hp.lr * hp.alpha) * (U + np.float32(c) * k[None, :] * G))
        worst = max(worst, float(np.abs(Wg.astype(np.float64) - Wr).max() / np.abs(Wr).max()))
    return float(np.abs(Wg.astype(np.float64) - Wr).max() / np.abs(Wr).max()), worst


def test_one_bf16_plane_of_z_drifts_and_two_planes_do_not():
    m, n, r, steps = 128, 344, 32, 100
    one, _ = _emulate("one_plane", m, n, r, steps, seed=3)
    two, _ = _emulate("two_planes", m, n, r, steps, seed=3)
    exact, _ = _emulate("exact", m, n, r, steps, seed=3)
    print(f"W error after {steps} steps, relative to max |W|: one plane {one:.4f}, two planes {two:.4f}, fp32 Z {exact:.4f}")
    # an ulp of the largest weights is 2^-8 = 0.0039 of them: the two-plane and exact forms stay within a
    # couple of ulps, the one-plane form walks several ulps away
    assert two <= 1.5 * exact + 1e-3
    assert two <= 2e-2 / 2
    assert one >= 2.0 * two
