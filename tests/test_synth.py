"""Input generators: determinism, storage rounding, workload tables (no GPU)."""
import numpy as np
import torch

from paper_2410_01623_amd import synth


def test_bf16_helpers_match_library_conversion():
    x = (np.random.default_rng(0).standard_normal(10000) * 0.02).astype(np.float32)
    bits = synth.f32_to_bf16_bits(x)
    ref = torch.tensor(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(synth.bf16_bits_to_f32(bits), ref.to(torch.float32).numpy())
    v = synth.as_bf16_values(x)
    assert np.array_equal(synth.as_bf16_values(v), v)


def test_generators_are_seeded_and_distinct():
    wl = synth.WORKLOADS["llama60m_r128_bf16"]
    a = synth.gen_G(wl, 3, 5)
    b = synth.gen_G(wl, 3, 5)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, synth.gen_G(wl, 3, 6))
    assert not np.array_equal(a, synth.gen_G(wl, 2, 5))
    assert a.shape == (512, 512) and a.dtype == np.float32
    assert np.array_equal(synth.as_bf16_values(a), a)
    W = synth.gen_W(wl, 6)
    assert W.shape == (1376, 512) and abs(W.std() - 0.02) < 1e-3


def test_workload_tables():
    wl = synth.WORKLOADS[synth.HEADLINE]
    assert wl.n_matrices == 168 and wl.rank == 512
    assert sum(m * n for m, n in wl.shapes) == 24 * (4 * 2048 * 2048 + 3 * 2048 * 5461)
    w3 = synth.WORKLOADS["llama350m_r256_bf16"]
    g39 = synth.gen_G(w3, 0, 39, shape=(64, 96))
    g40 = synth.gen_G(w3, 0, 40, shape=(64, 96))
    assert np.abs(g40).mean() > 8 * np.abs(g39).mean()      # injected 20x spike
    w2 = synth.WORKLOADS["llama60m_r128_bf16"]
    g = synth.gen_G(w2, 4, 0)
    col = np.sqrt((g.astype(np.float64) ** 2).mean(axis=0)) / 1e-3
    assert col.min() > 0.07 and col.max() < 14 and col.max() / col.min() > 20   # log-uniform [0.1, 10]


def test_projectors_are_orthonormal_and_capture_top_subspace():
    rng = np.random.default_rng(1)
    U, _ = np.linalg.qr(rng.standard_normal((24, 24)))
    Vt, _ = np.linalg.qr(rng.standard_normal((40, 40)))
    s = np.concatenate([[10, 9, 8, 7], np.full(20, 0.1)])
    G = (U * s) @ Vt[:, :24].T
    P = synth.projector_from_gradient(G, 4)
    assert P.shape == (24, 4) and np.max(np.abs(P.T @ P - np.eye(4))) < 1e-12
    assert np.linalg.norm(P.T @ U[:, :4]) ** 2 > 4 - 1e-9        # same subspace as u_1..u_4 (Eq. 7)
    Q = synth.projector_from_gradient(G.T, 4)                     # m > n: right singular vectors
    assert Q.shape == (24, 4) and np.linalg.norm(Q.T @ U[:, :4]) ** 2 > 4 - 1e-9
    wl = synth.WORKLOADS[synth.HEADLINE]
    R = synth.random_orthonormal_projector(wl, 0, 64, 16)
    assert np.max(np.abs(R.T @ R - np.eye(16))) < 1e-12
