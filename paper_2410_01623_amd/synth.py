"""Seeded synthetic inputs for the Fira optimizer step (weights, gradients, projectors).

This module only *draws inputs*: shapes, random values, storage-format rounding of those
values, and the projector that the step receives as an argument.  It contains none of the
method's arithmetic (no Adam, no scaling factors, no limiter, no weight update) and is the one
module that both the CPU oracle's tests and the GPU path's tests/bench may use, so that both
sides see the same bytes.

The paper trains LLaMA models on C4 (Sec. 5.1, Table "Hyper-parameters of LLaMA architectures");
neither the data nor the models exist here.  The gradients below only borrow the *layer shapes*
of that table and stand in for real gradients.

numpy only; no torch import, no GPU.
"""
from __future__ import annotations

import dataclasses
from typing import List, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------------------
# storage-format helpers (bf16 <-> fp32), used to make inputs exactly representable
# --------------------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of bf16 bit patterns, round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) >> 16
    return u.astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def as_bf16_values(x: np.ndarray) -> np.ndarray:
    """Round a float array to the nearest bf16 value, returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(np.asarray(x, dtype=np.float32)))


# --------------------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------------------


@dataclasses.dataclass(frozen=True)
class Hparams:
    """Hyper-parameters of Algorithm 1's input line: eta, beta1, beta2, eps, alpha, gamma."""

    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    alpha: float = 1.0
    gamma: float = 1.01


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark/parity configuration: a list of weight-matrix shapes plus a gradient recipe."""

    name: str
    config_id: int
    blocks: int
    block_shapes: Tuple[Tuple[int, int], ...]  # (m, n) of each matrix in one block
    rank: int
    dtype: str  # "f32" or "bf16": storage type of W and G
    grad: str  # "gauss", "colscale", "student_t"
    grad_scale: float
    steps: int
    spike_step: int = -1  # step index whose gradient is multiplied by spike_factor
    spike_factor: float = 1.0
    refresh_every: int = 0  # projector refresh period T (0 = never after the first)
    hp: Hparams = Hparams()

    @property
    def shapes(self) -> List[Tuple[int, int]]:
        return [s for _ in range(self.blocks) for s in self.block_shapes]

    @property
    def n_matrices(self) -> int:
        return self.blocks * len(self.block_shapes)


def _llama_block(d: int, f: int) -> Tuple[Tuple[int, int], ...]:
    # q, k, v, o: d x d; gate, up: d x f; down: f x d
    return ((d, d), (d, d), (d, d), (d, d), (d, f), (d, f), (f, d))


WORKLOADS = {
    "single_256x688_r64_f32": Workload(
        "single_256x688_r64_f32", 1, 1, ((256, 688),), 64, "f32", "gauss", 0.02, 10),
    "llama60m_r128_bf16": Workload(
        "llama60m_r128_bf16", 2, 8, _llama_block(512, 1376), 128, "bf16", "colscale", 1e-3, 100,
        refresh_every=50),
    "llama350m_r256_bf16": Workload(
        "llama350m_r256_bf16", 3, 24, _llama_block(1024, 2736), 256, "bf16", "student_t", 1e-3, 60,
        spike_step=40, spike_factor=20.0),
    "llama1b_r512_bf16": Workload(
        "llama1b_r512_bf16", 4, 24, _llama_block(2048, 5461), 512, "bf16", "gauss", 1e-3, 10),
    "llama7b_r1024_bf16": Workload(
        "llama7b_r1024_bf16", 5, 32, _llama_block(4096, 11008), 1024, "bf16", "gauss", 1e-3, 3),
    # Fine-tuning shape set (Appendix "Detailed Fine-Tuning Setting": rank 32 on Q, K, V, Up, Down of a
    # 4096-wide model): a very skinny R, the step is almost pure streaming of G and W.
    "llama7b_finetune_r32_bf16": Workload(
        "llama7b_finetune_r32_bf16", 6, 32, ((4096, 4096), (4096, 4096), (4096, 4096), (4096, 11008), (11008, 4096)),
        32, "bf16", "gauss", 1e-3, 3),
}
HEADLINE = "llama1b_r512_bf16"


def _rng(config_id: int, stream: int, mat: int) -> np.random.Generator:
    """Counter-based generator: one independent Philox stream per (config, purpose/step, matrix)."""
    return np.random.Generator(np.random.Philox(key=[1000 * config_id + stream, mat]))


_W_STREAM = 7  # weights use stream 7; gradients use stream 100 + step
_COL_STREAM = 8  # per-column scales of the "colscale" recipe
_P_STREAM = 9  # random orthonormal projectors


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = x.astype(np.float32)
    return as_bf16_values(x) if dtype == "bf16" else x


def gen_W(wl: Workload, mat: int, shape: Tuple[int, int] | None = None) -> np.ndarray:
    """Initial weights W ~ N(0, 0.02^2), float32 values representable in the workload's dtype."""
    m, n = shape or wl.shapes[mat]
    g = _rng(wl.config_id, _W_STREAM, mat)
    return _store(0.02 * g.standard_normal((m, n), dtype=np.float32), wl.dtype)


def gen_G(wl: Workload, mat: int, step: int, shape: Tuple[int, int] | None = None) -> np.ndarray:
    """Gradient of matrix `mat` at 0-based `step`, float32 values representable in the dtype."""
    m, n = shape or wl.shapes[mat]
    g = _rng(wl.config_id, 100 + step, mat)
    if wl.grad == "gauss":
        x = g.standard_normal((m, n), dtype=np.float32)
    elif wl.grad == "colscale":
        x = g.standard_normal((m, n), dtype=np.float32)
        u = _rng(wl.config_id, _COL_STREAM, mat).uniform(-1.0, 1.0, size=n)
        x = x * (10.0 ** u).astype(np.float32)[None, :]
    elif wl.grad == "student_t":
        x = g.standard_t(3.0, size=(m, n)).astype(np.float32)
    else:
        raise ValueError(wl.grad)
    x = np.float32(wl.grad_scale) * x
    if step == wl.spike_step:
        x = np.float32(wl.spike_factor) * x
    return _store(x, wl.dtype)


# --------------------------------------------------------------------------------------
# projectors (the step takes P as an argument; building it is the caller's business)
# --------------------------------------------------------------------------------------


def projector_from_gradient(G: np.ndarray, r: int) -> np.ndarray:
    """Top-r singular vectors of G on its short side (Eq. 7): left vectors (m x r) when m <= n,
    right vectors (n x r) when m > n.  Computed in fp64 through the Gram matrix of the short side,
    returned as fp64; the caller rounds to the storage type."""
    G = np.asarray(G, dtype=np.float64)
    m, n = G.shape
    gram = G @ G.T if m <= n else G.T @ G
    w, U = np.linalg.eigh(gram)  # ascending
    P = U[:, ::-1][:, :r]
    # re-orthonormalise (eigh is already orthonormal to ~1e-15; QR fixes the sign convention)
    Q, Rr = np.linalg.qr(P)
    Q = Q * np.sign(np.diag(Rr))[None, :]
    return np.ascontiguousarray(Q)


def random_orthonormal_projector(wl: Workload, mat: int, short: int, r: int) -> np.ndarray:
    """A seeded orthonormal basis (short x r) of a random r-dimensional subspace, fp64."""
    g = _rng(wl.config_id, _P_STREAM, mat)
    Q, Rr = np.linalg.qr(g.standard_normal((short, r)))
    return np.ascontiguousarray(Q * np.sign(np.diag(Rr))[None, :])


def store_projector(P: np.ndarray, dtype: str) -> np.ndarray:
    """Round a projector to the storage type the library is given (float32 values)."""
    return _store(np.asarray(P), dtype)


def shapes_of(wl: Workload, mats: Sequence[int]) -> List[Tuple[int, int]]:
    s = wl.shapes
    return [s[i] for i in mats]
