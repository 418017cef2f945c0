"""Run-to-run determinism of the HIP path at the headline shapes: the library uses no atomics and sums
partials in a fixed order, and its pipelined kernels order their own asynchronous loads with explicit
queue-depth waits.  A matrix that is fed the same inputs as another one (in its own buffers, at other
addresses, scheduled elsewhere on the chip) must therefore stay bit-identical to it, step after step;
a wait that lets a kernel read a tile before it has landed shows up here as a divergence."""
import pytest
import torch

from paper_2410_01623_amd import fira, synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("norm_mode", [fira.FIRA_NORM_GRAM, fira.FIRA_NORM_RESIDUAL], ids=["gram", "residual"])
def test_twin_matrices_stay_bit_identical(norm_mode):
    wl = synth.WORKLOADS[synth.HEADLINE]
    shapes = wl.shapes
    n, nb = len(shapes), len(wl.block_shapes)
    steps = 150
    dev = "cuda:0"
    ctx = fira.FiraContext(shapes, wl.rank, fira.FIRA_BF16, device=dev)
    ctx.fira_set_options(scaling=fira.FIRA_SCALE_COLUMN, norm_mode=norm_mode)
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    P, W0 = {}, {}
    for j in range(nb):
        m, nn = shapes[j]
        # an orthonormal basis keeps the Gram route open; both routes run the same contractions
        q, _ = torch.linalg.qr(torch.randn((min(m, nn), wl.rank), device=dev, generator=gen))
        P[j] = q.to(torch.bfloat16).contiguous()
        W0[j] = (0.02 * torch.randn(shapes[j], device=dev, generator=gen)).to(torch.bfloat16)
    for i in range(n):
        ctx.fira_set_projector(i, P[i % nb])
    W = [W0[i % nb].clone() for i in range(n)]
    preps = []
    for _ in range(3):
        base = [(1e-3 * torch.randn(shapes[j], device=dev, generator=gen)).to(torch.bfloat16) for j in range(nb)]
        preps.append(ctx.prepare(list(range(n)), W, [base[i % nb].clone() for i in range(n)]))
    for s in range(steps):
        ctx.fira_step(prepared=preps[s % 3])
        bad = [i for i in range(nb, n) if not torch.equal(W[i], W[i % nb])]
        assert not bad, f"step {s}: matrices {bad[:8]} differ from their twins"
    assert all(bool(torch.isfinite(W[j]).all()) for j in range(nb))


def test_step_replays_from_a_hip_graph():
    """fira_step only enqueues kernels once its work list is cached and the projectors' gate values are in
    (from the second step after an installation on), so a training loop can capture it in a HIP graph.  Three replays with fresh gradients (copied into the
    captured buffers, with eager work and synchronisations in between) must give, bit for bit, what eager
    steps give on a twin context."""
    dev = "cuda:0"
    shapes = [(256, 640), (640, 256), (384, 384)]
    r = 128
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    side = torch.cuda.Stream(device=dev)
    ctx_e = fira.FiraContext(shapes, r, fira.FIRA_BF16, device=dev)                  # eager twin
    ctx_g = fira.FiraContext(shapes, r, fira.FIRA_BF16, device=dev, stream=side)     # captured
    W_e = [(0.02 * torch.randn(s, device=dev, generator=gen)).to(torch.bfloat16) for s in shapes]
    W_g = [w.clone() for w in W_e]
    G_e = [torch.zeros(s, device=dev, dtype=torch.bfloat16) for s in shapes]
    G_g = [torch.zeros(s, device=dev, dtype=torch.bfloat16) for s in shapes]
    for i, (m, n) in enumerate(shapes):
        q, _ = torch.linalg.qr(torch.randn((min(m, n), r), device=dev, generator=gen))
        P = q.to(torch.bfloat16).contiguous()
        torch.cuda.synchronize()
        ctx_e.fira_set_projector(i, P)
        ctx_g.fira_set_projector(i, P)
    idx = list(range(len(shapes)))
    prep_e, prep_g = ctx_e.prepare(idx, W_e, G_e), ctx_g.prepare(idx, W_g, G_g)

    def load_new_gradients():
        for ge, gg, s in zip(G_e, G_g, shapes):
            g = (1e-2 * torch.randn(s, device=dev, generator=gen)).to(torch.bfloat16)
            ge.copy_(g)
            gg.copy_(g)
        torch.cuda.synchronize()

    # two eager steps on both: the first caches the work lists and measures the gate of the Gram route (on the
    # residual route), the second collects the gate values and runs the launch sequence that is captured
    for _ in range(2):
        load_new_gradients()
        ctx_e.fira_step(prepared=prep_e)
        ctx_g.fira_step(prepared=prep_g)
        torch.cuda.synchronize()
    assert ctx_g.fira_last_step_fused()
    for a, b in zip(W_e, W_g):
        assert torch.equal(a, b)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ctx_g.fira_step(prepared=prep_g)
    torch.cuda.synchronize()
    for rep in range(3):
        load_new_gradients()
        graph.replay()
        ctx_e.fira_step(prepared=prep_e)
        torch.cuda.synchronize()
        _ = sum(float(w.float().abs().sum()) for w in W_g)      # eager work between the replays
        for i in range(len(shapes)):
            assert torch.equal(W_g[i], W_e[i]), f"replay {rep}, matrix {i}"
    # A learning-rate schedule reaches the captured step: lr * alpha is read from device memory, which
    # fira_set_hparams rewrites in stream order.
    for rep, lr in enumerate([5e-4, 2.5e-4]):
        for c in (ctx_e, ctx_g):
            c.fira_set_hparams(fira.make_hparams(lr=lr))
        load_new_gradients()
        before = [w.clone() for w in W_g]
        graph.replay()
        ctx_e.fira_step(prepared=prep_e)
        torch.cuda.synchronize()
        for i in range(len(shapes)):
            assert torch.equal(W_g[i], W_e[i]), f"replay with lr {lr}, matrix {i}"
            assert not torch.equal(W_g[i], before[i])
