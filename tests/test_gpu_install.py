"""fira_set_projectors: the batched installation must leave exactly what per-matrix fira_set_projector calls
leave (operand copies, gate estimate, the steps that follow), for lists longer than one launch batch, mixed
orientations, ranks and storage types, and it must reject bad lists without touching anything."""
import numpy as np
import pytest
import torch

from paper_2410_01623_amd import fira

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed=3):
    # 21 matrices: more than one batch of 16, both orientations, three ranks, the last three stored in fp32
    shapes = [(256, 640), (640, 256), (384, 384), (128, 900), (900, 128), (512, 512)] * 3 + [(64, 200), (200, 64), (96, 96)]
    ranks = [128, 128, 64, 32, 32, 256] * 3 + [16, 16, 96]
    dtypes = [fira.FIRA_BF16] * 18 + [fira.FIRA_F32] * 3
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    P = []
    for (m, n), r in zip(shapes, ranks):
        q, _ = torch.linalg.qr(torch.randn((min(m, n), r), device=DEV, generator=gen))
        P.append(q.contiguous())
    # one projector far from orthonormal: its gate value must come back the same from both ways
    P[4] = (P[4] * 1.5).contiguous()
    return shapes, ranks, dtypes, P, gen


def _wg(shapes, dtypes, gen):
    td = {fira.FIRA_BF16: torch.bfloat16, fira.FIRA_F32: torch.float32}
    W = [(0.02 * torch.randn(s, device=DEV, generator=gen)).to(td[d]) for s, d in zip(shapes, dtypes)]
    G = [(1e-3 * torch.randn(s, device=DEV, generator=gen)).to(td[d]) for s, d in zip(shapes, dtypes)]
    return W, G


@pytest.mark.parametrize("p_dtype", [torch.float32, torch.bfloat16])
def test_batched_installation_equals_single_calls(p_dtype):
    shapes, ranks, dtypes, P, gen = _case()
    P = [p.to(p_dtype).contiguous() for p in P]
    n = len(shapes)
    one = fira.FiraContext(shapes, ranks, dtypes, device=DEV)
    many = fira.FiraContext(shapes, ranks, dtypes, device=DEV)
    for i in range(n):
        one.fira_set_projector(i, P[i])
    order = list(reversed(range(n)))          # any order of the list
    many.fira_set_projectors(order, [P[i] for i in order])
    torch.cuda.synchronize()
    for i in range(n):
        assert torch.equal(one.fira_get_projector(i), many.fira_get_projector(i)), f"matrix {i}: operand copies differ"
        ga, gb = one.fira_get_gate(i), many.fira_get_gate(i)
        assert ga[0] == gb[0], f"matrix {i}: gate estimate {ga[0]} vs {gb[0]}"
    assert one.fira_get_gate(4)[0] > 0.5 and one.fira_get_gate(0)[0] < 0.02
    W, G = _wg(shapes, dtypes, gen)
    W1, W2 = [w.clone() for w in W], [w.clone() for w in W]
    idx = list(range(n))
    for _ in range(3):
        one.fira_step(idx, W1, G)
        many.fira_step(idx, W2, G)
    torch.cuda.synchronize()
    for i in range(n):
        assert torch.equal(W1[i], W2[i]), f"matrix {i}: weights differ after three steps"
        assert one.fira_get_gate(i) == many.fira_get_gate(i)


def test_second_call_replaces_part_of_the_list():
    """A later call for a few matrices (new bases) changes those and leaves the others' projectors alone."""
    shapes, ranks, dtypes, P, gen = _case(seed=5)
    n = len(shapes)
    ctx = fira.FiraContext(shapes, ranks, dtypes, device=DEV)
    ctx.fira_set_projectors(range(n), P)
    before = [ctx.fira_get_projector(i) for i in range(n)]
    sub = [2, 7, 19]
    newP = [P[i].flip(1).contiguous() for i in sub]
    ctx.fira_set_projectors(sub, newP)
    torch.cuda.synchronize()
    for i in range(n):
        now = ctx.fira_get_projector(i)
        if i in sub:
            assert torch.equal(now, before[i].flip(1))
        else:
            assert torch.equal(now, before[i])


def test_bad_lists_are_rejected_and_change_nothing():
    shapes = [(64, 96), (96, 64)]
    ctx = fira.FiraContext(shapes, 16, fira.FIRA_BF16, device=DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(1)
    P = [torch.linalg.qr(torch.randn((64, 16), device=DEV, generator=gen))[0].contiguous() for _ in shapes]
    ctx.fira_set_projectors([0, 1], P)
    before = [ctx.fira_get_projector(i) for i in range(2)]
    other = [(-p).contiguous() for p in P]
    for idx in ([0, 0], [0, 2], [-1, 1]):
        with pytest.raises(fira.FiraError) as e:
            ctx.fira_set_projectors(idx, other)
        assert e.value.status == fira.FIRA_ERR_INVALID_ARG
    ctx.fira_set_projectors([], [])            # an empty list is fine
    torch.cuda.synchronize()
    for i in range(2):
        assert torch.equal(ctx.fira_get_projector(i), before[i])
