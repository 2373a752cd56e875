"""GPU parity of mmtrain_stack_fwd / mmtrain_stack_bwd (a stack of layers, with and without recomputation)
against the fp64 oracle, and the properties that tie the stack to the single-layer entry points."""
import numpy as np
import pytest
import torch

from oracle import bf16_storage
from oracle import layer_oracle as orc
from paper_2408_04275_amd import parity
from paper_2408_04275_amd import binding as mm
from paper_2408_04275_amd import workloads as wl
from paper_2408_04275_amd.harness import LayerRunner, StackRunner
from util import assert_parity, say

pytestmark = pytest.mark.gpu

CU = np.array([0, 1, 1, 70, 199, 200, 457, 648], dtype=np.int32)      # length-1, empty, mid-tile boundaries
MODES = np.array([0, 1, 1, 0, 1, 0, 1], dtype=np.uint8)


def draw(shape, n_layers, seed):
    Ws = [wl.make_weights(shape, seed + 100 * l, std=0.05) for l in range(n_layers)]
    x, dy = wl.make_activations(shape, int(CU[-1]), seed)
    return Ws, x, dy


def shapes():
    return [wl.LayerShape("stack-dec-f32", wl.DECODER, wl.F32, 256, 4, 2, 64, 512, 648),
            wl.LayerShape("stack-dec-bf16", wl.DECODER, wl.BF16, 272, 4, 2, 64, 688, 648),
            wl.LayerShape("stack-enc-bf16", wl.ENCODER, wl.BF16, 272, 4, 4, 64, 528, 648)]


@pytest.mark.parametrize("shape", shapes(), ids=lambda s: s.name)
@pytest.mark.parametrize("recompute", [False, True])
def test_stack_matches_the_oracle(shape, recompute):
    n = 3
    modes = MODES if shape.kind == wl.DECODER else np.ones(len(MODES), dtype=np.uint8)
    Ws, x, dy = draw(shape, n, seed=11)
    ry, caches = orc.stack_fwd(shape.kind, shape.n_heads, shape.n_kv_heads, shape.head_dim, CU, modes, Ws, x,
                               eps=shape.norm_eps, rope_base=shape.rope_base)
    rdx, rG = orc.stack_bwd(Ws, caches, dy)
    fy = fdx = None
    fG = [{} for _ in range(n)]
    if shape.dtype == wl.BF16:                       # what bf16 storage alone costs this stack, tensor by tensor
        ey, edx, eG = bf16_storage.stack_fwd_bwd_rounded(shape.kind, shape.n_heads, shape.n_kv_heads, shape.head_dim, CU, modes,
                                                         Ws, x, dy, eps=shape.norm_eps, rope_base=shape.rope_base)
        fy, fdx = parity.errors(ey, ry), parity.errors(edx, rdx)
        fG = [{k: parity.errors(eG[l][k], rG[l][k]) for k in rG[l]} for l in range(n)]
    r = StackRunner(shape, Ws, CU, modes, recompute=recompute)
    r.set_inputs(x, dy)
    r.step()
    y, dx, G = r.results()
    what = f"{shape.name} recompute={recompute} "
    worst = [assert_parity(what + "y", y, ry, shape.dtype, floor=fy), assert_parity(what + "dx", dx, rdx, shape.dtype, floor=fdx)]
    for l in range(n):
        assert set(G[l]) == set(rG[l])
        for k in rG[l]:
            worst.append(assert_parity(what + f"layer {l} d{k}", G[l][k], rG[l][k], shape.dtype, floor=fG[l].get(k)))
    say(what + "max_err %.2e" % max(e["max_err"] for e in worst))


@pytest.mark.parametrize("shape", shapes()[1:], ids=lambda s: s.name)
def test_recomputation_is_bit_identical_and_smaller(shape):
    n = 4
    modes = MODES if shape.kind == wl.DECODER else np.ones(len(MODES), dtype=np.uint8)
    Ws, x, dy = draw(shape, n, seed=12)
    runs = []
    for recompute in (False, True):
        r = StackRunner(shape, Ws, CU, modes, recompute=recompute)
        r.set_inputs(x, dy)
        r.step()
        torch.cuda.synchronize()
        runs.append(r)
    a, b = runs
    assert torch.equal(a.y, b.y) and torch.equal(a.dx, b.dx)
    for ga, gb in zip(a.g, b.g):
        for k in ga:
            assert torch.equal(ga[k], gb[k]), k
    assert b.ctx_bytes < a.ctx_bytes


def test_one_layer_stack_is_the_layer():
    shape = shapes()[1]
    Ws, x, dy = draw(shape, 1, seed=13)
    s = StackRunner(shape, Ws, CU, MODES)
    s.set_inputs(x, dy)
    s.step()
    l = LayerRunner(shape, Ws[0], CU, MODES)
    l.set_inputs(x, dy)
    l.step()
    torch.cuda.synchronize()
    assert torch.equal(s.y, l.y) and torch.equal(s.dx, l.dx)
    for k in l.g:
        assert torch.equal(s.g[0][k], l.g[k]), k


def test_frozen_stack_and_accumulation():
    shape = shapes()[1]
    n = 2
    Ws, x, dy = draw(shape, n, seed=14)
    full = StackRunner(shape, Ws, CU, MODES, recompute=True)
    full.set_inputs(x, dy)
    full.step()
    frozen = StackRunner(shape, Ws, CU, MODES, recompute=True, with_grads=False)   # grads = NULL: input gradient only
    frozen.set_inputs(x, dy)
    frozen.step()
    torch.cuda.synchronize()
    assert torch.equal(full.dx, frozen.dx)
    # a second microbatch accumulated on top of the first: twice the gradient, up to one storage rounding
    once = [{k: v.clone() for k, v in g.items()} for g in full.g]
    full.step(mm.BWD_ACCUMULATE_WGRAD)
    torch.cuda.synchronize()
    for g1, g2 in zip(once, full.g):
        for k in g1:
            ref = 2.0 * g1[k].float()
            assert torch.allclose(g2[k].float(), ref, rtol=1e-2, atol=1e-2 * float(ref.abs().max())), k
