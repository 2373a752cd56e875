"""Pins for the fp64 oracle: each test checks it against something other than itself.

None of these needs a GPU.  A plausible mistake anywhere in the oracle (a dropped
term, a wrong sign or index, a transposed operand, a mask off by one) fails at
least one of them:

  * brute-force scalar-loop attention (tiny shapes),
  * an independent float64 evaluation of the whole layer through PyTorch CPU
    library routines with autograd supplying every gradient,
  * central finite differences on every input and parameter,
  * packed == unpacked, closed forms, rotary / mask / segment-order / GQA invariants.

The paper prints no worked numeric example of a layer, so there is no golden
fixture for it; these properties are what fixes the oracle.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from oracle import layer_oracle as orc
from paper_2408_04275_amd import workloads as wl

DEC, ENC = orc.DECODER, orc.ENCODER


def small_shape(kind, nh=4, nkv=2, d=8, H=24, F=40):
    return wl.LayerShape("t", kind, wl.F32, H, nh, nkv if kind == DEC else nh, d, F, 64)


def draw(shape, cu, seed=0, std=0.3):
    W = {k: v.astype(np.float64) for k, v in wl.make_weights(shape, seed, std=std).items()}
    x, dy = wl.make_activations(shape, int(cu[-1]), seed)
    return W, x.astype(np.float64), dy.astype(np.float64)


def run(shape, cu, modes, W, x, dy=None, **kw):
    y, cache = orc.layer_fwd(shape.kind, shape.n_heads, shape.n_kv_heads, shape.head_dim, cu, modes, W, x, **kw)
    if dy is None:
        return y, cache
    dx, G = orc.layer_bwd(W, cache, dy)
    return y, dx, G, cache


CU5 = np.array([0, 7, 8, 20, 20, 33], dtype=np.int32)        # includes a length-1 and an empty segment
MODES5 = np.array([0, 1, 1, 0, 0], dtype=np.uint8)


# ----------------------------------------------------------------------------
# P1: brute-force attention
# ----------------------------------------------------------------------------
def brute_attention(q, k, v, cu, modes, scale):
    T, nh, d = q.shape
    group = nh // k.shape[1]
    o = np.zeros_like(q)
    for s in range(len(cu) - 1):
        for i in range(cu[s], cu[s + 1]):
            for h in range(nh):
                g = h // group
                js = [j for j in range(cu[s], cu[s + 1]) if modes[s] == 1 or j <= i]
                sc = [scale * sum(q[i, h, c] * k[j, g, c] for c in range(d)) for j in js]
                mx = max(sc)
                w = [math.exp(t - mx) for t in sc]
                z = sum(w)
                for c in range(d):
                    o[i, h, c] = sum(w[n] * v[j, g, c] for n, j in enumerate(js)) / z
    return o


def test_attention_matches_brute_force():
    rng = np.random.default_rng(1)
    T, nh, nkv, d = 33, 4, 2, 8
    q, k, v = (rng.standard_normal((T, n, d)) * 1.5 for n in (nh, nkv, nkv))
    o, lse = orc.attention_fwd(q, k, v, CU5, MODES5, 0.37)
    ref = brute_attention(q, k, v, CU5, MODES5, 0.37)
    assert np.max(np.abs(o - ref)) < 1e-12


def test_softmax_rows_and_lse():
    rng = np.random.default_rng(2)
    L, d = 19, 8
    q, k = rng.standard_normal((L, d)) * 2, rng.standard_normal((L, d)) * 2
    for mode in (0, 1):
        P, lse = orc._probabilities(q, k, 0.4, mode)
        assert np.max(np.abs(P.sum(-1) - 1)) < 1e-14
        S = q @ k.T * 0.4
        np.testing.assert_allclose(P[P > 0], np.exp(S - lse[:, None])[P > 0], rtol=1e-12)
        if mode == 0:
            assert np.all(np.triu(P, 1) == 0) and np.all(np.diag(P) > 0)
        else:
            assert np.all(P > 0)


# ----------------------------------------------------------------------------
# P10: the layer through PyTorch CPU library routines, float64, autograd
# ----------------------------------------------------------------------------
def torch_layer(shape, cu, modes, W, x, eps=1e-5, base=10000.0):
    """Independent formulation: one dense [T, T] additive mask from segment ids, complex-number
    rotary, library norms / activations / softmax; autograd provides all gradients."""
    T, H = x.shape
    nh, nkv, d = shape.n_heads, shape.n_kv_heads, shape.head_dim
    seg = torch.zeros(T, dtype=torch.long)
    pos = torch.zeros(T, dtype=torch.float64)
    bid = torch.zeros(T, dtype=torch.bool)
    for s in range(len(cu) - 1):
        seg[cu[s]:cu[s + 1]] = s
        pos[cu[s]:cu[s + 1]] = torch.arange(cu[s + 1] - cu[s], dtype=torch.float64)
        bid[cu[s]:cu[s + 1]] = bool(modes[s])
    idx = torch.arange(T)
    allowed = (seg[:, None] == seg[None, :]) & (bid[:, None] | (idx[None, :] <= idx[:, None]))
    bias = torch.zeros(T, T, dtype=torch.float64).masked_fill(~allowed, float("-inf"))

    def rot(u):  # u [T, n, d]; pair (i, i + d/2) as a complex number times exp(i * phi)
        half = d // 2
        theta = base ** (-torch.arange(half, dtype=torch.float64) * 2 / d)
        z = torch.complex(u[..., :half], u[..., half:]) * torch.polar(torch.ones(T, half, dtype=torch.float64),
                                                                      pos[:, None] * theta)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    dec = shape.kind == DEC
    if dec:
        h1 = Fn.rms_norm(x, (H,), W["norm1_w"], eps)
        qkv = Fn.linear(h1, W["w_qkv"])
    else:
        h1 = Fn.layer_norm(x, (H,), W["norm1_w"], W["norm1_b"], eps)
        qkv = Fn.linear(h1, W["w_qkv"], W["b_qkv"])
    q, k, v = torch.split(qkv, [nh * d, nkv * d, nkv * d], dim=1)
    q, k, v = q.reshape(T, nh, d), k.reshape(T, nkv, d), v.reshape(T, nkv, d)
    if dec:
        q, k = rot(q), rot(k)
    k = k.repeat_interleave(nh // nkv, dim=1)
    v = v.repeat_interleave(nh // nkv, dim=1)
    sc = torch.einsum("ihc,jhc->hij", q, k) / math.sqrt(d) + bias[None]
    o = torch.einsum("hij,jhc->ihc", torch.softmax(sc, dim=-1), v).reshape(T, nh * d)
    y1 = x + Fn.linear(o, W["w_o"], None if dec else W["b_o"])
    if dec:
        h2 = Fn.rms_norm(y1, (H,), W["norm2_w"], eps)
        gu = Fn.linear(h2, W["w_fc1"])
        F = gu.shape[1] // 2
        m = Fn.silu(gu[:, :F]) * gu[:, F:]
        return y1 + Fn.linear(m, W["w_fc2"])
    h2 = Fn.layer_norm(y1, (H,), W["norm2_w"], W["norm2_b"], eps)
    m = Fn.gelu(Fn.linear(h2, W["w_fc1"], W["b_fc1"]))
    return y1 + Fn.linear(m, W["w_fc2"], W["b_fc2"])


@pytest.mark.parametrize("kind", [DEC, ENC])
def test_layer_matches_torch_autograd(kind):
    shape = small_shape(kind)
    cu = np.array([0, 7, 8, 20, 33], dtype=np.int32)
    modes = np.array([0, 1, 1, 0], dtype=np.uint8) if kind == DEC else np.ones(4, dtype=np.uint8)
    W, x, dy = draw(shape, cu, seed=3)
    y, dx, G, _ = run(shape, cu, modes, W, x, dy)
    tW = {k: torch.tensor(v, requires_grad=True) for k, v in W.items()}
    tx = torch.tensor(x, requires_grad=True)
    ty = torch_layer(shape, cu, modes, tW, tx)
    ty.backward(torch.tensor(dy))
    assert np.max(np.abs(y - ty.detach().numpy())) < 1e-10
    assert np.max(np.abs(dx - tx.grad.numpy())) < 1e-10
    assert set(G) == set(W)
    for name in W:
        ref = tW[name].grad.numpy()
        assert np.max(np.abs(G[name] - ref)) < 1e-10 * max(1.0, np.max(np.abs(ref))), name


# ----------------------------------------------------------------------------
# P4: finite differences
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("kind", [DEC, ENC])
def test_finite_differences(kind):
    shape = small_shape(kind, H=16, F=24)
    cu = np.array([0, 5, 6, 17], dtype=np.int32)
    modes = np.array([0, 1, 0], dtype=np.uint8) if kind == DEC else np.ones(3, dtype=np.uint8)
    W, x, dy = draw(shape, cu, seed=4)
    _, dx, G, _ = run(shape, cu, modes, W, x, dy)
    rng = np.random.default_rng(5)

    def loss(Wp, xp):
        return float(np.sum(run(shape, cu, modes, Wp, xp)[0] * dy))

    targets = [("x", x, dx)] + [(n, W[n], G[n]) for n in W]
    for name, arr, grad in targets:
        flat = arr.reshape(-1)
        for i in rng.choice(flat.size, size=min(flat.size, 200), replace=False):
            old = flat[i]
            h = 1e-6 * max(1.0, abs(old))
            flat[i] = old + h
            lp = loss(W, x)
            flat[i] = old - h
            lm = loss(W, x)
            flat[i] = old
            num = (lp - lm) / (2 * h)
            ana = grad.reshape(-1)[i]
            assert abs(num - ana) <= 2e-6 * max(1.0, abs(ana)), (name, i, num, ana)


@pytest.mark.parametrize("kind", [DEC, ENC])
def test_stack_matches_torch_autograd(kind):
    # three layers with different weights: the stack's output and every layer's gradients against autograd
    # through the independently written torch layer
    shape = small_shape(kind)
    cu = np.array([0, 7, 8, 20, 33], dtype=np.int32)
    modes = np.array([0, 1, 1, 0], dtype=np.uint8) if kind == DEC else np.ones(4, dtype=np.uint8)
    Ws = []
    for l in range(3):
        W, x, dy = draw(shape, cu, seed=10 + l)
        Ws.append(W)
    y, caches = orc.stack_fwd(shape.kind, shape.n_heads, shape.n_kv_heads, shape.head_dim, cu, modes, Ws, x,
                              eps=shape.norm_eps, rope_base=shape.rope_base)
    dx, Gs = orc.stack_bwd(Ws, caches, dy)
    tWs = [{k: torch.tensor(v, requires_grad=True) for k, v in W.items()} for W in Ws]
    tx = torch.tensor(x, requires_grad=True)
    th = tx
    for tW in tWs:
        th = torch_layer(shape, cu, modes, tW, th)
    th.backward(torch.tensor(dy))
    assert np.max(np.abs(y - th.detach().numpy())) < 1e-9
    assert np.max(np.abs(dx - tx.grad.numpy())) < 1e-9
    for G, tW in zip(Gs, tWs):
        for name in tW:
            ref = tW[name].grad.numpy()
            assert np.max(np.abs(G[name] - ref)) < 1e-9 * max(1.0, np.max(np.abs(ref))), name


# ----------------------------------------------------------------------------
# P2 / P8: packed == unpacked, segment-order invariance
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("kind", [DEC, ENC])
def test_packed_equals_unpacked(kind):
    shape = small_shape(kind)
    modes = MODES5 if kind == DEC else np.ones(5, dtype=np.uint8)
    W, x, dy = draw(shape, CU5, seed=6)
    y, dx, G, _ = run(shape, CU5, modes, W, x, dy)
    Gsum = {k: np.zeros_like(v) for k, v in G.items()}
    for s in range(5):
        a, b = CU5[s], CU5[s + 1]
        if a == b:
            continue
        ys, dxs, Gs, _ = run(shape, np.array([0, b - a]), modes[s:s + 1], W, x[a:b], dy[a:b])
        assert np.max(np.abs(ys - y[a:b])) < 1e-11
        assert np.max(np.abs(dxs - dx[a:b])) < 1e-11
        for k in Gs:
            Gsum[k] += Gs[k]
    for k in G:
        assert np.max(np.abs(Gsum[k] - G[k])) < 1e-10, k


def test_segment_order_invariance():
    # Reordering whole subsequences permutes outputs block-wise and leaves the summed
    # weight gradients unchanged: the commutativity argument of Section 5.2.
    shape = small_shape(DEC)
    W, x, dy = draw(shape, CU5, seed=7)
    y, dx, G, _ = run(shape, CU5, MODES5, W, x, dy)
    perm = [3, 0, 4, 2, 1]
    blocks = [(CU5[s], CU5[s + 1]) for s in perm]
    xp = np.concatenate([x[a:b] for a, b in blocks])
    dyp = np.concatenate([dy[a:b] for a, b in blocks])
    cup = np.concatenate([[0], np.cumsum([b - a for a, b in blocks])]).astype(np.int32)
    yp, dxp, Gp, _ = run(shape, cup, MODES5[perm], W, xp, dyp)
    assert np.max(np.abs(yp - np.concatenate([y[a:b] for a, b in blocks]))) < 1e-11
    assert np.max(np.abs(dxp - np.concatenate([dx[a:b] for a, b in blocks]))) < 1e-11
    for k in G:
        assert np.max(np.abs(Gp[k] - G[k])) < 1e-10, k


# ----------------------------------------------------------------------------
# P5: closed forms
# ----------------------------------------------------------------------------
def test_length_one_segments_output_value_rows():
    shape = small_shape(DEC)
    cu = np.arange(0, 7, dtype=np.int32)                      # six segments of one token
    W, x, _ = draw(shape, cu, seed=8)
    y, c = run(shape, cu, np.zeros(6, dtype=np.uint8), W, x)
    nh, nkv, d = 4, 2, 8
    v_rep = np.repeat(c["v"], nh // nkv, axis=1).reshape(6, nh * d)
    assert np.max(np.abs(c["o"] - v_rep)) < 1e-14
    assert np.max(np.abs(c["y1"] - (x + v_rep @ W["w_o"].T))) < 1e-13


def test_equal_keys_give_running_and_segment_means():
    rng = np.random.default_rng(9)
    L, d = 12, 8
    q = rng.standard_normal((L, 1, d))
    k = np.tile(rng.standard_normal((1, 1, d)), (L, 1, 1))
    v = rng.standard_normal((L, 1, d))
    cu = np.array([0, L])
    o, _ = orc.attention_fwd(q, k, v, cu, [0], 0.5)
    run_mean = np.cumsum(v, axis=0) / np.arange(1, L + 1)[:, None, None]
    assert np.max(np.abs(o - run_mean)) < 1e-13
    o, _ = orc.attention_fwd(q, k, v, cu, [1], 0.5)
    assert np.max(np.abs(o - v.mean(0, keepdims=True))) < 1e-13


@pytest.mark.parametrize("kind", [DEC, ENC])
def test_zero_output_projections_make_identity(kind):
    shape = small_shape(kind)
    modes = MODES5 if kind == DEC else np.ones(5, dtype=np.uint8)
    W, x, dy = draw(shape, CU5, seed=10)
    for n in ("w_o", "w_fc2", "b_o", "b_fc2"):
        if n in W:
            W[n][...] = 0
    y, dx, _, _ = run(shape, CU5, modes, W, x, dy)
    assert np.array_equal(y, x) and np.array_equal(dx, dy)


def test_norm_closed_forms():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((5, 32)) * 3 + 1
    h, r = orc.rmsnorm_fwd(x, np.ones(32), 1e-12)
    assert np.max(np.abs(np.mean(h * h, -1) - 1)) < 1e-10
    h2, _ = orc.rmsnorm_fwd(7.5 * x, np.ones(32), 1e-12)
    assert np.max(np.abs(h - h2)) < 1e-10
    g, b = rng.standard_normal(32), rng.standard_normal(32)
    ln, mu, r = orc.layernorm_fwd(x, np.ones(32), np.zeros(32), 1e-12)
    assert np.max(np.abs(ln.mean(-1))) < 1e-12 and np.max(np.abs(ln.var(-1) - 1)) < 1e-9
    ln2, _, _ = orc.layernorm_fwd(x + 11.0, np.ones(32), np.zeros(32), 1e-12)
    assert np.max(np.abs(ln - ln2)) < 1e-10
    ln3, _, _ = orc.layernorm_fwd(x, g, b, 1e-5)
    ref = Fn.layer_norm(torch.tensor(x), (32,), torch.tensor(g), torch.tensor(b), 1e-5).numpy()
    assert np.max(np.abs(ln3 - ref)) < 1e-12


def test_activation_values():
    assert orc.gelu(np.array([0.0]))[0] == 0 and orc.sigmoid(np.array([0.0]))[0] == 0.5
    z = np.linspace(-4, 4, 41)
    np.testing.assert_allclose(orc.gelu(z), Fn.gelu(torch.tensor(z)).numpy(), atol=1e-14)
    # Phi(1) = 0.841344746068543 (standard normal CDF), so gelu(1) = Phi(1)
    assert abs(orc.gelu(np.array([1.0]))[0] - 0.841344746068543) < 1e-14
    num = (orc.gelu(z + 1e-6) - orc.gelu(z - 1e-6)) / 2e-6
    np.testing.assert_allclose(orc.gelu_grad(z), num, atol=1e-8)


def test_zero_gate_passes_residual():
    shape = small_shape(DEC)
    W, x, _ = draw(shape, CU5, seed=12)
    W["w_fc1"][:shape.ffn_hidden] = 0                           # gate rows
    y, c = run(shape, CU5, MODES5, W, x)
    assert np.array_equal(y, c["y1"])


# ----------------------------------------------------------------------------
# P6: rotary properties
# ----------------------------------------------------------------------------
def test_rope_properties():
    rng = np.random.default_rng(13)
    u = rng.standard_normal((9, 3, 8))
    pos = np.arange(9)
    r = orc.rope(u, pos, 10000.0)
    assert np.array_equal(r[0], u[0])                           # position 0 is the identity
    np.testing.assert_allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(u, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(orc.rope(r, pos, 10000.0, inverse=True), u, atol=1e-13)
    # pair (i, i + d/2), angle pos * base^(-2i/d): written out for one element
    t, i, d = 5, 1, 8
    phi = t * 10000.0 ** (-2 * i / d)
    assert abs(r[t, 0, i] - (u[t, 0, i] * math.cos(phi) - u[t, 0, i + 4] * math.sin(phi))) < 1e-14
    assert abs(r[t, 0, i + 4] - (u[t, 0, i + 4] * math.cos(phi) + u[t, 0, i] * math.sin(phi))) < 1e-14


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(14)
    q, k, v = (rng.standard_normal((10, 2, 8)) for _ in range(3))
    cu = np.array([0, 10])
    outs = []
    for shift in (0, 37):
        pos = np.arange(10) + shift
        o, _ = orc.attention_fwd(orc.rope(q, pos, 1e4), orc.rope(k, pos, 1e4), v, cu, [0], 0.3)
        outs.append(o)
    assert np.max(np.abs(outs[0] - outs[1])) < 1e-10


# ----------------------------------------------------------------------------
# P7: mask properties
# ----------------------------------------------------------------------------
def test_causality_and_segment_isolation():
    shape = small_shape(DEC)
    W, x, _ = draw(shape, CU5, seed=15)
    y, _ = run(shape, CU5, MODES5, W, x)
    t = 12                                                      # inside segment 2 = [8, 20), bidirectional
    x2 = x.copy(); x2[t] += 1.0
    y2, _ = run(shape, CU5, MODES5, W, x2)
    changed = np.any(y2 != y, axis=1)
    assert changed[8:20].all() and not changed[:8].any() and not changed[20:].any()
    t = 25                                                      # inside segment 4 = [20, 33), causal
    x3 = x.copy(); x3[t] += 1.0
    y3, _ = run(shape, CU5, MODES5, W, x3)
    changed = np.any(y3 != y, axis=1)
    assert changed[25:33].all() and not changed[:25].any()


def test_bidirectional_encoder_is_permutation_equivariant():
    shape = small_shape(ENC)
    cu = np.array([0, 9, 20], dtype=np.int32)
    W, x, _ = draw(shape, cu, seed=16)
    y, _ = run(shape, cu, [1, 1], W, x)
    perm = np.concatenate([np.random.default_rng(0).permutation(9), np.arange(9, 20)])
    yp, _ = run(shape, cu, [1, 1], W, x[perm])
    assert np.max(np.abs(yp - y[perm])) < 1e-12


# ----------------------------------------------------------------------------
# P9: grouped-query attention
# ----------------------------------------------------------------------------
def test_gqa_equals_mha_with_replicated_kv():
    g = small_shape(DEC, nh=4, nkv=2)
    m = small_shape(DEC, nh=4, nkv=4)
    W, x, dy = draw(g, CU5, seed=17)
    nq, nk, d = g.nq, g.nkv, g.head_dim
    wq, wk, wv = W["w_qkv"][:nq], W["w_qkv"][nq:nq + nk], W["w_qkv"][nq + nk:]
    rep = lambda w: np.repeat(w.reshape(2, d, -1), 2, axis=0).reshape(4 * d, -1)
    Wm = dict(W, w_qkv=np.concatenate([wq, rep(wk), rep(wv)]))
    y, dx, G, _ = run(g, CU5, MODES5, W, x, dy)
    ym, dxm, Gm, _ = run(m, CU5, MODES5, Wm, x, dy)
    assert np.max(np.abs(y - ym)) < 1e-12 and np.max(np.abs(dx - dxm)) < 1e-12
    fold = lambda w: w.reshape(2, 2, d, -1).sum(1).reshape(2 * d, -1)
    gm = Gm["w_qkv"]
    folded = np.concatenate([gm[:nq], fold(gm[nq:nq + 4 * d]), fold(gm[nq + 4 * d:])])
    assert np.max(np.abs(folded - G["w_qkv"])) < 1e-11


# ----------------------------------------------------------------------------
# workload generators (host logic)
# ----------------------------------------------------------------------------
def test_workload_layouts():
    cu, modes, kinds = wl.make_segments(1)
    assert cu.tolist() == [0, 128, 224, 384, 512] and modes.tolist() == [0, 0, 0, 0]
    assert wl.make_segments(1, image_bidir=True)[1].tolist() == [0, 0, 0, 1]
    cu, modes, _ = wl.make_segments(2)
    assert len(cu) == 17 and cu[-1] <= 16384 and set(np.diff(cu)) <= {256, 576, 1024} and modes.all()
    for cfg in (3, 5):
        for seed in range(5):
            cu, modes, kinds = wl.make_segments(cfg, seed)
            L = np.diff(cu)
            assert cu[-1] == 8192 and L.min() >= 1 and not modes.any()
            assert all(l == 576 for l, k in zip(L, kinds) if k == "image")
    seed = wl.longtail_seed()
    cu, _, _ = wl.make_segments(4, seed)
    assert cu[-1] == 8192 and np.diff(cu).max() >= 6000
    a = wl.round_bf16(np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 3.14159], dtype=np.float32))
    assert a.tolist() == [1.0, 1.015625, 3.140625]              # ties to even, then a plain rounding
    ref = torch.tensor([3.14159, -1e-3, 65504.0]).to(torch.bfloat16).float().numpy()
    assert np.array_equal(wl.round_bf16(np.array([3.14159, -1e-3, 65504.0], dtype=np.float32)), ref)


def test_model_flops_convention():
    s3 = wl.SHAPES[3]
    cu = np.array([0, 8192]); modes = np.array([0], dtype=np.uint8)
    f = wl.model_flops(s3, cu, modes)
    assert abs(f["gemm_fwd"] - 3.3157e12) / 3.3157e12 < 1e-3    # 2 * T * 202 375 168 parameters
    assert f["attn_fwd"] == 4 * 128 * 32 * (8192 * 8193 // 2)
    assert f["fwd_bwd"] == 3 * f["fwd"]


def test_allowed_ranges_are_monotonic_in_the_token_index():
    """The attention mask of a pack (Section "Intra-microbatch Reordering": sequences packed back to back, each
    attending within itself, causally or bidirectionally) gives every query an allowed key range [lo, hi) and every
    key an allowed query range; both bounds never decrease from one token to the next.  The GPU kernels take a
    wavefront's extreme bounds from its first and last token on the strength of this.  Checked here on the mask the
    oracle builds, by brute force over random packs with empty and one-token segments."""
    from oracle import layer_oracle as orc
    rng = np.random.default_rng(5)
    for case in range(40):
        n = int(rng.integers(1, 9))
        lens = rng.integers(0, 40, n)
        lens[rng.integers(0, n)] = int(rng.integers(1, 70))
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        modes = rng.integers(0, 2, n).astype(np.uint8)
        T = int(cu[-1])
        allowed = np.zeros((T, T), dtype=bool)                  # allowed[q, k]
        q = rng.standard_normal((T, 1, 4))
        for s in range(n):
            a, b = int(cu[s]), int(cu[s + 1])
            if b > a:
                P, _ = orc._probabilities(q[a:b, 0], q[a:b, 0], 1.0, int(modes[s]))
                allowed[a:b, a:b] = P > 0
        for M in (allowed, allowed.T):                          # per query over keys, per key over queries
            lo = np.array([np.flatnonzero(r)[0] for r in M])
            hi = np.array([np.flatnonzero(r)[-1] + 1 for r in M])
            for t in range(T):
                assert M[t, lo[t]:hi[t]].all(), "allowed partners form one interval"
            assert (np.diff(lo) >= 0).all() and (np.diff(hi) >= 0).all(), (case, cu.tolist(), modes.tolist())
