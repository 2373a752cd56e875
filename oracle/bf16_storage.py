"""What bf16 storage alone costs: the fp64 oracle's layer with a rounding to bf16 at every point where a layer
that feeds bf16 matrix cores has to store a tensor, and nothing else changed.

TEST INFRASTRUCTURE ONLY, like the rest of this package: it calls layer_oracle's operators and numpy, shares
no code with the HIP path and is never imported by it.

Why it exists.  The stated tolerance is a maximum relative error of 2e-2 for bf16 inputs with fp32
accumulation.  A bf16 rounding has a relative error of up to 2^-9; a layer rounds about ten tensors between
x and a gradient, and an element of a result that is small against its tensor's scale carries the absolute
error of the large terms summed into it.  How large the element-wise deviation from the unrounded fp64
result is for ANY implementation that keeps its tensors in bf16 is therefore a property of the layer's
shape, weights and pack, not of the implementation; this module measures it with no GPU involved, and the
parity tests hold the HIP path to a stated multiple of it (tests/golden/bf16_floor.json for the full-size
workloads, computed on the spot for small cases).

Where it rounds (R = round to nearest even to bf16, the value kept in fp64):
  forward   h1 = R(norm1(x));  qkv = R(h1 Wqkv^T + b);  q, k = R(rope(q, k));  o = R(attention);
            y1 = R(x + o Wo^T + b);  h2 = R(norm2(y1));  pre = R(h2 Wfc1^T + b);  m = R(act(pre));
            y = R(y1 + m Wfc2^T + b)
  backward  every input gradient and every parameter gradient once, where the chain rule of layer_oracle
            produces it (the rotary embedding's inverse rotation is applied before the rounding of dq, dk)
  inside attention: the probabilities as the operand of the product with V (unnormalised, relative to the
            row maximum; the row sum is taken before the rounding), and in backward the probabilities as
            the operand of dV = P^T dO and dS as the operand of dQ and dK -- a matrix-core product takes
            bf16 operands, so these roundings belong to storage as much as the ones above.
Everything between the roundings is fp64.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

from . import layer_oracle as orc

f64 = np.float64


def bf16_round(a) -> np.ndarray:
    """Round to the nearest bf16 value (ties to even); returns float64.  Finite inputs only."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(f64)


R = bf16_round


def attention_fwd_rounded(q, k, v, cu, modes, scale):
    """layer_oracle.attention_fwd with the probabilities rounded as the operand of the product with V."""
    T, nh, d = q.shape
    group = nh // k.shape[1]
    o = np.zeros((T, nh, d), dtype=f64)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        L = b - a
        allowed = np.tril(np.ones((L, L), dtype=bool)) if int(modes[s]) == orc.CAUSAL else np.ones((L, L), dtype=bool)
        for h in range(nh):
            S = np.where(allowed, (q[a:b, h] @ k[a:b, h // group].T) * scale, -np.inf)
            E = np.exp(S - np.max(S, axis=-1, keepdims=True))
            o[a:b, h] = (R(E) @ v[a:b, h // group]) / np.sum(E, axis=-1, keepdims=True)
    return o


def attention_bwd_rounded(do, o, q, k, v, cu, modes, scale):
    """layer_oracle.attention_bwd with P rounded for dV and dS rounded for dQ, dK; D = rowsum(dO * O) from the
    stored (rounded) output, as a backward pass that does not keep P has to form it."""
    T, nh, d = q.shape
    group = nh // k.shape[1]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        for h in range(nh):
            g = h // group
            P, _ = orc._probabilities(q[a:b, h], k[a:b, g], scale, int(modes[s]))
            dO = do[a:b, h]
            dv[a:b, g] += R(P).T @ dO
            dP = dO @ v[a:b, g].T
            D = np.sum(dO * o[a:b, h], axis=-1, keepdims=True)
            dS = R(P * (dP - D))
            dq[a:b, h] = (dS @ k[a:b, g]) * scale
            dk[a:b, g] += (dS.T @ q[a:b, h]) * scale
    return dq, dk, dv


def layer_fwd_bwd_rounded(kind: int, n_heads: int, n_kv_heads: int, head_dim: int, cu, modes,
                          weights: Dict[str, np.ndarray], x, dy, eps: float = 1e-5, rope_base: float = 10000.0,
                          round_param_grads: bool = True):
    """Forward + backward of one layer with bf16 storage roundings.  Returns (y, dx, grads).

    round_param_grads=False models fp32 main-gradient buffers (parameter gradients leave the products unrounded)."""
    W = {k_: np.asarray(v_, dtype=f64) for k_, v_ in weights.items() if v_ is not None}
    x = np.asarray(x, dtype=f64)
    dy = np.asarray(dy, dtype=f64)
    cu = np.asarray(cu, dtype=np.int64)
    T = x.shape[0]
    nh, nkv, d = n_heads, n_kv_heads, head_dim
    nq, nk = nh * d, nkv * d
    scale = 1.0 / np.sqrt(d)
    dec = kind == orc.DECODER
    Rg = R if round_param_grads else (lambda a: np.asarray(a, dtype=f64))

    def bias(name):
        return 0.0 if dec else W[name][None, :]

    # ---- forward
    if dec:
        h1, r1 = orc.rmsnorm_fwd(x, W["norm1_w"], eps)
    else:
        h1, mu1, r1 = orc.layernorm_fwd(x, W["norm1_w"], W["norm1_b"], eps)
    h1 = R(h1)
    qkv = R(h1 @ W["w_qkv"].T + bias("b_qkv"))
    q = qkv[:, :nq].reshape(T, nh, d)
    k = qkv[:, nq:nq + nk].reshape(T, nkv, d)
    v = qkv[:, nq + nk:].reshape(T, nkv, d)
    if dec:
        pos = orc.positions(cu)
        q, k = R(orc.rope(q, pos, rope_base)), R(orc.rope(k, pos, rope_base))
    o3 = R(attention_fwd_rounded(q, k, v, cu, modes, scale))
    o = o3.reshape(T, nq)
    y1 = R(x + o @ W["w_o"].T + bias("b_o"))
    if dec:
        h2, r2 = orc.rmsnorm_fwd(y1, W["norm2_w"], eps)
    else:
        h2, mu2, r2 = orc.layernorm_fwd(y1, W["norm2_w"], W["norm2_b"], eps)
    h2 = R(h2)
    pre = R(h2 @ W["w_fc1"].T + bias("b_fc1"))
    if dec:
        F = W["w_fc2"].shape[1]
        gate, up = pre[:, :F], pre[:, F:]
        m = R(gate * orc.sigmoid(gate) * up)
    else:
        m = R(orc.gelu(pre))
    y = R(y1 + m @ W["w_fc2"].T + bias("b_fc2"))

    # ---- backward
    G: Dict[str, np.ndarray] = {}
    d_m = R(dy @ W["w_fc2"])
    G["w_fc2"] = Rg(dy.T @ m)
    del m
    if not dec:
        G["b_fc2"] = Rg(np.sum(dy, axis=0))
    if dec:
        sg = orc.sigmoid(gate)
        d_pre = R(np.concatenate([d_m * up * sg * (1.0 + gate * (1.0 - sg)), d_m * gate * sg], axis=1))
        del sg
    else:
        d_pre = R(d_m * orc.gelu_grad(pre))
        G["b_fc1"] = Rg(np.sum(d_pre, axis=0))
    del d_m, pre
    d_h2 = R(d_pre @ W["w_fc1"])
    G["w_fc1"] = Rg(d_pre.T @ h2)
    del d_pre
    if dec:
        d_n2, dg = orc.rmsnorm_bwd(d_h2, y1, W["norm2_w"], r2)
    else:
        d_n2, dg, db = orc.layernorm_bwd(d_h2, y1, W["norm2_w"], mu2, r2)
        G["norm2_b"] = Rg(db)
    G["norm2_w"] = Rg(dg)
    d_y1 = R(dy + d_n2)
    d_o = R(d_y1 @ W["w_o"])
    G["w_o"] = Rg(d_y1.T @ o)
    if not dec:
        G["b_o"] = Rg(np.sum(d_y1, axis=0))
    dq, dk, dv = attention_bwd_rounded(d_o.reshape(T, nh, d), o3, q, k, v, cu, modes, scale)
    if dec:
        dq, dk = orc.rope(dq, pos, rope_base, inverse=True), orc.rope(dk, pos, rope_base, inverse=True)
    d_qkv = R(np.concatenate([dq.reshape(T, nq), dk.reshape(T, nk), dv.reshape(T, nk)], axis=1))
    d_h1 = R(d_qkv @ W["w_qkv"])
    G["w_qkv"] = Rg(d_qkv.T @ h1)
    if not dec:
        G["b_qkv"] = Rg(np.sum(d_qkv, axis=0))
    if dec:
        d_n1, dg = orc.rmsnorm_bwd(d_h1, x, W["norm1_w"], r1)
    else:
        d_n1, dg, db = orc.layernorm_bwd(d_h1, x, W["norm1_w"], mu1, r1)
        G["norm1_b"] = Rg(db)
    G["norm1_w"] = Rg(dg)
    dx = R(d_y1 + d_n1)
    return y, dx, G


def stack_fwd_bwd_rounded(kind, n_heads, n_kv_heads, head_dim, cu, modes, weights_per_layer, x, dy, **kw):
    """A stack of such layers: each layer's rounded output is the next one's input, gradients travel back the
    same way.  (A layer's backward needs only its own input, so every layer's forward is simply run again.)"""
    xs = [np.asarray(x, dtype=f64)]
    zero = np.zeros_like(xs[0])
    for Wl in weights_per_layer[:-1]:
        y, _, _ = layer_fwd_bwd_rounded(kind, n_heads, n_kv_heads, head_dim, cu, modes, Wl, xs[-1], zero, **kw)
        xs.append(y)
    g = np.asarray(dy, dtype=f64)
    grads = [None] * len(weights_per_layer)
    y_out = None
    for l in range(len(weights_per_layer) - 1, -1, -1):
        y, g, grads[l] = layer_fwd_bwd_rounded(kind, n_heads, n_kv_heads, head_dim, cu, modes, weights_per_layer[l],
                                               xs[l], g, **kw)
        if y_out is None:
            y_out = y
    return y_out, g, grads
