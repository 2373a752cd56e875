"""fp64 CPU oracle for one transformer layer over a packed microbatch.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
path is checked against.  It shares no code with the HIP path and must never be
imported by it: only the tests, the smoke check and the benchmark's CPU-baseline
leg may call it.

What it computes.  The paper (Section 2.1, Section 2.2, Section 7 "Models",
Table 2) names the layers -- a Llama-style LLM-backbone decoder layer and a
ViT-style modality-encoder layer -- and the input form -- a fixed-length
sequence made by interleaving text and image subsequences (Section 2.3,
Section 7 "Datasets") -- but not their arithmetic.  The arithmetic below is the
standard public definition of those layers:

  decoder:  y1 = x + Wo . attn(rope(Wqkv . rmsnorm(x)))        (pre-norm, no biases)
            y  = y1 + Wdown . (silu(Wgate . h2) * (Wup . h2)),  h2 = rmsnorm(y1)
  encoder:  the same skeleton with LayerNorm (gain and bias), biases on all
            four linears, no rotary embedding, and an erf-GELU two-matrix MLP.

A pack of T tokens is cut into S segments by cu_seqlens (cu[0] = 0, cu[S] = T).
Attention never crosses a segment boundary.  Inside a segment it is causal
(key j <= query i) or bidirectional, per segment.  Rotary positions restart at
0 in every segment and pair feature i with feature i + d/2 ("half-split").
Grouped-query attention: query head h reads key/value head h // (nh / nkv).

Everything is float64, nothing is rounded, nothing is tiled or fused: full
score matrices per (segment, head), softmax by subtracting the row maximum,
exponentiating and dividing by the row sum.  Matrix products use numpy's matmul
as a library step.  The backward pass is the chain rule written out operator by
operator in the reverse order of the forward pass.

Parity pins (tests/test_oracle_*.py): brute-force scalar-loop attention on tiny
inputs; finite differences of every input and parameter; an independent
float64 autograd evaluation of the same layer through PyTorch CPU library
routines; packed == unpacked; closed forms (length-1 segments, equal keys, zero
output projections); rotary, masking, segment-order and grouped-query
invariants.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np
from scipy.special import erf

DECODER, ENCODER = 0, 1
CAUSAL, BIDIR = 0, 1

f64 = np.float64


# ----------------------------------------------------------------------------
# segments
# ----------------------------------------------------------------------------
def positions(cu: np.ndarray) -> np.ndarray:
    """pos[t] = t - cu[seg(t)]: the index of token t inside its own segment."""
    T = int(cu[-1])
    pos = np.zeros(T, dtype=np.int64)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        pos[a:b] = np.arange(b - a)
    return pos


# ----------------------------------------------------------------------------
# normalisation
# ----------------------------------------------------------------------------
def rmsnorm_fwd(x, g, eps):
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1) + eps)          # [T]
    return x * r[:, None] * g[None, :], r


def rmsnorm_bwd(dout, x, g, r):
    xhat = x * r[:, None]
    ghat = dout * g[None, :]
    dg = np.sum(dout * xhat, axis=0)
    din = r[:, None] * (ghat - xhat * np.mean(ghat * xhat, axis=-1, keepdims=True))
    return din, dg


def layernorm_fwd(x, g, b, eps):
    mu = np.mean(x, axis=-1)
    var = np.mean((x - mu[:, None]) ** 2, axis=-1)            # biased variance
    r = 1.0 / np.sqrt(var + eps)
    return (x - mu[:, None]) * r[:, None] * g[None, :] + b[None, :], mu, r


def layernorm_bwd(dout, x, g, mu, r):
    xhat = (x - mu[:, None]) * r[:, None]
    ghat = dout * g[None, :]
    dg = np.sum(dout * xhat, axis=0)
    db = np.sum(dout, axis=0)
    din = r[:, None] * (ghat - np.mean(ghat, axis=-1, keepdims=True)
                        - xhat * np.mean(ghat * xhat, axis=-1, keepdims=True))
    return din, dg, db


# ----------------------------------------------------------------------------
# rotary position embedding (half-split pairing)
# ----------------------------------------------------------------------------
def rope(u, pos, base, inverse=False):
    """Rotate every head of u [T, n, d] by angle pos[t] * base^(-2i/d) on the pair (i, i + d/2).

    inverse=True rotates by the negative angle, which is the transpose of the
    forward rotation and therefore its backward pass.
    """
    T, n, d = u.shape
    half = d // 2
    theta = base ** (-2.0 * np.arange(half, dtype=f64) / d)   # [d/2]
    phi = pos.astype(f64)[:, None] * theta[None, :]           # [T, d/2]
    c, s = np.cos(phi)[:, None, :], np.sin(phi)[:, None, :]
    if inverse:
        s = -s
    lo, hi = u[..., :half], u[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


# ----------------------------------------------------------------------------
# segment-masked attention
# ----------------------------------------------------------------------------
def _probabilities(qs, ks, scale, mode):
    """Softmax of the masked scaled scores of one (segment, head); also log-sum-exp per row."""
    S = (qs @ ks.T) * scale                                   # [L, L]
    if mode == CAUSAL:
        L = S.shape[0]
        S = np.where(np.tril(np.ones((L, L), dtype=bool)), S, -np.inf)
    m = np.max(S, axis=-1, keepdims=True)
    E = np.exp(S - m)
    Z = np.sum(E, axis=-1, keepdims=True)
    return E / Z, (m + np.log(Z))[:, 0]


def attention_fwd(q, k, v, cu, modes, scale):
    """q [T, nh, d], k and v [T, nkv, d]  ->  o [T, nh, d], lse [nh, T]."""
    T, nh, d = q.shape
    group = nh // k.shape[1]
    o = np.zeros((T, nh, d), dtype=f64)
    lse = np.zeros((nh, T), dtype=f64)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        for h in range(nh):
            P, l = _probabilities(q[a:b, h], k[a:b, h // group], scale, int(modes[s]))
            o[a:b, h] = P @ v[a:b, h // group]
            lse[h, a:b] = l
    return o, lse


def attention_bwd(do, q, k, v, cu, modes, scale):
    """Gradients of attention_fwd with respect to q, k, v given do [T, nh, d]."""
    T, nh, d = q.shape
    group = nh // k.shape[1]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        for h in range(nh):
            g = h // group
            P, _ = _probabilities(q[a:b, h], k[a:b, g], scale, int(modes[s]))
            dO = do[a:b, h]
            dv[a:b, g] += P.T @ dO
            dP = dO @ v[a:b, g].T
            D = np.sum(P * dP, axis=-1, keepdims=True)
            dS = P * (dP - D)
            dq[a:b, h] = (dS @ k[a:b, g]) * scale
            dk[a:b, g] += (dS.T @ q[a:b, h]) * scale
    return dq, dk, dv


# ----------------------------------------------------------------------------
# activations
# ----------------------------------------------------------------------------
def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


# ----------------------------------------------------------------------------
# the layer
# ----------------------------------------------------------------------------
def _f64(d: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: np.asarray(v, dtype=f64) for k, v in d.items() if v is not None}


def layer_fwd(kind: int, n_heads: int, n_kv_heads: int, head_dim: int, cu, modes,
              weights: Dict[str, np.ndarray], x, eps: float = 1e-5, rope_base: float = 10000.0,
              softmax_scale: float = 0.0) -> Tuple[np.ndarray, dict]:
    """Forward pass.  Returns (y, cache); cache holds every intermediate the backward pass reads."""
    W = _f64(weights)
    x = np.asarray(x, dtype=f64)
    T, H = x.shape
    nh, nkv, d = n_heads, n_kv_heads, head_dim
    nq, nk = nh * d, nkv * d
    scale = softmax_scale if softmax_scale > 0 else 1.0 / np.sqrt(d)
    cu = np.asarray(cu, dtype=np.int64)
    c = {"x": x, "cu": cu, "modes": np.asarray(modes), "scale": scale, "kind": kind,
         "dims": (nh, nkv, d), "eps": eps, "rope_base": rope_base}

    # --- attention block
    if kind == DECODER:
        h1, c["r1"] = rmsnorm_fwd(x, W["norm1_w"], eps)
    else:
        h1, c["mu1"], c["r1"] = layernorm_fwd(x, W["norm1_w"], W["norm1_b"], eps)
    qkv = h1 @ W["w_qkv"].T
    if kind == ENCODER:
        qkv = qkv + W["b_qkv"][None, :]
    q = qkv[:, :nq].reshape(T, nh, d)
    k = qkv[:, nq:nq + nk].reshape(T, nkv, d)
    v = qkv[:, nq + nk:].reshape(T, nkv, d)
    if kind == DECODER:
        pos = positions(cu)
        q, k = rope(q, pos, rope_base), rope(k, pos, rope_base)
        c["pos"] = pos
    o, lse = attention_fwd(q, k, v, cu, modes, scale)
    o2 = o.reshape(T, nq)
    y1 = x + o2 @ W["w_o"].T
    if kind == ENCODER:
        y1 = y1 + W["b_o"][None, :]
    c.update(h1=h1, q=q, k=k, v=v, o=o2, lse=lse, y1=y1)

    # --- MLP block
    if kind == DECODER:
        h2, c["r2"] = rmsnorm_fwd(y1, W["norm2_w"], eps)
        F = W["w_fc2"].shape[1]
        gu = h2 @ W["w_fc1"].T                                 # [T, 2F]: gate columns, then up columns
        gate, up = gu[:, :F], gu[:, F:]
        m = gate * sigmoid(gate) * up
        c.update(gate=gate, up=up)
    else:
        h2, c["mu2"], c["r2"] = layernorm_fwd(y1, W["norm2_w"], W["norm2_b"], eps)
        z = h2 @ W["w_fc1"].T + W["b_fc1"][None, :]
        m = gelu(z)
        c.update(z=z)
    y = y1 + m @ W["w_fc2"].T
    if kind == ENCODER:
        y = y + W["b_fc2"][None, :]
    c.update(h2=h2, m=m)
    return y, c


def layer_bwd(weights: Dict[str, np.ndarray], cache: dict, dy) -> Tuple[np.ndarray, Dict[str, np.ndarray]]:
    """Backward pass.  Returns (dx, grads) with grads keyed like the weights."""
    W = _f64(weights)
    c = cache
    kind = c["kind"]
    nh, nkv, d = c["dims"]
    nq, nk = nh * d, nkv * d
    dy = np.asarray(dy, dtype=f64)
    T = dy.shape[0]
    G: Dict[str, np.ndarray] = {}

    # --- MLP block:  y = y1 + m . Wfc2^T (+ b)
    d_m = dy @ W["w_fc2"]
    G["w_fc2"] = dy.T @ c["m"]
    if kind == ENCODER:
        G["b_fc2"] = np.sum(dy, axis=0)
    if kind == DECODER:
        gate, up = c["gate"], c["up"]
        sg = sigmoid(gate)
        d_gate = d_m * up * sg * (1.0 + gate * (1.0 - sg))
        d_up = d_m * gate * sg
        d_pre = np.concatenate([d_gate, d_up], axis=1)
    else:
        d_pre = d_m * gelu_grad(c["z"])
        G["b_fc1"] = np.sum(d_pre, axis=0)
    d_h2 = d_pre @ W["w_fc1"]
    G["w_fc1"] = d_pre.T @ c["h2"]
    if kind == DECODER:
        d_n2, G["norm2_w"] = rmsnorm_bwd(d_h2, c["y1"], W["norm2_w"], c["r2"])
    else:
        d_n2, G["norm2_w"], G["norm2_b"] = layernorm_bwd(d_h2, c["y1"], W["norm2_w"], c["mu2"], c["r2"])
    d_y1 = dy + d_n2

    # --- attention block:  y1 = x + o . Wo^T (+ b)
    d_o = d_y1 @ W["w_o"]
    G["w_o"] = d_y1.T @ c["o"]
    if kind == ENCODER:
        G["b_o"] = np.sum(d_y1, axis=0)
    dq, dk, dv = attention_bwd(d_o.reshape(T, nh, d), c["q"], c["k"], c["v"], c["cu"], c["modes"], c["scale"])
    if kind == DECODER:
        dq = rope(dq, c["pos"], c["rope_base"], inverse=True)
        dk = rope(dk, c["pos"], c["rope_base"], inverse=True)
    d_qkv = np.concatenate([dq.reshape(T, nq), dk.reshape(T, nk), dv.reshape(T, nk)], axis=1)
    d_h1 = d_qkv @ W["w_qkv"]
    G["w_qkv"] = d_qkv.T @ c["h1"]
    if kind == ENCODER:
        G["b_qkv"] = np.sum(d_qkv, axis=0)
    if kind == DECODER:
        d_n1, G["norm1_w"] = rmsnorm_bwd(d_h1, c["x"], W["norm1_w"], c["r1"])
    else:
        d_n1, G["norm1_w"], G["norm1_b"] = layernorm_bwd(d_h1, c["x"], W["norm1_w"], c["mu1"], c["r1"])
    dx = d_y1 + d_n1
    return dx, G


def layer_fwd_bwd(kind, n_heads, n_kv_heads, head_dim, cu, modes, weights, x, dy, **kw):
    """Convenience: forward then backward.  Returns (y, dx, grads, cache)."""
    y, cache = layer_fwd(kind, n_heads, n_kv_heads, head_dim, cu, modes, weights, x, **kw)
    dx, grads = layer_bwd(weights, cache, dy)
    return y, dx, grads, cache


# ----------------------------------------------------------------------------
# a stack of layers (Section 4.2: the backbone is a sequence of identical transformer layers)
# ----------------------------------------------------------------------------
def stack_fwd(kind, n_heads, n_kv_heads, head_dim, cu, modes, weights_per_layer, x, **kw):
    """y = layer[n-1](... layer[0](x)).  Returns (y, caches), one cache per layer."""
    caches = []
    h = np.asarray(x, dtype=f64)
    for W in weights_per_layer:
        h, cache = layer_fwd(kind, n_heads, n_kv_heads, head_dim, cu, modes, W, h, **kw)
        caches.append(cache)
    return h, caches


def stack_bwd(weights_per_layer, caches, dy):
    """Chain rule down the stack.  Returns (dx, grads), grads being one dictionary per layer."""
    g = np.asarray(dy, dtype=f64)
    grads = [None] * len(caches)
    for l in range(len(caches) - 1, -1, -1):
        g, grads[l] = layer_bwd(weights_per_layer[l], caches[l], g)
    return g, grads
