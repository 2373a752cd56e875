"""Seeded synthetic workloads: layer shapes, packed-segment layouts and tensors.

This module only *draws inputs*.  It holds none of the layer's arithmetic, so
both the CPU oracle's tests and the HIP path's tests can feed on it without
sharing any code of the method itself.

The paper trains on fixed-length 8192-token sequences made by interleaving text
subsequences and image subsequences (one token per 16x16 patch), and reports the
subsequence sizes as highly skewed (Section 2.3 "Data Heterogeneity", Section 7
"Datasets").  The dataset itself is not available here; the generators below
produce packs with that structure from the length distributions each workload
names.  Layer shapes for the decoder workloads follow the paper's Table 2
(LLM backbone configurations).

Everything is numpy on the host.  Tensors are returned as float32 arrays whose
values are already rounded to the workload's storage dtype (bf16 or fp32), so
the oracle (which promotes to fp64) and the GPU path (which converts to its
storage dtype exactly) start from identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

DECODER, ENCODER = 0, 1
CAUSAL, BIDIR = 0, 1
F32, BF16 = 0, 1


@dataclass(frozen=True)
class LayerShape:
    name: str
    kind: int          # DECODER | ENCODER
    dtype: int         # F32 | BF16 (storage dtype of activations, weights, grads)
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_hidden: int
    max_tokens: int
    norm_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def nq(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def nkv(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def nqkv(self) -> int:
        return self.nq + 2 * self.nkv

    @property
    def fc1_rows(self) -> int:
        # decoder: gate rows then up rows; encoder: one matrix
        return 2 * self.ffn_hidden if self.kind == DECODER else self.ffn_hidden


# The five workloads, in the order they are listed in BASELINE.json ("configs").
SHAPES: Dict[int, LayerShape] = {
    1: LayerShape("tiny-decoder-fp32", DECODER, F32, 256, 4, 4, 64, 688, 512),
    2: LayerShape("vit-encoder-bf16", ENCODER, BF16, 1024, 16, 16, 64, 4096, 16384),
    3: LayerShape("7b-decoder-bf16", DECODER, BF16, 4096, 32, 32, 128, 11008, 8192),
    4: LayerShape("7b-decoder-bf16-longtail", DECODER, BF16, 4096, 32, 32, 128, 11008, 8192),
    5: LayerShape("72b-decoder-bf16-gqa", DECODER, BF16, 8192, 64, 8, 128, 29568, 8192),
    # 6 is not one of the benchmark's five workloads: the published ViT-Huge encoder shape (the paper names its
    # encoder "ViT-Huge (0.63B)" without dimensions): hidden 1280, 16 heads of 80, MLP 5120; packs as for 2
    6: LayerShape("vit-huge-encoder-bf16", ENCODER, BF16, 1280, 16, 16, 80, 5120, 16384),
}


def scaled_shape(shape: LayerShape, **kw) -> LayerShape:
    """A copy of `shape` with some fields replaced (for reduced-size parity cases)."""
    return replace(shape, **kw)


# ----------------------------------------------------------------------------
# dtype rounding (input preparation only)
# ----------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    bits = bits + 0x7FFF + ((bits >> 16) & 1)
    out = ((bits >> 16) << 16).astype(np.uint32)
    return out.view(np.float32).reshape(a.shape)


def round_to(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.asarray(a, dtype=np.float32)
    return round_bf16(a) if dtype == BF16 else a


# ----------------------------------------------------------------------------
# segment layouts
# ----------------------------------------------------------------------------
def _cu(lengths: List[int]) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return cu


def _interleaved_pack(rng: np.random.Generator, total: int) -> Tuple[List[int], List[str]]:
    """Text runs (uniform 64..2048) interleaved with 576-token image spans (count ~ Poisson(4))."""
    n_img = int(min(rng.poisson(4.0), (total - 64) // 576))
    budget = total - 576 * n_img
    text: List[int] = []
    while budget > 0:
        L = int(rng.integers(64, 2049))
        L = min(L, budget)
        budget -= L
        if L < 64 and text:
            text[-1] += L          # a short remainder joins the previous text run
        else:
            text.append(L)
    spans = [(L, "text") for L in text] + [(576, "image")] * n_img
    order = rng.permutation(len(spans))
    spans = [spans[i] for i in order]
    return [s[0] for s in spans], [s[1] for s in spans]


def _longtail_pack(rng: np.random.Generator, total: int) -> Tuple[List[int], List[str]]:
    """Segment lengths ~ round(LogNormal(6, 1.2)) clipped to [16, total], drawn until `total` is filled."""
    lengths: List[int] = []
    left = total
    while left > 0:
        L = int(np.clip(np.rint(rng.lognormal(6.0, 1.2)), 16, total))
        L = min(L, left)
        lengths.append(L)
        left -= L
    return lengths, ["text"] * len(lengths)


def longtail_seed(total: int = 8192, dominant: int = 6000) -> int:
    """Smallest seed >= 0 whose long-tailed pack holds one segment of at least `dominant` tokens."""
    seed = 0
    while True:
        lengths, _ = _longtail_pack(np.random.default_rng(seed), total)
        if max(lengths) >= dominant:
            return seed
        seed += 1


def make_segments(config: int, seed: int = 0, image_bidir: bool = False, group: str = "span"):
    """Segment layout of one packed microbatch.

    Returns (cu_seqlens int32 [S+1], modes uint8 [S], kinds list[str]).
    `image_bidir` (decoder workloads only) gives image spans bidirectional
    attention instead of causal; encoder packs are always bidirectional.
    `group` says what a "document" is for the decoder workloads 3-5: "span" (default) makes every text run and
    every image span a segment of its own; "sample" takes the whole fixed-length sequence as ONE causal document,
    the paper's training sample (Section 2.3: a sample is one sequence of interleaved subsequences), in which
    text attends to the images in front of it.  Same spans, same tokens; only cu_seqlens and with it the number
    of unmasked pairs (the attention FLOP count) change.
    """
    rng = np.random.default_rng(seed)
    if config == 1:
        lengths, kinds = [128, 96, 160, 128], ["text", "text", "text", "image"]
    elif config in (2, 6):
        lengths = [int(v) for v in rng.choice([256, 576, 1024], size=16)]
        kinds = ["image"] * 16
    elif config in (3, 5):
        lengths, kinds = _interleaved_pack(rng, SHAPES[config].max_tokens)
    elif config == 4:
        lengths, kinds = _longtail_pack(rng, SHAPES[4].max_tokens)
    else:
        raise ValueError(f"unknown config {config}")
    if group not in ("span", "sample"):
        raise ValueError(f"unknown grouping {group!r}")
    if group == "sample" and config in (3, 4, 5):
        lengths, kinds = [int(sum(lengths))], ["sample"]
    modes = np.zeros(len(lengths), dtype=np.uint8)
    for i, k in enumerate(kinds):
        if SHAPES[config].kind == ENCODER or (image_bidir and k == "image"):
            modes[i] = BIDIR
    return _cu(lengths), modes, kinds


def random_segments(rng: np.random.Generator, total: int, n_seg: int, with_empty: bool = False):
    """A random split of `total` tokens into `n_seg` segments with random mask modes (for small parity cases)."""
    if with_empty:
        cuts = np.sort(rng.integers(0, total + 1, size=n_seg - 1))
    else:
        # distinct interior boundaries, so no segment is empty
        cuts = np.sort(rng.choice(np.arange(1, total), size=n_seg - 1, replace=False))
    cu = np.concatenate([[0], cuts, [total]]).astype(np.int32)
    modes = rng.integers(0, 2, size=n_seg).astype(np.uint8)
    return cu, modes


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
WEIGHT_NAMES = ("norm1_w", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "norm2_w", "norm2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def weight_shapes(shape: LayerShape) -> Dict[str, Tuple[int, ...]]:
    """Shapes of the layer's parameters; encoder-only entries are absent for the decoder."""
    H, F1, F = shape.hidden, shape.fc1_rows, shape.ffn_hidden
    out = {
        "norm1_w": (H,), "w_qkv": (shape.nqkv, H), "w_o": (H, shape.nq),
        "norm2_w": (H,), "w_fc1": (F1, H), "w_fc2": (H, F),
    }
    if shape.kind == ENCODER:
        out.update({"norm1_b": (H,), "b_qkv": (shape.nqkv,), "b_o": (H,),
                    "norm2_b": (H,), "b_fc1": (F1,), "b_fc2": (H,)})
    return out


def make_weights(shape: LayerShape, seed: int = 0, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Matrices and biases ~ N(0, std^2); norm gains 1 + N(0, std^2); rounded to the storage dtype."""
    rng = np.random.default_rng([seed, 101])
    out = {}
    for name, shp in weight_shapes(shape).items():
        a = rng.standard_normal(shp, dtype=np.float32) * np.float32(std)
        if name in ("norm1_w", "norm2_w"):
            a = a + np.float32(1.0)
        out[name] = round_to(a, shape.dtype)
    return out


def make_activations(shape: LayerShape, total_tokens: int, seed: int = 0):
    """x and the upstream gradient dy, both ~ N(0,1), rounded to the storage dtype."""
    rng = np.random.default_rng([seed, 202])
    x = round_to(rng.standard_normal((total_tokens, shape.hidden), dtype=np.float32), shape.dtype)
    dy = round_to(rng.standard_normal((total_tokens, shape.hidden), dtype=np.float32), shape.dtype)
    return x, dy


# ----------------------------------------------------------------------------
# model FLOPs (the convention every reported TFLOP/s uses)
# ----------------------------------------------------------------------------
def attention_pairs(cu: np.ndarray, modes: np.ndarray) -> int:
    """Number of unmasked (query, key) pairs in the pack."""
    L = np.diff(np.asarray(cu, dtype=np.int64))
    m = np.asarray(modes)
    return int(np.sum(np.where(m == BIDIR, L * L, L * (L + 1) // 2)))


def model_flops(shape: LayerShape, cu: np.ndarray, modes: np.ndarray) -> Dict[str, float]:
    """Forward and forward+backward model FLOPs.

    GEMMs: 2*T*K*N forward, twice that again backward (input and weight
    gradients).  Attention: only unmasked pairs, 4*d per pair per query head
    forward and 8*d backward.  Recomputation, masked-tile waste and elementwise
    work are not credited.
    """
    T = int(cu[-1])
    H, F = shape.hidden, shape.ffn_hidden
    gemm_params = shape.nqkv * H + H * shape.nq + shape.fc1_rows * H + H * F
    gemm_fwd = 2.0 * T * gemm_params
    attn_fwd = 4.0 * shape.head_dim * shape.n_heads * attention_pairs(cu, modes)
    return {"gemm_fwd": gemm_fwd, "attn_fwd": attn_fwd,
            "fwd": gemm_fwd + attn_fwd, "fwd_bwd": 3.0 * (gemm_fwd + attn_fwd)}


def hardware_flops(shape: LayerShape, cu: np.ndarray, modes: np.ndarray) -> Dict[str, float]:
    """FLOPs the matrix cores actually execute for one forward + backward, as opposed to model_flops: the GEMMs
    as they are, attention with everything the tiled kernels compute and model FLOPs do not credit --
    the masked part of every 32 x 32 block that is not skipped as a whole (diagonal and segment-boundary blocks),
    the recomputation of the scores in both backward kernels (dQ kernel: scores, dP, dQ = 6 d per pair;
    dK/dV kernel: scores, dP, dV, dK = 8 d per pair) and the zero padding of head dimensions that are not 64 or 128.
    The block rules restate the kernels' launch geometry: forward and dQ: 256 queries per workgroup walk the
    keys [first query's first key, last query's last key) in 64-key steps, and a wavefront (32 queries) runs a 32-key
    block unless the block lies outside [its first query's first key, its last query's last key); dK/dV: 128 keys per
    workgroup, 32 per wavefront, walk the queries in 64-query steps, skipping per block (64-wide heads) or per step
    (wider heads)."""
    cu = np.asarray(cu, dtype=np.int64)
    T = int(cu[-1])
    d_pad = 64 if shape.head_dim <= 64 else 128
    seg = np.repeat(np.arange(len(cu) - 1), np.diff(cu))
    start, end = cu[seg], cu[seg + 1]
    bidir = np.asarray(modes)[seg] == BIDIR
    tok = np.arange(T)
    q_lo, q_hi = start, np.where(bidir, end, tok + 1)             # keys a query sees
    k_lo, k_hi = np.where(bidir, start, tok), end                 # queries that see a key
    blocks_q = 0                                                  # 32 x 32 blocks run by the forward / dQ kernels
    for q0 in range(0, T, 256):
        kbeg, kend = int(q_lo[q0]), int(q_hi[min(q0 + 256, T) - 1])
        for w0 in range(q0, min(q0 + 256, T), 32):
            w1 = min(w0 + 32, T) - 1
            lo, hi = int(q_lo[w0]), int(q_hi[w1])
            for kb in range(kbeg, kend + (-(kend - kbeg)) % 64, 32):
                blocks_q += kb < hi and kb + 32 > lo
    blocks_k = 0                                                  # ... by the dK/dV kernel
    per_step = d_pad > 64
    for k0 in range(0, T, 128):
        qbeg, qend = int(k_lo[k0]), int(k_hi[min(k0 + 128, T) - 1])
        for w0 in range(k0, min(k0 + 128, T), 32):
            w1 = min(w0 + 32, T) - 1
            lo, hi = int(k_lo[w0]), int(k_hi[w1])
            for qt in range(qbeg, qend, 64):
                if per_step:
                    blocks_k += 2 * (qt < hi and qt + 64 > lo)
                else:
                    blocks_k += (qt < hi and qt + 32 > lo) + (qt + 32 < hi and qt + 64 > lo)
    pairs_q, pairs_k = 1024.0 * blocks_q, 1024.0 * blocks_k
    nh = shape.n_heads
    m = model_flops(shape, cu, modes)
    attn_fwd = 4.0 * d_pad * nh * pairs_q
    attn_bwd = 6.0 * d_pad * nh * pairs_q + 8.0 * d_pad * nh * pairs_k
    return {"gemm_fwd_bwd": 3.0 * m["gemm_fwd"], "attn_fwd": attn_fwd, "attn_bwd": attn_bwd,
            "fwd_bwd": 3.0 * m["gemm_fwd"] + attn_fwd + attn_bwd}
