"""The error metrics and bars every parity check uses.

Three per-tensor figures, all against the fp64 oracle:

  max_err  = max_i |got_i - ref_i| / max_i |ref_i|       "maximum relative error": the largest
             deviation relative to the tensor's scale.  Bar 2e-2 for bf16 storage.
  floor_err = max_i |got_i - ref_i| / max(|ref_i|, rms(ref))   element-wise relative error whose
             denominator is floored at the tensor's RMS (a plain |a-b|/|b| is unbounded on
             near-zero elements, whose error is set by the larger terms summed into them).
  l2_err   = ||got - ref||_2 / ||ref||_2.

Why floor_err cannot carry the 2e-2 bar for bf16.  One bf16 rounding of a tensor has l2_err
1.7e-3.  A layer that keeps its GEMM operands and outputs in bf16 rounds about ten tensors
between x and a gradient; each adds in quadrature (a product such as silu(g)*u adds twice, and
the attention backward pass amplifies the roundings of q and k), which gives l2_err of 3e-3 to
7e-3 for ANY such implementation: the oracle itself with roundings inserted at the storage
points shows it (tests/test_bf16_storage_floor.py; at the 7B layer's dimensions the same
emulation gives l2_err 7.2e-3 and floor_err 5.8e-2 on dx).  These errors are close to Gaussian,
so the largest of N of them is about sqrt(2 ln N) sigma: 4.9 sigma at N = 1.3e5, 6 sigma at
N = 9e7, i.e. floor_err of 2.5e-2 to 6e-2 with no mistake anywhere.  The floor also grows with the
layer's width, because N(0, 0.02^2) weights make the branches outweigh the residual stream and the
softmax peaky: the same emulation at the 72B layer's dimensions gives l2_err 1.05e-2 on y, half of it
from the roundings of h1, q and k alone.  floor_err is therefore held to 1e-1 and l2_err to 1.5e-2
(about 1.5x the storage floor of the widest workload; a wrong mask, index or operand shows as
l2_err >= 1e-1); max_err carries the 2e-2.  For fp32 storage all three are held to 1e-4.
"""
from __future__ import annotations

import numpy as np

F32, BF16 = 0, 1
BARS = {F32: {"max_err": 1e-4, "floor_err": 1e-4, "l2_err": 1e-4},
        BF16: {"max_err": 2e-2, "floor_err": 1e-1, "l2_err": 1.5e-2}}


def errors(got, ref) -> dict:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return {"max_err": 0.0, "floor_err": 0.0, "l2_err": 0.0}
    if not np.all(np.isfinite(got)):
        return {"max_err": float("inf"), "floor_err": float("inf"), "l2_err": float("inf")}
    diff = np.abs(got - ref)
    amax = float(np.max(np.abs(ref)))
    rms = float(np.sqrt(np.mean(ref * ref)))
    norm = float(np.linalg.norm(ref))
    if amax == 0.0:                      # an all-zero reference must be matched exactly
        bad = float(np.max(diff))
        return {"max_err": bad, "floor_err": bad, "l2_err": bad}
    return {"max_err": float(np.max(diff)) / amax,
            "floor_err": float(np.max(diff / np.maximum(np.abs(ref), rms))),
            "l2_err": float(np.linalg.norm(got - ref)) / norm}


def check(name: str, got, ref, dtype: int, bars: dict | None = None) -> dict:
    """Assert the three bars for one tensor; returns the measured errors."""
    e = errors(got, ref)
    b = dict(BARS[dtype])
    if bars:
        b.update(bars)
    for k, bar in b.items():
        assert e[k] <= bar, f"{name}: {k} {e[k]:.3e} > {bar:.1e}  (all: {e})"
    return e


def parity_error(got, ref) -> float:
    return errors(got, ref)["floor_err"]


def l2_error(got, ref) -> float:
    return errors(got, ref)["l2_err"]
