"""The error metrics and bars every parity check uses.

Per-tensor figures, all against the fp64 oracle:

  max_err   = max_i |got_i - ref_i| / max_i |ref_i|      "maximum relative error": the largest
              deviation relative to the tensor's scale.  Bar 2e-2 for bf16 storage (the stated tolerance).
  floor_err = max_i |got_i - ref_i| / max(|ref_i|, rms(ref))   element-wise relative error whose
              denominator is floored at the tensor's RMS (a plain |a-b|/|b| is unbounded on
              near-zero elements, whose error is set by the larger terms summed into them).
  l2_err    = ||got - ref||_2 / ||ref||_2.
  big_err   = max over the elements with |ref_i| >= rms(ref) of |got_i - ref_i| / |ref_i|: the plain
              element-wise relative error on every element that is not small against its tensor
              (reported, and never larger than floor_err).

History of the bars.  The first bar tried was floor_err <= 2e-2.  The first GPU run read 3.1e-2 to 4.8e-2 on
dq and on several weight gradients with every product correct to fp32 rounding, which led to the question of what
bf16 storage alone costs.  The answer is computed, not assumed: oracle/bf16_storage.py is the fp64 oracle with a
rounding at every point where a bf16 layer stores a tensor; compared with the unrounded oracle it gives each
tensor's storage floor -- floor_err 4e-2 / l2_err 5e-3 at small widths, floor_err 6e-2 / l2_err 7e-3 on dx at the
7B width, 1.1e-1 to 1.5e-1 / 1.4e-2 at the 72B width (N(0, 0.02^2) weights make the branches outweigh the residual
stream as the width grows, and the largest of N near-Gaussian errors grows like sqrt(2 ln N)).  No implementation that
keeps GEMM operands in bf16 can be below that floor, so:

  * max_err <= 2e-2 carries the stated tolerance, always;
  * where the storage floor of the very case is known -- tests/golden/bf16_floor.json for the full-size
    workloads (written from the oracle alone by tests/golden/make_bf16_floor.py), computed on the spot for the
    small layer cases -- l2_err is held to 1.25 x and floor_err to 1.5 x that tensor's floor (FLOOR_MARGIN, bars_from_floor);
  * operator-level checks (one GEMM, attention alone), which have no layer to emulate, use the flat bars of
    BARS: 1e-1 and 1.5e-2, above every floor measured at small width (tests/test_bf16_storage_floor.py).

For fp32 storage all three figures are held to 1e-4.
"""
from __future__ import annotations

import numpy as np

F32, BF16 = 0, 1
BARS = {F32: {"max_err": 1e-4, "floor_err": 1e-4, "l2_err": 1e-4},
        BF16: {"max_err": 2e-2, "floor_err": 1e-1, "l2_err": 1.5e-2}}
# A tensor may deviate from the fp64 oracle by this multiple of what bf16 storage alone costs it.  l2_err is a stable
# statistic: the HIP path reads 0.95 to 1.1 times the emulated floor on every tensor seen, and is held to 1.25 times.
# floor_err is the largest of N ratios, and the HIP path's roundings are not the emulation's bit for bit (fp32 against fp64
# accumulation and a hardware exponential flip a share of them), so it is the maximum of another draw of the same errors:
# on a gain gradient of 128 to 272 elements the two maxima differ by up to 1.44 with l2_err equal to 3 % (the first margin
# tried was 1.3 on both figures; seven small cases read 1.32 to 1.44 on such vectors and on nothing else).
FLOOR_MARGIN = {"l2_err": 1.25, "floor_err": 1.5}
# A tensor whose storage floor is below this is held to this (fp32 accumulation order shows at 1e-6 to 1e-5).
FLOOR_MIN = {"floor_err": 1e-4, "l2_err": 2e-5}


def errors(got, ref) -> dict:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    zero = {"max_err": 0.0, "floor_err": 0.0, "l2_err": 0.0, "big_err": 0.0}
    if ref.size == 0:
        return zero
    if not np.all(np.isfinite(got)):
        return {k: float("inf") for k in zero}
    diff = np.abs(got - ref)
    aref = np.abs(ref)
    amax = float(np.max(aref))
    rms = float(np.sqrt(np.mean(ref * ref)))
    norm = float(np.linalg.norm(ref))
    if amax == 0.0:                      # an all-zero reference must be matched exactly
        bad = float(np.max(diff))
        return {k: bad for k in zero}
    big = aref >= rms
    return {"max_err": float(np.max(diff)) / amax,
            "floor_err": float(np.max(diff / np.maximum(aref, rms))),
            "l2_err": float(np.sqrt(np.sum(diff * diff))) / norm,
            "big_err": float(np.max(diff[big] / aref[big])) if np.any(big) else 0.0}


def bars_from_floor(floor: dict) -> dict:
    """Bars of one bf16 tensor from its storage floor (the `errors` of the rounded oracle against the plain one)."""
    return {"max_err": BARS[BF16]["max_err"],
            "floor_err": FLOOR_MARGIN["floor_err"] * max(floor["floor_err"], FLOOR_MIN["floor_err"]),
            "l2_err": FLOOR_MARGIN["l2_err"] * max(floor["l2_err"], FLOOR_MIN["l2_err"])}


def check(name: str, got, ref, dtype: int, bars: dict | None = None, floor: dict | None = None) -> dict:
    """Assert the bars for one tensor; returns the measured errors.  `floor` (bf16 only) replaces the flat
    auxiliary bars by FLOOR_MARGIN times the tensor's storage floor; `bars` overrides single entries."""
    e = errors(got, ref)
    b = dict(BARS[dtype])
    if floor is not None and dtype == BF16:
        b = bars_from_floor(floor)
    if bars:
        b.update(bars)
    for k, bar in b.items():
        assert e[k] <= bar, f"{name}: {k} {e[k]:.3e} > {bar:.2e}  (all: {e}; storage floor: {floor})"
    return e


def parity_error(got, ref) -> float:
    return errors(got, ref)["floor_err"]


def l2_error(got, ref) -> float:
    return errors(got, ref)["l2_err"]
