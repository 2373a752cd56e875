"""Cost of a pack for the paper's intra-microbatch reordering (Algorithm 1, Section 5.2), fitted to this library's
measured step time.

Algorithm 1 balances "sizes" over the data-parallel groups; the section's insight is that the size must be the
computation time a sample causes, not its token count.  For one transformer layer that time has a part linear in
the tokens (the GEMMs and the memory-bound kernels) and a part linear in the unmasked (query, key) pairs (attention),
both additive over the samples of a pack:

    step_ms(pack) = c0 + a * tokens + b * pairs          cost(sample) = a * tokens + b * pairs(sample)

The GEMMs work on tiles of 256 token rows, so a pack's `tokens` is its token count rounded up to whole tiles (a
5144-token pack runs as long as a 5376-token one); a sample's cost uses its own length, which keeps the costs additive.

`measure` times forward + backward of a pack with HIP events on the launch stream; `fit` solves the least-squares
problem; `sample_costs` turns segment lengths into the `sizes` argument of mmtrain_intra_reorder.

    python -m paper_2408_04275_amd.costmodel [--config 3] [--steps 10]      prints the fit as a text table

Nothing here is on the layer's hot path: it calls the C ABI through the same harness the tests use.
"""
from __future__ import annotations

import argparse
import sys
from typing import Iterable, List, Sequence, Tuple

import numpy as np

from . import workloads as wl


TILE_ROWS = 256          # rows of a GEMM tile: a pack costs what its token count rounded up to whole tiles costs


def pack_features(cu: np.ndarray, modes: np.ndarray) -> Tuple[int, int]:
    """(tokens rounded up to whole GEMM tiles, unmasked pairs) of a pack."""
    T = int(cu[-1])
    return -(-T // TILE_ROWS) * TILE_ROWS, wl.attention_pairs(cu, modes)


def measure(shape: wl.LayerShape, W, cu: np.ndarray, modes: np.ndarray, steps: int = 10, warmup: int = 3) -> float:
    """Median milliseconds of one forward + backward over `steps` steps (events on the stream the library launches on)."""
    import torch
    from .harness import LayerRunner
    T = int(cu[-1])
    r = LayerRunner(shape, W, cu, modes)
    x, dy = wl.make_activations(shape, T, 0)
    r.set_inputs(x, dy)
    for _ in range(warmup):
        r.step()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    marks[0].record()
    for i in range(steps):
        r.step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    return float(np.median([marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]))


def fit(features: Sequence[Tuple[int, int]], ms: Sequence[float]):
    """Least squares of ms = c0 + a * tokens + b * pairs.  Returns ((c0, a, b), relative residuals)."""
    A = np.array([[1.0, t, p] for t, p in features], dtype=np.float64)
    y = np.asarray(ms, dtype=np.float64)
    scale = np.array([1.0, 1e-3, 1e-7])                       # condition the columns (ms per kilo-token, per 1e7 pairs)
    coef, *_ = np.linalg.lstsq(A * scale, y, rcond=None)
    coef = coef * scale
    return tuple(float(c) for c in coef), (A @ coef - y) / y


def predict(coef, tokens: int, pairs: int) -> float:
    c0, a, b = coef
    return c0 + a * tokens + b * pairs


def sample_costs(coef, lengths: Iterable[int], bidir: Iterable[bool] = None) -> np.ndarray:
    """Cost in milliseconds that each sample (one segment of the given length) adds to a pack."""
    L = np.asarray(list(lengths), dtype=np.float64)
    bd = np.zeros(len(L), dtype=bool) if bidir is None else np.asarray(list(bidir), dtype=bool)
    pairs = np.where(bd, L * L, L * (L + 1) / 2)
    _, a, b = coef
    return a * L + b * pairs


def training_packs(config: int = 3) -> List[Tuple[str, np.ndarray, np.ndarray]]:
    """The packs the fit is made on: the workload's generator at seeds 0-4, the long-tailed pack, and seeded random
    packs of 2048 to 8192 tokens (the token count has to vary for its coefficient to be identified)."""
    packs = []
    for seed in range(5):
        cu, modes, _ = wl.make_segments(config, seed)
        packs.append((f"workload {config} seed {seed}", cu, modes))
    cu, modes, _ = wl.make_segments(4, wl.longtail_seed())
    packs.append(("long-tailed pack", cu, modes))
    rng = np.random.default_rng(2024)
    for T, n_seg in ((2048, 1), (2048, 6), (4096, 2), (4096, 9), (6144, 3), (6144, 12), (8192, 1), (8192, 24)):
        cu, modes = wl.random_segments(rng, T, n_seg)
        modes[:] = wl.CAUSAL
        packs.append((f"random pack T={T} S={n_seg}", cu, modes))
    return packs


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--config", type=int, default=3, choices=[3, 5])
    ap.add_argument("--steps", type=int, default=10)
    args = ap.parse_args(argv)
    shape = wl.SHAPES[args.config]
    W = wl.make_weights(shape, 0)
    packs = training_packs(args.config)
    feats, times = [], []
    for name, cu, modes in packs:
        feats.append(pack_features(cu, modes))
        times.append(measure(shape, W, cu, modes, args.steps))
    coef, res = fit(feats, times)
    print(f"layer {shape.name}: step_ms = {coef[0]:.4f} + {coef[1] * 1e3:.5f} * kilo-tokens + {coef[2] * 1e6:.5f} * mega-pairs")
    print("%-28s %8s %12s %10s %10s %8s" % ("pack", "tokens", "pairs", "ms", "fit ms", "resid"))
    for (name, _, _), (t, p), ms, r in zip(packs, feats, times, res):
        print("%-28s %8d %12d %10.3f %10.3f %+7.1f%%" % (name, t, p, ms, predict(coef, t, p), 100 * r))
    return 0


if __name__ == "__main__":
    sys.exit(main())
