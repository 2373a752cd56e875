"""GPU parity on seeded random layer shapes and packs: widths that are no multiple of a tile, every supported head
dimension, grouped-query ratios, packs with empty and one-token segments and random per-segment mask modes.  Small enough
for the fp64 oracle to take a fraction of a second per case."""
import numpy as np
import pytest

from paper_2408_04275_amd import workloads as wl
from util import compare_layer, gpu_run, oracle_run, say, storage_floors, summary

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = np.random.default_rng(7000 + seed)
    dtype = wl.BF16 if seed % 2 else wl.F32
    kind = wl.ENCODER if seed % 3 == 0 else wl.DECODER
    d = int(rng.choice([32, 64, 80, 96, 128] if dtype == wl.BF16 else [64, 128]))
    nh = int(rng.choice([1, 2, 3, 4, 6, 8]))
    nkv = nh if kind == wl.ENCODER else int(rng.choice([k for k in (1, 2, 3, 4, 6, 8) if nh % k == 0]))
    H = 16 * int(rng.integers(4, 25))
    F = 16 * int(rng.integers(4, 41))
    T = int(rng.integers(65, 900))
    n_cuts = int(rng.integers(0, 9))
    cuts = np.sort(rng.integers(0, T + 1, size=n_cuts))           # repeated cut points give empty segments
    cu = np.concatenate([[0], cuts, [T]]).astype(np.int32)
    S = len(cu) - 1
    modes = np.ones(S, dtype=np.uint8) if kind == wl.ENCODER else rng.integers(0, 2, size=S).astype(np.uint8)
    shape = wl.LayerShape(f"random-{seed}", kind, dtype, H, nh, nkv, d, F, T)
    return shape, cu, modes


@pytest.mark.parametrize("seed", range(24))
def test_random_shape(seed):
    shape, cu, modes = random_case(seed)
    W = wl.make_weights(shape, seed, std=0.05)
    x, dy = wl.make_activations(shape, int(cu[-1]), seed)
    ref = oracle_run(shape, cu, modes, W, x, dy)
    floors = storage_floors(shape, cu, modes, W, x, dy, ref)
    got = gpu_run(shape, cu, modes, W, x, dy)
    what = (f"random {seed}: kind={shape.kind} dtype={shape.dtype} H={shape.hidden} heads={shape.n_heads}/{shape.n_kv_heads}x"
            f"{shape.head_dim} F={shape.ffn_hidden} T={int(cu[-1])} segments={np.diff(cu).tolist()} ")
    errs = compare_layer(shape, got, ref, what, floors=floors)
    say(f"{what}: {summary(errs, floors)}")
