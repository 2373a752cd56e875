"""The full-size parity cases: which workload, seed, mask variant and (for sampled cases) which segments.

Shared by tests/test_gpu_full.py (the GPU side) and tests/golden/make_bf16_floor.py (which writes the bf16
storage floor of every case from the oracle alone), so that both always talk about the same inputs.
Input drawing only: no arithmetic of the layer lives here.
"""
import hashlib

import numpy as np

from paper_2408_04275_amd import workloads as wl

# name -> (workload, seed or None for the long-tail seed, image spans bidirectional, sampled segments or 0 = whole pack)
CASES = {
    "config2_full": (2, 0, False, 0),
    "config2_worst_case_16x1024": (2, "worst", False, 0),
    "config6_vit_huge_full": (6, 1, False, 0),
    "config3_full": (3, 0, False, 0),
    "config4_longtail_full": (4, None, False, 0),
    "config3_image_bidir_sampled": (3, 0, True, 4),
    "config5_sampled": (5, 0, False, 3),
    "config5_full": (5, 0, False, 0),
}


def segments(name):
    """(shape, seed, cu, modes, picked segments or None) of a case."""
    config, seed, image_bidir, n_sample = CASES[name]
    shape = wl.SHAPES[config]
    if seed == "worst":                   # workload 2's fixed worst case: sixteen images of 1024 patches, 16384 tokens
        seed = 0
        cu = (np.arange(17) * 1024).astype(np.int32)
        modes = np.full(16, wl.BIDIR, dtype=np.uint8)
    else:
        if seed is None:
            seed = wl.longtail_seed()
        cu, modes, _ = wl.make_segments(config, seed, image_bidir=image_bidir)
    pick = None
    if n_sample:
        S = len(cu) - 1
        rng = np.random.default_rng([seed, 303])
        pick = sorted(set(rng.choice(S, size=min(n_sample, S), replace=False).tolist()) | {S - 1})
    return shape, seed, cu, modes, pick


def inputs(name):
    """Everything both sides need.  For a sampled case `rows` are the tokens of the picked segments and
    (sub_cu, sub_modes) the pack made of those segments alone; otherwise rows is None."""
    shape, seed, cu, modes, pick = segments(name)
    T = int(cu[-1])
    W = wl.make_weights(shape, seed)
    x, dy = wl.make_activations(shape, T, seed)
    case = {"shape": shape, "seed": seed, "cu": cu, "modes": modes, "W": W, "x": x, "dy": dy, "pick": pick,
            "rows": None, "sub_cu": cu, "sub_modes": modes}
    if pick is not None:
        case["rows"] = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in pick])
        case["sub_cu"] = np.concatenate([[0], np.cumsum([cu[s + 1] - cu[s] for s in pick])]).astype(np.int32)
        case["sub_modes"] = modes[pick]
    return case


def fingerprint(name):
    """Identifies a case's inputs (segment layout, seed, shape) in the stored floor file."""
    shape, seed, cu, modes, pick = segments(name)
    h = hashlib.sha256()
    h.update(repr((shape, int(seed), cu.tolist(), modes.tolist(), pick)).encode())
    return h.hexdigest()[:16]
