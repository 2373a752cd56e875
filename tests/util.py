"""Shared helpers of the GPU parity tests: run the oracle and the HIP path on the same seeded inputs."""
import os
import sys
import time

import numpy as np

from oracle import bf16_storage
from oracle import layer_oracle as orc
from paper_2408_04275_amd import workloads as wl
from paper_2408_04275_amd import parity


PROGRESS_LOG = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "progress.log")


def say(msg):
    """Progress line of a long test: appended to PROGRESS_LOG (pytest captures stdout/stderr), so that a long oracle
    run leaves a trace while it works."""
    line = f"[{time.strftime('%H:%M:%S')}] {msg}"
    print(line, flush=True)
    try:
        os.makedirs(os.path.dirname(PROGRESS_LOG), exist_ok=True)
        with open(PROGRESS_LOG, "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def oracle_run(shape, cu, modes, W, x, dy):
    y, cache = orc.layer_fwd(shape.kind, shape.n_heads, shape.n_kv_heads, shape.head_dim, cu, modes, W, x,
                             eps=shape.norm_eps, rope_base=shape.rope_base)
    dx, G = orc.layer_bwd(W, cache, dy)
    return y, dx, G


def storage_floors(shape, cu, modes, W, x, dy, ref=None, round_param_grads=True):
    """Per tensor, what bf16 storage alone costs this very case: the oracle with storage roundings against the plain
    oracle (`ref`, computed here if not given).  None for fp32 storage."""
    if shape.dtype != wl.BF16:
        return None
    if ref is None:
        ref = oracle_run(shape, cu, modes, W, x, dy)
    y, dx, G = bf16_storage.layer_fwd_bwd_rounded(shape.kind, shape.n_heads, shape.n_kv_heads, shape.head_dim, cu, modes, W, x,
                                                  dy, eps=shape.norm_eps, rope_base=shape.rope_base,
                                                  round_param_grads=round_param_grads)
    floors = {"y": parity.errors(y, ref[0]), "dx": parity.errors(dx, ref[1])}
    floors.update({k: parity.errors(G[k], ref[2][k]) for k in G})
    return floors


def gpu_run(shape, cu, modes, W, x, dy, flags=0, grad_names=None, repeat=1):
    from paper_2408_04275_amd.harness import LayerRunner
    r = LayerRunner(shape, W, cu, modes, grad_names=grad_names)
    r.set_inputs(x, dy)
    for _ in range(repeat):
        r.step(flags)
    return r.results()


def assert_parity(name, got, ref, dtype, bars=None, floor=None):
    """The per-tensor bars of paper_2408_04275_amd.parity; returns the measured errors."""
    return parity.check(name, got, ref, dtype, bars, floor)


def compare_layer(shape, got, ref, what="", bars=None, floors=None):
    """Every output tensor of a layer call against the oracle's.  floors: per tensor name, the bf16 storage floor of this
    case (storage_floors, or the stored table of the full-size cases); the auxiliary bars then follow from it."""
    y, dx, G = got
    ry, rdx, rG = ref
    fl = floors or {}
    errs = {"y": assert_parity(what + "y", y, ry, shape.dtype, bars, fl.get("y")),
            "dx": assert_parity(what + "dx", dx, rdx, shape.dtype, bars, fl.get("dx"))}
    assert set(G) == set(rG), (sorted(G), sorted(rG))
    for k in rG:
        errs[k] = assert_parity(what + "d" + k, G[k], rG[k], shape.dtype, bars, fl.get(k))
    return errs


def summary(errs, floors=None):
    worst = {m: max(e[m] for e in errs.values()) for m in ("max_err", "floor_err", "l2_err", "big_err")}
    text = " ".join(f"{k}={v:.1e}" for k, v in worst.items())
    if floors:
        ratio = {m: max(errs[k][m] / max(floors[k][m], 1e-30) for k in errs if k in floors) for m in ("floor_err", "l2_err")}
        text += "; largest ratio to the bf16 storage floor: " + " ".join(f"{k} x{v:.2f}" for k, v in ratio.items())
    return text
