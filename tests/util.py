"""Shared helpers of the GPU parity tests: run the oracle and the HIP path on the same seeded inputs."""
import os
import sys
import time

import numpy as np

from oracle import layer_oracle as orc
from paper_2408_04275_amd import workloads as wl
from paper_2408_04275_amd import parity


PROGRESS_LOG = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "progress.log")


def say(msg):
    """Progress line of a long test: appended to gpurun_out/progress.log (pytest captures stdout/stderr),
    so that a long oracle run leaves a trace while it works."""
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


def gpu_run(shape, cu, modes, W, x, dy, flags=0, grad_names=None, repeat=1):
    from paper_2408_04275_amd.harness import LayerRunner
    r = LayerRunner(shape, W, cu, modes, grad_names=grad_names)
    r.set_inputs(x, dy)
    for _ in range(repeat):
        r.step(flags)
    return r.results()


def assert_parity(name, got, ref, dtype, bars=None):
    """The three per-tensor bars of paper_2408_04275_amd.parity; returns the measured errors."""
    return parity.check(name, got, ref, dtype, bars)


def compare_layer(shape, got, ref, what="", bars=None):
    y, dx, G = got
    ry, rdx, rG = ref
    errs = {"y": assert_parity(what + "y", y, ry, shape.dtype, bars), "dx": assert_parity(what + "dx", dx, rdx, shape.dtype, bars)}
    assert set(G) == set(rG), (sorted(G), sorted(rG))
    for k in rG:
        errs[k] = assert_parity(what + "d" + k, G[k], rG[k], shape.dtype, bars)
    return errs


def summary(errs):
    worst = {m: max(e[m] for e in errs.values()) for m in ("max_err", "floor_err", "l2_err")}
    return " ".join(f"{k}={v:.1e}" for k, v in worst.items())
