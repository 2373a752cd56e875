#!/usr/bin/env python3
"""Writes tests/golden/bf16_floor.json: what bf16 storage alone costs every tensor of every full-size parity case.

    python tests/golden/make_bf16_floor.py [case ...]        (default: every case of tests/full_cases.py)

For each case it runs the fp64 oracle and the oracle with bf16 storage roundings (oracle/bf16_storage.py) on the
case's seeded inputs and stores, per tensor, the three error figures of the second against the first.  It calls
only oracle/ and the input generators; no GPU and nothing of the HIP path is involved.  The 72B-shaped cases take
about 90 TFLOP of fp64 each for the whole pack (minutes on a few cores, about 45 GB of host memory).
Existing entries of cases that are not recomputed are kept.
"""
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))

from oracle import bf16_storage, layer_oracle as orc          # noqa: E402
import full_cases                                              # noqa: E402

OUT = os.path.join(HERE, "bf16_floor.json")


def errors(got, ref):
    """The figures of paper_2408_04275_amd.parity.errors, restated here so that this script depends on the oracle
    and the generators alone."""
    diff = np.abs(got - ref)
    aref = np.abs(ref)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return {"max_err": float(np.max(diff) / np.max(aref)),
            "floor_err": float(np.max(diff / np.maximum(aref, rms))),
            "l2_err": float(np.sqrt(np.sum(diff * diff)) / np.linalg.norm(ref))}


def floor_of(name):
    c = full_cases.inputs(name)
    shape = c["shape"]
    x, dy = c["x"], c["dy"]
    if c["rows"] is not None:
        x, dy = x[c["rows"]], dy[c["rows"]]
    args = (shape.kind, shape.n_heads, shape.n_kv_heads, shape.head_dim, c["sub_cu"], c["sub_modes"], c["W"], x)
    t0 = time.time()
    y, cache = orc.layer_fwd(*args, eps=shape.norm_eps, rope_base=shape.rope_base)
    dx, G = orc.layer_bwd(c["W"], cache, dy)
    del cache
    print(f"  {name}: oracle {time.time() - t0:.0f} s", flush=True)
    t0 = time.time()
    ye, dxe, Ge = bf16_storage.layer_fwd_bwd_rounded(*args, dy, eps=shape.norm_eps, rope_base=shape.rope_base)
    print(f"  {name}: oracle with bf16 storage {time.time() - t0:.0f} s", flush=True)
    out = {"y": errors(ye, y), "dx": errors(dxe, dx)}
    for k in G:
        out[k] = errors(Ge[k], G[k])
    return {"fingerprint": full_cases.fingerprint(name), "tokens": int(c["sub_cu"][-1]), "tensors": out}


def main():
    names = sys.argv[1:] or list(full_cases.CASES)
    table = {}
    if os.path.exists(OUT):
        with open(OUT) as f:
            table = json.load(f)
    for name in names:
        print(name, flush=True)
        table[name] = floor_of(name)
        worst = {m: max(t[m] for t in table[name]["tensors"].values()) for m in ("max_err", "floor_err", "l2_err")}
        print("  worst over tensors:", " ".join(f"{k}={v:.2e}" for k, v in worst.items()), flush=True)
        with open(OUT, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
            f.write("\n")


if __name__ == "__main__":
    main()
