"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.

Every case of tests/full_cases.py is compared tensor by tensor with the fp64 oracle: max_err against the stated 2e-2,
floor_err and l2_err against the stored bf16 storage floor of that very case and tensor (tests/golden/bf16_floor.json,
written from the oracle alone).  Workloads 1-5 run on the whole pack.  Two cases are SAMPLED on top of that: the
upstream gradient is zero outside a seeded subset of segments, so that -- by the packed == unpacked property the oracle
is pinned to -- the oracle run on the sub-pack alone gives y and dx on those rows and ALL weight gradients of the
full-size call (a fast second look at the 72B shape, and the 7B pack with bidirectional image spans).
"""
import json
import os

import numpy as np
import pytest

import full_cases
from util import compare_layer, gpu_run, oracle_run, say, summary

pytestmark = pytest.mark.gpu

with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "bf16_floor.json")) as _f:
    FLOORS = json.load(_f)


def stored_floors(name):
    entry = FLOORS[name]
    assert entry["fingerprint"] == full_cases.fingerprint(name), \
        f"{name}: the stored storage floor belongs to other inputs; run tests/golden/make_bf16_floor.py {name}"
    return entry["tensors"]


def run_case(name):
    c = full_cases.inputs(name)
    shape, cu = c["shape"], c["cu"]
    T, S = int(cu[-1]), len(cu) - 1
    floors = stored_floors(name)
    if c["rows"] is None:
        say(f"{name}: T={T}, {S} segments (max {int(np.diff(cu).max())}); HIP path")
        got = gpu_run(shape, cu, c["modes"], c["W"], c["x"], c["dy"])
        say(f"{name}: HIP path done; running the fp64 oracle on the whole pack")
        ref = oracle_run(shape, cu, c["modes"], c["W"], c["x"], c["dy"])
    else:
        rows = c["rows"]
        say(f"{name}: T={T}, {S} segments; sampled segments {c['pick']} ({len(rows)} tokens); HIP path")
        dy_masked = np.zeros_like(c["dy"])
        dy_masked[rows] = c["dy"][rows]
        y, dx, G = gpu_run(shape, cu, c["modes"], c["W"], c["x"], dy_masked)
        other = np.setdiff1d(np.arange(T), rows)
        assert not np.any(dx[other]), "tokens whose upstream gradient is zero and that share no segment with the rest must get dx = 0"
        got = (y[rows], dx[rows], G)
        say(f"{name}: HIP path done; running the fp64 oracle on the sub-pack")
        ref = oracle_run(shape, c["sub_cu"], c["sub_modes"], c["W"], c["x"][rows], c["dy"][rows])
    errs = compare_layer(shape, got, ref, name + " ", floors=floors)
    say(f"{name}: worst over {len(errs)} tensors: {summary(errs, floors)}")


def test_config2_encoder_full():
    run_case("config2_full")


def test_config2_encoder_worst_case_pack():
    # sixteen images of 1024 patches: the largest pack workload 2 allows (16384 tokens)
    run_case("config2_worst_case_16x1024")


def test_vit_huge_encoder_full():
    # not one of the five benchmark workloads: the ViT-Huge shape (head dimension 80) on a workload-2 pack
    run_case("config6_vit_huge_full")


def test_config3_decoder_7b_full():
    run_case("config3_full")


def test_config4_longtail_full():
    run_case("config4_longtail_full")


def test_config3_decoder_7b_image_spans_bidirectional():
    # same pack, image spans bidirectional: both mask branches inside one launch at full size
    run_case("config3_image_bidir_sampled")


def test_config5_decoder_72b_gqa_sampled():
    run_case("config5_sampled")


def test_config5_decoder_72b_gqa_full():
    # the whole 8192-token pack of the 72B-shaped layer through the fp64 oracle: about 45 TFLOP on the host cores
    run_case("config5_full")
