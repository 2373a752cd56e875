"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.

Workloads 1-4 are compared tensor by tensor with the fp64 oracle run on the whole pack.  Workload 5
(44 TFLOP of fp64 on the host) is compared on SAMPLED segments: the upstream gradient is zero outside a
seeded subset of segments, so that -- by the packed == unpacked property the oracle is pinned to -- the
oracle run on the sub-pack alone gives y and dx on those rows and ALL weight gradients of the full call.
"""
import numpy as np
import pytest

from paper_2408_04275_amd import workloads as wl
from util import compare_layer, gpu_run, oracle_run, say, summary

pytestmark = pytest.mark.gpu


def full_case(config, seed, image_bidir=False):
    shape = wl.SHAPES[config]
    cu, modes, _ = wl.make_segments(config, seed, image_bidir=image_bidir)
    T = int(cu[-1])
    say(f"config {config}: T={T}, {len(cu) - 1} segments (max {int(np.diff(cu).max())}); drawing inputs")
    W = wl.make_weights(shape, seed)
    x, dy = wl.make_activations(shape, T, seed)
    got = gpu_run(shape, cu, modes, W, x, dy)
    say(f"config {config}: HIP path done; running the fp64 oracle")
    ref = oracle_run(shape, cu, modes, W, x, dy)
    errs = compare_layer(shape, got, ref, f"config {config} ")
    say(f"config {config}: worst over {len(errs)} tensors: {summary(errs)}")


def test_config2_encoder_full():
    full_case(2, 0)


def test_vit_huge_encoder_full():
    # not one of the five benchmark workloads: the ViT-Huge shape (head dimension 80) on a workload-2 pack
    full_case(6, 1)


def test_config3_decoder_7b_full():
    full_case(3, 0)


def test_config4_longtail_full():
    seed = wl.longtail_seed()
    full_case(4, seed)


def test_config3_decoder_7b_image_spans_bidirectional():
    # same pack, image spans bidirectional: both mask branches inside one launch at full size; sampled check
    sampled_case(3, 0, image_bidir=True, n_sample=4)


def sampled_case(config, seed, image_bidir=False, n_sample=3, bars=None):
    shape = wl.SHAPES[config]
    cu, modes, kinds = wl.make_segments(config, seed, image_bidir=image_bidir)
    T, S = int(cu[-1]), len(cu) - 1
    rng = np.random.default_rng([seed, 303])
    pick = sorted(set(rng.choice(S, size=min(n_sample, S), replace=False).tolist()) | {S - 1})
    say(f"config {config} sampled: T={T}, {S} segments; sampled segments {pick} "
        f"({sum(int(cu[s + 1] - cu[s]) for s in pick)} tokens)")
    W = wl.make_weights(shape, seed)
    x, dy = wl.make_activations(shape, T, seed)
    rows = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in pick])
    dy_masked = np.zeros_like(dy)
    dy_masked[rows] = dy[rows]
    y, dx, G = gpu_run(shape, cu, modes, W, x, dy_masked)
    say(f"config {config} sampled: HIP path done; running the fp64 oracle on the sub-pack")
    sub_cu = np.concatenate([[0], np.cumsum([cu[s + 1] - cu[s] for s in pick])]).astype(np.int32)
    ref = oracle_run(shape, sub_cu, modes[pick], W, x[rows], dy[rows])
    errs = compare_layer(shape, (y[rows], dx[rows], G), ref, f"config {config} sampled ", bars)
    other = np.setdiff1d(np.arange(T), rows)
    assert not np.any(dx[other]), "tokens whose upstream gradient is zero and that share no segment with the rest must get dx = 0"
    say(f"config {config} sampled: worst over {len(errs)} tensors: {summary(errs)}")


def test_config5_decoder_72b_gqa_sampled():
    # Hidden size 8192 and MLP width 29568 put the bf16 storage floor itself (the fp64 oracle with a
    # rounding at every stored tensor, nothing else changed) at l2 1.39e-2 and floor-at-RMS 1.1e-1 on dx
    # for 1024 tokens of this layer, growing slowly with the number of elements; the two bars that are not
    # the stated max-relative-error bar are widened accordingly for this configuration only.
    sampled_case(5, 0, n_sample=3, bars={"floor_err": 1.6e-1, "l2_err": 1.8e-2})
