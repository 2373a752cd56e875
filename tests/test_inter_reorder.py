"""Algorithm 2 (inter-microbatch reordering) and the 1F1B timeline it reasons about: the oracle against hand-worked
examples, closed forms of the schedule and its structural properties; the library (host C++ behind the C ABI)
against the oracle, exactly."""
import itertools
import os

import numpy as np
import pytest

from oracle import pipeline_oracle as po
from paper_2408_04275_amd import binding as mm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg2_examples.txt")


def read_golden():
    rec = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, val = line.split(":", 1)
        rows = [[float(v) for v in row.split()] for row in val.split("|")]
        rec[key.strip()] = rows if len(rows) > 1 else rows[0]
    return rec


def uniform(p, l, f, b):
    return [[f] * l for _ in range(p)], [[b] * l for _ in range(p)]


def random_times(rng, p, l, integers):
    if integers:       # many ties
        return rng.integers(0, 9, (p, l)).astype(float), rng.integers(0, 9, (p, l)).astype(float)
    return rng.random((p, l)), 2.0 * rng.random((p, l))


# ---- oracle: timeline ------------------------------------------------------------------

def test_timeline_hand_worked_example():
    g = read_golden()
    assert po.makespan(g["T.fwd"], g["T.bwd"]) == g["T.makespan"][0]
    assert po.intervals(g["T.fwd"], g["T.bwd"]) == g["T.intervals"]


@pytest.mark.parametrize("p,l", [(1, 1), (1, 5), (4, 1), (4, 3), (4, 4), (4, 6), (3, 17), (8, 32)])
def test_uniform_closed_forms(p, l):
    """Equal stages: the textbook iteration time (l + p - 1)(f + b); the first gradient returns after the first
    microbatch has crossed the other p - 1 stages twice; every later wait is one forward pass long."""
    f, b = 1.25, 2.5
    F, B = uniform(p, l, f, b)
    assert po.makespan(F, B) == pytest.approx((l + p - 1) * (f + b), abs=1e-12)
    iv = po.intervals(F, B)
    if p > 1:
        assert iv[0] == pytest.approx((p - 1) * (f + b), abs=1e-12)
        # forward passes still to run at the first stage after the first: min(p - 1, l - 1) fill interval 1
        for i in range(2, l + 1):
            assert iv[i - 1] == pytest.approx(f, abs=1e-12)
    # idle time of the first stage = makespan - its work = the unfilled parts of the intervals
    if p > 1 and l >= p:
        unfilled = (iv[0] - (p - 1) * f) + sum(iv[l - p + 1:])
        assert unfilled == pytest.approx((p - 1) * (f + b), abs=1e-12)


def test_single_stage_and_single_microbatch():
    rng = np.random.default_rng(0)
    f, b = random_times(rng, 1, 7, False)
    assert po.makespan(f.tolist(), b.tolist()) == pytest.approx(float(f.sum() + b.sum()), abs=1e-12)
    f, b = random_times(rng, 6, 1, False)
    assert po.makespan(f.tolist(), b.tolist()) == pytest.approx(float(f.sum() + b.sum()), abs=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_schedule_is_valid_1f1b(seed):
    """Properties of the schedule that do not come from the recursion: every stage runs its microbatches' forward
    passes in order and its backward passes in order, without overlap; inputs precede their consumers; stage s never
    holds more than p - s microbatches between forward and backward (the memory bound 1F1B exists for); the
    iteration is at least as long as any stage's work and as any microbatch's way down and back."""
    rng = np.random.default_rng(seed)
    p, l = int(rng.integers(1, 7)), int(rng.integers(1, 15))
    f, b = random_times(rng, p, l, seed % 2 == 0)
    start, end = po.simulate_1f1b(f.tolist(), b.tolist())
    assert len(end) == 2 * p * l
    for s in range(p):
        ops = sorted((k for k in end if k[1] == s), key=lambda k: (start[k], end[k]))
        for a, c in zip(ops, ops[1:]):
            assert end[a] <= start[c] + 1e-12
        for j in range(l):
            assert start[("B", s, j)] >= end[("F", s, j)] - 1e-12
            if s > 0:
                assert start[("F", s, j)] >= end[("F", s - 1, j)] - 1e-12
                assert start[("B", s - 1, j)] >= end[("B", s, j)] - 1e-12
            if j > 0:
                assert start[("F", s, j)] >= end[("F", s, j - 1)] - 1e-12
                assert start[("B", s, j)] >= end[("B", s, j - 1)] - 1e-12
        # microbatches in flight, counted in the stage's own operation order
        inflight = worst = 0
        for kind, _ in po.stage_order(p, l, s):
            inflight += 1 if kind == "F" else -1
            worst = max(worst, inflight)
        assert worst == min(p - s, l)
    ms = max(end.values())
    assert ms >= max(float(f[s].sum() + b[s].sum()) for s in range(p)) - 1e-12
    assert ms >= max(float(f[:, j].sum() + b[:, j].sum()) for j in range(l)) - 1e-12


def test_makespan_is_monotone_in_every_duration():
    rng = np.random.default_rng(3)
    f, b = random_times(rng, 4, 9, False)
    base = po.makespan(f.tolist(), b.tolist())
    for _ in range(40):
        s, j = int(rng.integers(4)), int(rng.integers(9))
        f2 = f.copy()
        f2[s, j] += 0.7
        assert po.makespan(f2.tolist(), b.tolist()) >= base - 1e-12


# ---- oracle: Algorithm 2 ---------------------------------------------------------------

def test_reorder_hand_worked_example():
    g = read_golden()
    order, seen = po.inter_reorder(g["R.fwd"], g["R.bwd"])
    assert order == [int(v) for v in g["R.order"]]
    assert seen == g["R.intervals_seen"]


def test_size_is_the_time_in_encoder_and_generator():
    """The hand-worked example in which the backbone's time varies too: the section's size (encoder + generator time,
    here the first and the last stage) and the total over all stages pick different first and last microbatches."""
    g = read_golden()
    order, seen = po.inter_reorder(g["S.fwd"], g["S.bwd"])
    assert order == [int(v) for v in g["S.order"]] and seen == g["S.intervals_seen"]
    order, seen = po.inter_reorder(g["S.fwd"], g["S.bwd"], sizes=g["S.total_sizes"])
    assert order == [int(v) for v in g["S.order_total_sizes"]] and seen == g["S.intervals_seen_total_sizes"]
    # explicit sizes equal to the default's give the default's result
    enc_gen = [g["S.fwd"][0][j] + g["S.bwd"][0][j] + g["S.fwd"][2][j] + g["S.bwd"][2][j] for j in range(5)]
    assert po.inter_reorder(g["S.fwd"], g["S.bwd"], sizes=enc_gen)[0] == [int(v) for v in g["S.order"]]


@pytest.mark.parametrize("seed", range(8))
def test_reorder_structure(seed):
    """What the section states about the result: a permutation; the smallest microbatch first; the p - 1 smallest of
    the rest at the end."""
    rng = np.random.default_rng(100 + seed)
    p, l = int(rng.integers(1, 6)), int(rng.integers(1, 16))
    f, b = random_times(rng, p, l, seed % 2 == 0)
    order, seen = po.inter_reorder(f.tolist(), b.tolist())
    assert sorted(order) == list(range(l))
    size = (f + b)[sorted({0, p - 1})].sum(axis=0)           # time in the first and the last stage
    assert size[order[0]] == size.min()
    n_rear = min(p - 1, l - 1)
    if n_rear:
        rest = sorted(np.delete(size, order[0]))
        assert sorted(size[order[l - n_rear:]]) == rest[:n_rear]
    # one interval per loop iteration: p - 1 microbatches for the first, one for each of the others
    n_loop = l - 1 - n_rear
    assert len(seen) == (0 if n_loop == 0 else 1 + max(0, n_loop - (p - 1)) if p > 1 else 1 + n_loop)


def test_get_interval_does_not_depend_on_what_fills_it():
    """The interval the loop asks for is fixed by the microbatches already placed: the final timeline shows the same
    wait at the first stage whenever the chosen forward pass fits into it."""
    rng = np.random.default_rng(5)
    p, l = 3, 9
    enc = np.exp(rng.normal(0, 0.3, l)) * 0.5          # first-stage passes shorter than the waits downstream cause
    f = np.vstack([enc, np.ones(l), np.ones(l)])
    b = 2 * f
    order, seen = po.inter_reorder(f.tolist(), b.tolist())
    final = po.intervals(po.permuted(f.tolist(), order), po.permuted(b.tolist(), order))
    assert seen[0] == pytest.approx(float(f[1:, order[0]].sum() + b[1:, order[0]].sum()), abs=1e-12)
    for i in range(2, len(seen) + 1):
        assert seen[i - 1] == pytest.approx(final[i - 1], abs=1e-12)


def test_reorder_shortens_heterogeneous_iterations_on_average():
    """The section's claim, on seeded inputs of its kind (a skewed first stage in front of constant ones): the
    reordered iteration is shorter on average, and never beats the best permutation."""
    rng = np.random.default_rng(1)
    ratios = []
    for _ in range(120):
        p, l = 4, 12
        enc = np.exp(rng.normal(0, 0.8, l))
        f = np.vstack([enc] + [np.ones(l)] * (p - 1))
        b = 2 * f
        order, _ = po.inter_reorder(f.tolist(), b.tolist())
        ratios.append(po.makespan(po.permuted(f.tolist(), order), po.permuted(b.tolist(), order))
                      / po.makespan(f.tolist(), b.tolist()))
    assert np.mean(ratios) < 0.98
    for _ in range(5):
        p, l = 3, 6
        enc = np.exp(rng.normal(0, 0.8, l))
        f = np.vstack([enc] + [np.ones(l)] * (p - 1))
        b = 2 * f
        order, _ = po.inter_reorder(f.tolist(), b.tolist())
        mine = po.makespan(po.permuted(f.tolist(), order), po.permuted(b.tolist(), order))
        best = min(po.makespan(po.permuted(f.tolist(), pm), po.permuted(b.tolist(), pm))
                   for pm in itertools.permutations(range(l)))
        assert mine >= best - 1e-12


# ---- the library against the oracle ------------------------------------------------------

def test_library_matches_hand_worked_examples():
    g = read_golden()
    rc, ms, iv = mm.mmtrain_pipeline_1f1b(g["T.fwd"], g["T.bwd"])
    assert rc == 0 and ms == g["T.makespan"][0] and list(iv) == g["T.intervals"]
    rc, order, seen = mm.mmtrain_inter_reorder(g["R.fwd"], g["R.bwd"])
    assert rc == 0 and list(order) == [int(v) for v in g["R.order"]] and list(seen) == g["R.intervals_seen"]
    rc, order, seen = mm.mmtrain_inter_reorder(g["S.fwd"], g["S.bwd"])
    assert rc == 0 and list(order) == [int(v) for v in g["S.order"]] and list(seen) == g["S.intervals_seen"]
    rc, order, seen = mm.mmtrain_inter_reorder(g["S.fwd"], g["S.bwd"], sizes=g["S.total_sizes"])
    assert rc == 0 and list(order) == [int(v) for v in g["S.order_total_sizes"]] and list(seen) == g["S.intervals_seen_total_sizes"]


@pytest.mark.parametrize("seed", range(4))
def test_library_matches_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(150):
        p, l = int(rng.integers(1, 8)), int(rng.integers(1, 20))
        f, b = random_times(rng, p, l, case % 2 == 0)
        sizes = None if case % 3 else (rng.integers(0, 5, l).astype(float) if case % 2 else rng.random(l))
        want, want_seen = po.inter_reorder(f.tolist(), b.tolist(), None if sizes is None else sizes.tolist())
        rc, order, seen = mm.mmtrain_inter_reorder(f, b, sizes)
        assert rc == 0
        assert list(order) == want, (p, l)
        np.testing.assert_allclose(seen, want_seen, rtol=0, atol=1e-12)
        rc, ms, iv = mm.mmtrain_pipeline_1f1b(f, b, order)
        assert rc == 0
        fo, bo = po.permuted(f.tolist(), want), po.permuted(b.tolist(), want)
        assert ms == pytest.approx(po.makespan(fo, bo), abs=1e-12)
        np.testing.assert_allclose(iv, po.intervals(fo, bo), rtol=0, atol=1e-12)


def test_library_large_case_runs_in_linear_work():
    rng = np.random.default_rng(7)
    p, l = 16, 2000
    f, b = random_times(rng, p, l, False)
    rc, order, seen = mm.mmtrain_inter_reorder(f, b)
    assert rc == 0 and sorted(order) == list(range(l))
    rc, ms, _ = mm.mmtrain_pipeline_1f1b(f, b, order)
    assert rc == 0 and ms >= float((f + b).sum(axis=1).max())


def test_library_rejects_bad_arguments():
    f, b = np.ones((2, 3)), np.ones((2, 3))
    lib = mm.load_library()
    bad = f.copy()
    bad[1, 1] = np.nan
    assert mm.mmtrain_inter_reorder(bad, b)[0] == mm.ERR_INVALID_ARG
    bad[1, 1] = -1.0
    assert mm.mmtrain_pipeline_1f1b(f, bad)[0] == mm.ERR_INVALID_ARG
    assert mm.mmtrain_pipeline_1f1b(f, b, [0, 0, 1])[0] == mm.ERR_INVALID_ARG
    assert mm.mmtrain_pipeline_1f1b(f, b, [0, 1, 3])[0] == mm.ERR_INVALID_ARG
    assert mm.mmtrain_inter_reorder(f, b, sizes=[1.0, np.inf, 2.0])[0] == mm.ERR_INVALID_ARG
    assert mm.mmtrain_inter_reorder(f, b, sizes=[1.0, -1.0, 2.0])[0] == mm.ERR_INVALID_ARG
    assert lib.mmtrain_inter_reorder(f.ctypes.data, b.ctypes.data, 0, 3, None, None, None, None) == mm.ERR_INVALID_ARG
    assert lib.mmtrain_inter_reorder(f.ctypes.data, b.ctypes.data, 2, 3, None, None, None, None) == mm.ERR_INVALID_ARG
    assert lib.mmtrain_inter_reorder(None, None, 2, 0, None, None, None, None) == mm.OK
    rc, ms, _ = mm.mmtrain_pipeline_1f1b(np.ones((2, 0)), np.ones((2, 0)))
    assert rc == mm.OK and ms == 0.0
