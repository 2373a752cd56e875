"""Algorithm 1 (intra-microbatch reordering): the oracle against what the paper and the mathematics fix, and
the C-ABI entry point against the oracle.  No GPU involved (host code only)."""
import os

import numpy as np
import pytest

from oracle import reorder_oracle as ro
from paper_2408_04275_amd import binding as mm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_example.txt")


def golden_cases():
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        left, right = line.split("->")
        nums = [int(v) for v in left.split()]
        yield nums[0], nums[1:], [int(v) for v in right.split()]


def test_oracle_reproduces_the_papers_example():
    cases = list(golden_cases())
    assert cases
    for m, sizes, want in cases:
        order, _ = ro.intra_reorder(sizes, m)
        assert [i + 1 for i in order] == want


def test_oracle_example_pins_the_tie_break():
    # strictly larger first sample: the third sample goes to the second group instead
    order, _ = ro.intra_reorder([4, 3, 2, 1], 2)
    assert [i + 1 for i in order] == [1, 4, 2, 3]


def test_oracle_is_a_permutation_and_groups_are_what_the_greedy_rule_gives():
    rng = np.random.default_rng(5)
    for _ in range(50):
        n, m = int(rng.integers(0, 40)), int(rng.integers(1, 9))
        sizes = rng.integers(1, 100, size=n).tolist()
        order, groups = ro.intra_reorder(sizes, m)
        assert sorted(order) == list(range(n))
        assert order == [d for g in groups for d in g]
        # within a group the samples appear in descending size (they were handed out in that order)
        for g in groups:
            assert all(sizes[g[i]] >= sizes[g[i + 1]] for i in range(len(g) - 1))
        # greedy invariant: when the last sample of the heaviest group was placed, that group was the lightest,
        # so max load <= mean load + (1 - 1/m) * largest size placed last there
        if n:
            loads = [sum(sizes[d] for d in g) for g in groups]
            j = int(np.argmax(loads))
            assert loads[j] - sizes[groups[j][-1]] <= (sum(sizes) - sizes[groups[j][-1]]) / m + 1e-9


@pytest.mark.parametrize("m", [2, 3, 4])
def test_oracle_is_within_four_thirds_of_the_optimum(m):
    # longest-first greedy partitioning is within 4/3 - 1/(3m) of the optimal maximum load; checked against
    # the brute-force optimum on every tiny instance drawn
    rng = np.random.default_rng(m)
    worst = 1.0
    for _ in range(60):
        n = int(rng.integers(1, 9 if m < 4 else 8))
        sizes = rng.integers(1, 20, size=n).tolist()
        _, groups = ro.intra_reorder(sizes, m)
        got, opt = ro.max_load(sizes, groups), ro.optimal_max_load(sizes, m)
        assert opt <= got <= (4.0 / 3.0 - 1.0 / (3.0 * m)) * opt + 1e-9
        worst = max(worst, got / opt)
    assert worst < 4.0 / 3.0


def test_oracle_known_worst_case_of_the_greedy_rule():
    # the classic tight instance for m = 2: sizes 3 3 2 2 2 -> greedy 7, optimum 6 (ratio 7/6 = 4/3 - 1/6)
    sizes = [3, 3, 2, 2, 2]
    _, groups = ro.intra_reorder(sizes, 2)
    assert ro.max_load(sizes, groups) == 7 and ro.optimal_max_load(sizes, 2) == 6


def test_c_abi_matches_the_oracle():
    rng = np.random.default_rng(11)
    for m, sizes, want in golden_cases():
        rc, order, begin, load = mm.mmtrain_intra_reorder(sizes, m)
        assert rc == 0 and (order + 1).tolist() == want
    for trial in range(200):
        n, m = int(rng.integers(0, 60)), int(rng.integers(1, 10))
        # small integers: many ties, which is where the two open choices of the algorithm show
        sizes = rng.integers(0, 8 if trial % 2 else 1000, size=n).astype(np.float64)
        rc, order, begin, load = mm.mmtrain_intra_reorder(sizes, m)
        assert rc == 0
        ref_order, ref_groups = ro.intra_reorder(sizes.tolist(), m)
        assert order.tolist() == ref_order
        assert begin.tolist() == np.concatenate([[0], np.cumsum([len(g) for g in ref_groups])]).tolist()
        assert np.allclose(load, [sum(sizes[d] for d in g) for g in ref_groups])


def test_cost_model_fit_recovers_its_coefficients_and_feeds_the_reordering():
    # the fit (least squares of c0 + a tokens + b pairs) on synthetic timings with known coefficients and 1 % noise;
    # the GPU test of the same name in tests/test_zy_gpu_costmodel.py fits this library's measured step time instead
    from paper_2408_04275_amd import costmodel as cm
    from paper_2408_04275_amd import workloads as wl
    rng = np.random.default_rng(3)
    c0, a, b = 0.15, 9.0e-4, 4.0e-8           # ms, ms per token, ms per pair
    feats = [cm.pack_features(cu, modes) for _, cu, modes in cm.training_packs(3)]
    assert len({t for t, _ in feats}) >= 4                       # the token count varies, so `a` is identified
    ms = [(c0 + a * t + b * p) * (1 + 0.01 * rng.standard_normal()) for t, p in feats]
    coef, res = cm.fit(feats, ms)
    assert abs(coef[1] / a - 1) < 0.05 and abs(coef[2] / b - 1) < 0.05 and np.max(np.abs(res)) < 0.04
    # a sample's cost is additive over a pack: the pack's prediction is c0 + the sum of its samples' costs
    cu, modes, _ = wl.make_segments(3, 9)
    t, p = cm.pack_features(cu, modes)
    assert cm.predict(coef, t, p) == pytest.approx(coef[0] + cm.sample_costs(coef, np.diff(cu)).sum(), rel=1e-12)
    # a skewed batch of samples: the reordered groups are no worse than the arrival order, and within the 4/3 bound
    lengths = np.clip(np.rint(rng.lognormal(6.0, 1.2, 32)), 16, 8192).astype(int)
    costs = cm.sample_costs(coef, lengths)
    m = 4
    rc, order, begin, load = mm.mmtrain_intra_reorder(costs, m)
    assert rc == 0
    arrival = [costs[j * 8:(j + 1) * 8].sum() for j in range(m)]
    assert load.max() <= max(arrival) + 1e-12
    assert load.max() <= (4.0 / 3.0) * max(costs.sum() / m, costs.max())


def test_c_abi_rejects_bad_arguments():
    assert mm.mmtrain_intra_reorder([1.0, 2.0], 0)[0] == mm.ERR_INVALID_ARG
    assert mm.mmtrain_intra_reorder([1.0, -2.0], 2)[0] == mm.ERR_INVALID_ARG
    assert mm.mmtrain_intra_reorder([1.0, float("nan")], 2)[0] == mm.ERR_INVALID_ARG
    assert mm.mmtrain_intra_reorder([1.0, float("inf")], 2)[0] == mm.ERR_INVALID_ARG
    rc, order, begin, load = mm.mmtrain_intra_reorder([], 3)
    assert rc == 0 and begin.tolist() == [0, 0, 0, 0]
