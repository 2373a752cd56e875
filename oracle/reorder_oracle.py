"""Test infrastructure only (imported by tests/ alone): the paper's intra-microbatch reordering
(Algorithm 1, Section "Intra-microbatch Reordering") written out step by step in plain Python, and a
brute-force optimum for tiny inputs to check its approximation bound against.

Readings: the algorithm does not say how equal sizes are ordered by the sort, nor which group `argmin`
picks among equally loaded ones.  The worked example in the same section (four samples, the first two the
largest, two groups, result order 1 3 2 4) is reproduced only by a stable sort together with the
lowest-index group, so those are taken.
"""
from itertools import product


def intra_reorder(sizes, m):
    """Returns (ret_samples, groups): sample indices (0-based) in the reordered batch, and per group."""
    n = len(sizes)
    sorted_samples = sorted(range(n), key=lambda i: -sizes[i])       # descending by size; Python's sort is stable
    groups = [[] for _ in range(m)]
    for i in range(n):
        loads = [sum(sizes[d] for d in group) for group in groups]
        min_index = loads.index(min(loads))                            # first (lowest-index) minimum
        groups[min_index].append(sorted_samples[i])
    ret_samples = []
    for group in groups:
        ret_samples.extend(group)
    return ret_samples, groups


def max_load(sizes, groups):
    return max((sum(sizes[d] for d in g) for g in groups), default=0)


def optimal_max_load(sizes, m):
    """Smallest possible maximum group load, by trying every assignment (m ** n of them)."""
    best = None
    for assign in product(range(m), repeat=len(sizes)):
        loads = [0] * m
        for d, j in enumerate(assign):
            loads[j] += sizes[d]
        worst = max(loads)
        if best is None or worst < best:
            best = worst
    return best if best is not None else 0
