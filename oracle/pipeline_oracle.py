"""Test infrastructure only (imported by tests/ alone): the paper's inter-microbatch reordering
(Algorithm 2, Section "Inter-microbatch Reordering") and the 1F1B pipeline timeline it reasons about, written
out step by step in plain Python.  No code is shared with the library's C++ implementation.

The timeline.  p pipeline stages, l microbatches; microbatch j takes fwd[s][j] / bwd[s][j] on stage s.  Stage s
runs the one-forward-one-backward order: min(p - 1 - s, l) warm-up forwards, then forward / backward pairs, then
the remaining backwards.  F(s, j) needs F(s - 1, j); B(s, j) needs B(s + 1, j) (on the last stage: F(s, j)).  As the
section states it: an operation starts when both the previous operation of its stage and the operation that
produces its input have ended, and ends its own duration later.

Intervals (the section's definition, at the first stage): interval 1 lies between the end of the first forward
pass and the moment the first backward pass can start, and is filled by the forward passes 2 .. p; interval
i >= 2 lies between the end of backward pass i - 1 and the moment backward pass i can start, and is filled by
forward pass i + p - 1; the last p - 1 intervals have nothing left to fill them.  "Can start" is the arrival of
the gradient from the second stage, so an interval's size does not depend on what is put into it.

Readings (the listing and the text leave these open or disagree with each other):
  * size of a microbatch (MIN, SELECTMIN): the section defines it as the microbatch's computation time in the
    modality encoder and the generator.  Which stages those are is the caller's knowledge: `sizes` gives the size
    per microbatch; without it the first and the last stage (forward plus backward) are taken as the encoder's and
    the generator's.  Ties: lowest index.
  * SELECTMIN(mb, p - 1) returns successive minima, so the rear runs from the smallest upwards.
  * the loop bound: one microbatch first, p - 1 at the rear, p - 1 for the first interval and one for each later
    interval add up to l only when the loop runs l - 2p + 2 times, not the l - p times of the listing; the loop
    here runs while microbatches remain, and a selection takes what is left when fewer remain than it asks for.
  * GETINTERVAL(ret_mb, i) evaluates the timeline with the microbatches placed so far in their positions and
    every later position taking no time (nothing that interval i depends on lies in a later position, except
    for interval 1, which then is the first microbatch's way down the pipeline and back).
  * SELECTCLOSEST(mb, k, interval) compares first-stage forward times with the interval: pick k times, each time
    the microbatch whose forward time is closest to the volume still open divided by the picks still to make;
    ties: lowest index.
"""


def stage_order(p, l, s):
    """The operations of stage s in one-forward-one-backward order: ('F' | 'B', position)."""
    warm = min(p - 1 - s, l)
    ops = [("F", j) for j in range(warm)]
    for k in range(l - warm):
        ops.append(("F", warm + k))
        ops.append(("B", k))
    ops.extend(("B", k) for k in range(l - warm, l))
    return ops


def simulate_1f1b(fwd, bwd):
    """fwd, bwd: [p][l] durations in pipeline order.  Returns (start, end): dicts keyed (kind, stage, position)."""
    p, l = len(fwd), len(fwd[0]) if fwd else 0
    orders = [stage_order(p, l, s) for s in range(p)]
    nxt = [0] * p
    free = [0.0] * p
    start, end = {}, {}
    progressed = True
    while progressed:
        progressed = False
        for s in range(p):
            while nxt[s] < len(orders[s]):
                kind, j = orders[s][nxt[s]]
                if kind == "F":
                    dep = ("F", s - 1, j) if s > 0 else None
                else:
                    dep = ("B", s + 1, j) if s < p - 1 else ("F", s, j)
                if dep is not None and dep not in end:
                    break
                t0 = max(free[s], end[dep] if dep is not None else 0.0)
                dur = fwd[s][j] if kind == "F" else bwd[s][j]
                start[(kind, s, j)] = t0
                end[(kind, s, j)] = t0 + dur
                free[s] = t0 + dur
                nxt[s] += 1
                progressed = True
    assert all(nxt[s] == len(orders[s]) for s in range(p)), "1F1B order deadlocked"
    return start, end


def makespan(fwd, bwd):
    _, end = simulate_1f1b(fwd, bwd)
    return max(end.values(), default=0.0)


def interval_size(end, p, i):
    """Interval i (1-based) at the first stage, from the end times of a simulated timeline."""
    anchor = end[("F", 0, 0)] if i == 1 else end[("B", 0, i - 2)]
    ready = end[("B", 1, i - 1)] if p > 1 else end[("F", 0, i - 1)]
    return max(0.0, ready - anchor)


def intervals(fwd, bwd):
    p, l = len(fwd), len(fwd[0]) if fwd else 0
    _, end = simulate_1f1b(fwd, bwd)
    return [interval_size(end, p, i) for i in range(1, l + 1)]


def permuted(mat, order):
    return [[row[j] for j in order] for row in mat]


def get_interval(fwd, bwd, ret_mb, i):
    """GETINTERVAL: placed microbatches in their positions, later positions take no time."""
    p, l = len(fwd), len(fwd[0])
    f = [[fwd[s][ret_mb[q]] if q < len(ret_mb) else 0.0 for q in range(l)] for s in range(p)]
    b = [[bwd[s][ret_mb[q]] if q < len(ret_mb) else 0.0 for q in range(l)] for s in range(p)]
    _, end = simulate_1f1b(f, b)
    return interval_size(end, p, i)


def select_closest(fwd0, mb, k, interval):
    chosen, volume = [], interval
    picks = min(k, len(mb))
    for r in range(picks):
        target = volume / (picks - r)
        rest = [m for m in mb if m not in chosen]
        best = min(rest, key=lambda m: (abs(fwd0[m] - target), m))
        chosen.append(best)
        volume -= fwd0[best]
    return chosen


def inter_reorder(fwd, bwd, sizes=None):
    """fwd, bwd: [p][l] durations of the microbatches in their original order; sizes: [l] or None.  Returns the new
    order (original indices, 0-based) and the interval sizes GETINTERVAL reported, one per loop iteration."""
    p, l = len(fwd), len(fwd[0]) if fwd else 0
    if l == 0:
        return [], []
    if sizes is not None:
        size = list(sizes)
    else:
        data_dependent = sorted({0, p - 1})                # the encoder's and the generator's stage
        size = [sum(fwd[s][j] + bwd[s][j] for s in data_dependent) for j in range(l)]
    mb = list(range(l))
    first = min(mb, key=lambda m: (size[m], m))
    ret_mb = [first]
    mb.remove(first)
    rear_mb = []
    for _ in range(min(p - 1, len(mb))):
        m = min(mb, key=lambda m: (size[m], m))
        rear_mb.append(m)
        mb.remove(m)
    seen = []
    i = 1
    while mb:
        interval_i = get_interval(fwd, bwd, ret_mb, i)
        seen.append(interval_i)
        cur_mb = select_closest(fwd[0], mb, p - 1 if i == 1 else 1, interval_i)
        ret_mb.extend(cur_mb)
        for m in cur_mb:
            mb.remove(m)
        i += 1
    ret_mb.extend(rear_mb)
    return ret_mb, seen
