"""Pins for the oracle's partition solver: brute-force enumeration of every
contiguous split, closed-form special cases, the homogeneous (textbook
linear-partition) reduction, a lower bound and scaling invariance."""
import itertools

import numpy as np
import pytest

import synth
from oracle.partition import solve_partition, estimate_capacity


def stage_times(costs, caps, bounds, out_bytes=None, bw=None):
    t = []
    for k in range(len(caps)):
        P = [0.0]
        for c in costs:
            P.append(P[-1] + c)
        t.append((P[bounds[k + 1]] - P[bounds[k]]) * caps[k])
    if out_bytes is not None:
        for k in range(1, len(caps)):
            t.append(2.0 * (out_bytes[bounds[k] - 1] / bw[k - 1]))
    return t


def brute_force(costs, caps, out_bytes=None, bw=None):
    Lc, N = len(costs), len(caps)
    best = float('inf')
    for cuts in itertools.combinations(range(1, Lc), N - 1):
        bounds = [0] + list(cuts) + [Lc]
        best = min(best, max(stage_times(costs, caps, bounds, out_bytes, bw)))
    return best


@pytest.mark.parametrize("Lc,N", [(l, n) for l in range(1, 13) for n in range(1, 5) if n <= l])
def test_bottleneck_equals_brute_force(Lc, N):
    for trial in range(6):
        seed = 1000 * Lc + 10 * N + trial
        costs = list(synth.integers(seed, "costs", (Lc,), 1, 2000))
        caps = list(synth.uniform(seed, "caps", (N,), 1.0, 10.0))
        bounds, bott = solve_partition(costs, caps)
        assert bounds[0] == 0 and bounds[-1] == Lc and all(b1 > b0 for b0, b1 in zip(bounds, bounds[1:]))
        assert bott == brute_force(costs, caps)                 # bit-equal
        assert max(stage_times(costs, caps, bounds)) == bott    # the returned split attains it
        D = list(synth.integers(seed, "D", (Lc,), 1, 5000))
        B = list(synth.uniform(seed, "B", (max(N - 1, 1),), 0.5, 4.0))
        bounds, bott = solve_partition(costs, caps, D, B)
        assert bott == brute_force(costs, caps, D, B)
        assert max(stage_times(costs, caps, bounds, D, B)) == bott


def test_special_cases():
    assert solve_partition([3.0, 1.0, 2.0], [2.0]) == ([0, 3], 12.0)
    bounds, bott = solve_partition([5.0] * 12, [1.0] * 4)
    assert bounds == [0, 3, 6, 9, 12] and bott == 15.0
    bounds, bott = solve_partition([1.0, 2.0, 3.0], [1.0, 1.0, 1.0])
    assert bounds == [0, 1, 2, 3] and bott == 3.0
    # capacity is a time multiplier: the slow device gets the small share
    bounds, _ = solve_partition([1.0] * 11, [1.0, 10.0])
    assert bounds == [0, 10, 11]
    bounds, _ = solve_partition([1.0] * 11, [10.0, 1.0])
    assert bounds == [0, 1, 11]
    # tie: the smallest last cut wins
    bounds, bott = solve_partition([3.0, 1.0, 3.0], [1.0, 1.0])
    assert bott == 4.0 and bounds == [0, 1, 3]
    for bad in ([[1.0, 2.0], [1.0, 1.0, 1.0]], [[1.0, -2.0], [1.0]], [[1.0, float('nan')], [1.0]], [[1.0], [0.0]]):
        with pytest.raises(ValueError):
            solve_partition(*bad)


def linear_partition_textbook(costs, N):
    """Homogeneous min-max contiguous split by binary search over the answer on
    integer costs (the classical 'painters partition' formulation)."""
    lo, hi = int(max(costs)), int(sum(costs))
    def feasible(cap):
        parts, cur = 1, 0
        for c in costs:
            if cur + c > cap:
                parts, cur = parts + 1, c
            else:
                cur += c
        return parts <= N
    while lo < hi:
        mid = (lo + hi) // 2
        if feasible(mid):
            hi = mid
        else:
            lo = mid + 1
    return lo


def test_homogeneous_reduces_to_linear_partition():
    for trial in range(40):
        Lc = 5 + trial % 18
        N = 1 + trial % 4
        costs = [int(c) for c in synth.integers(trial, "hc", (Lc,), 1, 500)]
        _, bott = solve_partition([float(c) for c in costs], [1.0] * N)
        assert bott == float(linear_partition_textbook(costs, N))


def test_lower_bound_and_scaling_invariance():
    for trial in range(50):
        costs = list(synth.integers(trial, "c", (22,), 100, 100000))
        caps = list(synth.uniform(trial, "k", (4,), 1.0, 10.0))
        bounds, bott = solve_partition(costs, caps)
        assert bott >= sum(costs) / sum(1.0 / c for c in caps) * (1 - 1e-12)
        b2, bott2 = solve_partition(costs, [c * 4.0 for c in caps])
        assert b2 == bounds and bott2 == bott * 4.0
        b3, _ = solve_partition([c * 0.5 for c in costs], caps)
        assert b3 == bounds


def test_capacity_estimate():
    costs = [2.0, 3.0, 5.0, 7.0]
    assert estimate_capacity(30.0, costs, 1, 2) == 30.0 / 8.0
    assert estimate_capacity(17.0, costs, 0, 3) == 1.0


# ---- weight redistribution (the paper's Algorithm "Weight Redistribution") ----------------------
# Table written from the rules of section "Fault Tolerance Mechanism": a needed layer that the worker does
# not hold is fetched from the stage that holds it now; indices above the failed one drop by one; a layer of
# the failed stage comes from the worker behind it in the chain (whose new index is the failed index); if the
# failed stage was the last one its backup is on the central node, index 0; a plain re-partition corrects
# nothing.   (bounds_cur, bounds_new, i_fail, i_cur, i_new) -> (M_need, L_local)
REDISTRIBUTION_TABLE = [
    # plain re-partition of 12 layers over 3 workers
    (([0, 4, 8, 12], [0, 6, 9, 12], None, 0, 0), ({1: [4, 5]}, [0, 1, 2, 3])),
    (([0, 4, 8, 12], [0, 6, 9, 12], None, 1, 1), ({2: [8]}, [6, 7])),
    (([0, 4, 8, 12], [0, 6, 9, 12], None, 2, 2), ({}, [9, 10, 11])),
    # shrink: worker 2 takes layers from both neighbours' old ranges
    (([0, 4, 8, 12], [0, 2, 4, 12], None, 2, 2), ({1: [4, 5, 6, 7]}, [8, 9, 10, 11])),
    # worker 1 of 4 fails; survivors are renumbered 0, 1 (was 2), 2 (was 3)
    (([0, 3, 6, 9, 12], [0, 4, 8, 12], 1, 0, 0), ({1: [3]}, [0, 1, 2])),
    (([0, 3, 6, 9, 12], [0, 4, 8, 12], 1, 2, 1), ({1: [4, 5]}, [6, 7])),
    (([0, 3, 6, 9, 12], [0, 4, 8, 12], 1, 3, 2), ({1: [8]}, [9, 10, 11])),
    # the last stage fails: its backup is on the central node
    (([0, 4, 8, 12], [0, 6, 12], 2, 1, 1), ({0: [8, 9, 10, 11]}, [6, 7])),
    (([0, 4, 8, 12], [0, 6, 12], 2, 0, 0), ({1: [4, 5]}, [0, 1, 2, 3])),
    # worker 0 (the central node's own stage is never the failed one) with a failure behind it
    (([0, 4, 8, 12], [0, 5, 12], 1, 0, 0), ({1: [4]}, [0, 1, 2, 3])),
    (([0, 4, 8, 12], [0, 5, 12], 1, 2, 1), ({1: [5, 6, 7]}, [8, 9, 10, 11])),
]


def test_redistribution_plan_table():
    from oracle.partition import redistribution_plan
    for (cur, new, i_fail, i_cur, i_new), (m_need, local) in REDISTRIBUTION_TABLE:
        got = redistribution_plan(new, cur, i_fail, i_cur, i_new)
        assert got == (m_need, local), ((cur, new, i_fail, i_cur, i_new), got)


def test_redistribution_plan_invariants():
    """Brute-force properties on random partitions: needed and local layers partition the new stage exactly;
    every needed layer is asked from a worker that exists in the new numbering; without a failure the source is
    the current holder; nothing is needed when the partition does not change."""
    from oracle.partition import redistribution_plan
    for t in range(300):
        L = 6 + t % 17
        n = 2 + t % 4
        cuts_c = sorted(set(int(x) for x in synth.integers(t, "c", (n - 1,), 1, L - 1)))
        cur = [0] + cuts_c + [L]
        n_cur = len(cur) - 1
        fail = None if t % 3 == 0 or n_cur < 3 else 1 + t % (n_cur - 1)
        n_new = n_cur - (fail is not None)
        cuts_n = sorted(set(int(x) for x in synth.integers(t, "n", (n_new - 1,), 1, L - 1)))[:n_new - 1] if n_new > 1 else []
        new = [0] + cuts_n + [L]
        n_new = len(new) - 1
        for i_cur in range(n_cur):
            if i_cur == fail:
                continue
            i_new = i_cur - 1 if fail is not None and i_cur > fail else i_cur
            if i_new >= n_new:
                continue
            m_need, local = redistribution_plan(new, cur, fail, i_cur, i_new)
            asked = sorted(l for ls in m_need.values() for l in ls)
            assert sorted(asked + local) == list(range(new[i_new], new[i_new + 1]))
            assert all(cur[i_cur] <= l < cur[i_cur + 1] for l in local)
            assert all(0 <= k < max(n_cur - (fail is not None), 1) for k in m_need)
            if fail is None:
                for k, ls in m_need.items():
                    assert all(cur[k] <= l < cur[k + 1] for l in ls)
        same, _ = redistribution_plan(cur, cur, None, 0, 0)
        assert same == {}


def test_renumber_workers():
    from oracle.partition import renumber_workers
    assert renumber_workers(["c", "w1", "w2", "w3"], [2]) == ["c", "w1", "w3"]
    assert renumber_workers(["c", "w1", "w2", "w3", "w4"], [1, 3]) == ["c", "w2", "w4"]
    assert renumber_workers(["c", "w1"], []) == ["c", "w1"]


# ------------------------------------------------------------ re-partition schedule and capacities
def test_repartition_schedule_first_after_10_then_every_100():
    """Section "Dynamic Model Partition": first after 10 batches, then every 100."""
    from oracle.partition import repartition_due
    due = [b for b in range(0, 450) if repartition_due(b)]
    assert due == [10, 110, 210, 310, 410]


def test_repartition_capacities_closed_form_and_fallback():
    """A worker that takes exactly k times the central node's profiled time for its layers has capacity k (capacity
    equations), whatever the cut; the central node stays at 1.0; one missing report makes everybody equal."""
    from oracle.partition import repartition_capacities, solve_partition
    costs = [3.0, 1.0, 4.0, 1.0, 5.0, 9.0, 2.0, 6.0]
    bounds = [0, 3, 5, 8]
    slow = [1.0, 2.5, 7.0]
    means = [123.0] + [slow[i] * sum(costs[bounds[i]:bounds[i + 1]]) for i in (1, 2)]     # worker 0's report is not used
    caps = repartition_capacities(means, costs, bounds)
    assert caps == [1.0, 2.5, 7.0]
    assert repartition_capacities([None, means[1], means[2]], costs, bounds) == caps           # central node: no report needed
    assert repartition_capacities([means[0], None, means[2]], costs, bounds) == [1.0, 1.0, 1.0]
    # the slower the later workers, the more layers the central node keeps
    b_equal, _ = solve_partition(costs, [1.0, 1.0, 1.0])
    b_meas, _ = solve_partition(costs, caps)
    assert b_meas[1] >= b_equal[1] and b_meas[1] > 3
