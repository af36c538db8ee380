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
