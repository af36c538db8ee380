"""Dynamic-programming model partition (test infrastructure).

Follows the paper's section "Dynamic Model Partition": the execution time of
layer m on worker k is the central node's profiled time multiplied by the
worker's computing capacity C_k (the per-layer estimate equation), A(j, 1) is
the whole prefix on device 0 (base case), and A(j, n) minimises over the last
cut the slowest of: the optimal (n-1)-device sub-pipeline, twice the transfer
of the cut layer's output, and the last stage on device n-1 (the recurrence
and the last-stage-time equation).

Readings where the text is silent or garbled:
  * capacity is a time multiplier (larger = slower), as the equations say;
  * layers are 0-based, bounds are half-open, every stage holds >= 1 layer, so
    for n stages over the first j layers the last cut l runs over n-1 .. j-1;
  * stage k runs on device k (no permutation search);
  * ties: cuts are scanned in ascending order and only a strictly smaller
    value replaces the incumbent;
  * float64: prefix sums accumulated in layer order, stage time
    (P[j] - P[l]) * C[k], exact max and compare;
  * the transfer term is used only when both output sizes and bandwidths are
    given: 2 * D[l-1] / B[n-2] for the hop from device n-2 to device n-1.
"""
import math


def solve_partition(costs, capacities, out_bytes=None, bandwidth=None):
    """Returns (bounds[N+1], bottleneck).  Stage k = layers [bounds[k], bounds[k+1])."""
    Lc, N = len(costs), len(capacities)
    if N < 1 or Lc < N:
        raise ValueError("need 1 <= N <= L")
    for v in list(costs) + list(capacities):
        if not (math.isfinite(v) and v > 0):
            raise ValueError("costs and capacities must be finite and positive")
    comm = out_bytes is not None and bandwidth is not None
    P = [0.0]
    for c in costs:
        P.append(P[-1] + float(c))
    INF = float('inf')
    # A[n][j]: best bottleneck of the first j layers on devices 0..n-1
    A = [[INF] * (Lc + 1) for _ in range(N + 1)]
    cut = [[0] * (Lc + 1) for _ in range(N + 1)]
    for j in range(1, Lc + 1):
        A[1][j] = P[j] * float(capacities[0])
    for n in range(2, N + 1):
        for j in range(n, Lc + 1):
            best, arg = INF, -1
            for l in range(n - 1, j):
                t = max(A[n - 1][l], (P[j] - P[l]) * float(capacities[n - 1]))
                if comm:
                    t = max(t, 2.0 * (float(out_bytes[l - 1]) / float(bandwidth[n - 2])))
                if t < best:
                    best, arg = t, l
            A[n][j], cut[n][j] = best, arg
    bounds = [0] * (N + 1)
    bounds[N] = Lc
    j = Lc
    for n in range(N, 1, -1):
        j = cut[n][j]
        bounds[n - 1] = j
    return bounds, A[N][Lc]


def estimate_capacity(stage_time, layer_costs, start, end):
    """Capacity equation: measured time of worker i's stage divided by the
    central node's time for the same layers start..end (inclusive)."""
    return stage_time / sum(layer_costs[start:end + 1])


def repartition_due(batches_done):
    """Re-partition schedule (section "Dynamic Model Partition"): the first one after
    10 trained batches, then one every 100 batches (10, 110, 210, ...)."""
    return batches_done == 10 or (batches_done > 10 and (batches_done - 10) % 100 == 0)


def repartition_capacities(mean_times, layer_costs, bounds_cur):
    """Capacities for the next re-partition.  mean_times[i]: average execution time
    worker i reported for its current stage [bounds_cur[i], bounds_cur[i+1]), None if
    it reported none.  The central node (worker 0) keeps capacity 1.0 (capacity
    equations); if any other worker has reported nothing, all workers are taken to be
    equal (section "Fault Tolerance Mechanism": the scheduler then uses the central
    node's times alone)."""
    n = len(bounds_cur) - 1
    if any(mean_times[i] is None for i in range(1, n)):
        return [1.0] * n
    caps = [1.0]
    for i in range(1, n):
        caps.append(estimate_capacity(mean_times[i], layer_costs, bounds_cur[i], bounds_cur[i + 1] - 1))
    return caps


def renumber_workers(worker_list, failed):
    """Worker list after failures (section "Fault Tolerance Mechanism"): with one
    failure every index above the failed one drops by one; with several, each failed
    entry is replaced by the alive workers behind it one by one.  Both are the
    stable removal of the failed entries.  Returns the new list."""
    dead = set(failed)
    return [w for i, w in enumerate(worker_list) if i not in dead]


def redistribution_plan(bounds_new, bounds_cur, i_fail, i_cur, i_new):
    """Weight redistribution (the paper's Algorithm "Weight Redistribution"), for the
    worker that held stage i_cur of bounds_cur and will hold stage i_new of
    bounds_new.  i_fail: index (in the current numbering) of the one failed
    worker, or None for a plain re-partition.  Bounds are half-open layer indices.

    Returns (M_need, L_local): M_need maps a worker index in the NEW numbering to
    the layers to fetch from it; L_local lists the layers of the new stage that the
    worker already holds.  A layer of the failed stage is fetched from the worker
    that follows it in the chain (chain replication puts its backup there: that
    worker's new index equals the failed index), or from worker 0 (the central
    node) when the failed stage was the last one."""
    n_cur = len(bounds_cur) - 1
    holder = {}                       # layer -> stage that holds it under the current partition
    for k in range(n_cur):
        for l in range(bounds_cur[k], bounds_cur[k + 1]):
            holder[l] = k

    def index_after_failure(k):
        """Where the weights of current stage k are found once the failed worker has left the list."""
        if i_fail is None or k < i_fail:
            return k
        if k > i_fail:
            return k - 1              # every worker behind the failed one moved up by one
        # the failed stage itself: its chain successor keeps the backup and has just taken over this index;
        # the last stage has no successor, its backup sits on the central node
        return 0 if i_fail == n_cur - 1 else k

    m_need, local = {}, []
    for l in range(bounds_new[i_new], bounds_new[i_new + 1]):
        if holder[l] == i_cur:
            local.append(l)
        else:
            m_need.setdefault(index_after_failure(holder[l]), []).append(l)
    return m_need, local
