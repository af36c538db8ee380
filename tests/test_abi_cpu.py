"""No-GPU checks of the C-ABI library: it loads, exports every symbol that
include/ftp.h declares, validates arguments, and its host-side partition solver
agrees bit for bit with the oracle."""
import os
import re

import numpy as np
import pytest

import synth
from oracle.partition import solve_partition as oracle_solve, estimate_capacity as oracle_capacity

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import paper_2110_02781_amd as P
    return P


def test_library_exports_every_declared_symbol(P):
    header = open(os.path.join(ROOT, "include", "ftp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(ftp_[a-z_0-9]+)\s*\(", header)))
    assert len(names) >= 20
    for n in names:
        assert hasattr(P.lib, n), f"{n} declared in ftp.h but not exported"


def test_solver_bit_exact_against_oracle(P):
    for t in range(300):
        Lc = 4 + t % 19
        N = 1 + t % 4
        costs = synth.integers(t, "costs", (Lc,), 1, 3000000)
        caps = synth.uniform(t, "caps", (N,), 1.0, 10.0)
        b, bott = P.solve_partition(costs, caps)
        ob, obott = oracle_solve(list(costs), list(caps))
        assert list(b) == ob and bott == obott
        if N > 1:
            D = synth.integers(t, "D", (Lc,), 1, 10 ** 7)
            bw = synth.uniform(t, "bw", (N - 1,), 0.1, 30.0)
            b, bott = P.solve_partition(costs, caps, D, bw)
            ob, obott = oracle_solve(list(costs), list(caps), list(D), list(bw))
            assert list(b) == ob and bott == obott
    # non-integer costs as well (prefix sums round): still the same operations in the same order
    for t in range(100):
        costs = synth.uniform(t, "fc", (22,), 0.001, 50.0)
        caps = synth.uniform(t, "fk", (4,), 1.0, 10.0)
        b, bott = P.solve_partition(costs, caps)
        ob, obott = oracle_solve(list(costs), list(caps))
        assert list(b) == ob and bott == obott


def test_equal_capacity_is_average_partition(P):
    b, bott = P.solve_partition([5.0] * 12, [1.0] * 4)
    assert list(b) == [0, 3, 6, 9, 12] and bott == 15.0


def test_solver_and_capacity_errors(P):
    for args in ([[1.0], [1.0, 1.0]], [[1.0, -1.0], [1.0]], [[1.0, float("nan")], [1.0]], [[1.0, 2.0], [0.0]],
                 [[1.0, 2.0], [float("inf")]]):
        with pytest.raises(P.FtpError):
            P.solve_partition(*args)
    assert P.estimate_capacity(30.0, [2.0, 3.0, 5.0, 7.0], 1, 2) == oracle_capacity(30.0, [2.0, 3.0, 5.0, 7.0], 1, 2)
    with pytest.raises(P.FtpError):
        P.estimate_capacity(1.0, [1.0, 2.0], 1, 2)


def test_model_description_matches_oracle_and_rejects_bad_chains(P):
    from oracle import models as OM
    for width, classes, stride, hw in ((1.0, 10, 1, 32), (1.4, 1000, 2, 224)):
        ou = OM.mobilenet_v2(width, classes, stride)
        hu = P.models.mobilenet_v2_units(width, classes, stride)
        m = P.model_create(hu, hw, hw, 3, P.F32)
        assert P.model_num_units(m) == len(ou) == 22
        shape = (hw, hw, 3)
        for i, u in enumerate(ou):
            assert P.model_unit_in_shape(m, i) == shape
            assert P.model_unit_param_count(m, i) == sum(int(np.prod(s)) for _, s, _, _ in OM.param_specs(u))
            assert P.model_unit_bn_channels(m, i) == sum(OM.bn_channels(u))
            shape = OM.unit_out_shape(u, shape)
        assert P.model_unit_in_shape(m, 22) == shape
        P.model_destroy(m)
    # identical initial weights from both sides' own layout tables
    ou, hu = OM.cnn1d(), P.models.cnn1d_units()
    op, hp = OM.init_params(ou, 3), P.models.init_unit_params(hu, 3)
    for a, b in zip(op, hp):
        flat = np.concatenate([x.ravel() for x in a]).astype(np.float32) if a else np.zeros(0, np.float32)
        assert np.array_equal(flat, b)
    bad = P.models.cnn1d_units()
    bad[1]["cin"] = 31
    with pytest.raises(P.FtpError):
        P.model_create(bad, 1, 128, 9, P.F32)
    with pytest.raises(P.FtpError):
        P.model_create(P.models.cnn1d_units()[:-1] + [dict(kind=99)], 1, 128, 9, P.F32)


def test_redistribution_plan_matches_oracle(P):
    """The library's host function against the oracle: the paper-derived table and 300 random partitions."""
    from oracle.partition import redistribution_plan as oracle_plan
    from test_oracle_partition import REDISTRIBUTION_TABLE
    for (cur, new, i_fail, i_cur, i_new), want in REDISTRIBUTION_TABLE:
        assert P.redistribution_plan(new, cur, i_fail, i_cur, i_new) == want
    for t in range(300):
        L = 6 + t % 17
        n = 2 + t % 4
        cur = [0] + sorted(set(int(x) for x in synth.integers(t, "c", (n - 1,), 1, L - 1))) + [L]
        n_cur = len(cur) - 1
        fail = None if t % 3 == 0 or n_cur < 3 else 1 + t % (n_cur - 1)
        n_new = n_cur - (fail is not None)
        new = [0] + (sorted(set(int(x) for x in synth.integers(t, "n", (n_new - 1,), 1, L - 1)))[:n_new - 1] if n_new > 1 else []) + [L]
        n_new = len(new) - 1
        for i_cur in range(n_cur):
            if i_cur == fail:
                continue
            i_new = i_cur - 1 if fail is not None and i_cur > fail else i_cur
            if i_new >= n_new:
                continue
            assert P.redistribution_plan(new, cur, fail, i_cur, i_new) == oracle_plan(new, cur, fail, i_cur, i_new)


def test_redistribution_plan_rejects_bad_arguments(P):
    with pytest.raises(RuntimeError):
        P.redistribution_plan([0, 4, 8], [0, 4, 9], None, 0, 0)          # different totals
    with pytest.raises(RuntimeError):
        P.redistribution_plan([0, 4, 4, 8], [0, 4, 8], None, 0, 0)       # empty stage
    with pytest.raises(RuntimeError):
        P.redistribution_plan([0, 4, 8], [0, 4, 8], 1, 1, 0)             # the failed worker asks
    with pytest.raises(RuntimeError):
        P.redistribution_plan([0, 4, 8], [0, 4, 8], None, 2, 0)          # index out of range


def test_renumber_workers_matches_oracle_and_the_plan(P):
    """Section "Fault Tolerance Mechanism": the worker list after failures, through the C ABI, against the oracle's
    table and random cases; and the index that ftp_redistribution_plan names for a unit of a failed stage is, in the
    renumbered list, the worker that followed the failed one."""
    from oracle.partition import renumber_workers as oracle_renumber
    assert P.renumber_workers([10, 11, 12, 13], [2]) == ([10, 11, 13], [0, 1, -1, 2])
    assert P.renumber_workers([10, 11, 12, 13, 14], [1, 3]) == ([10, 12, 14], [0, -1, 1, -1, 2])
    assert P.renumber_workers([7, 8], []) == ([7, 8], [0, 1])
    for t in range(200):
        n = 2 + t % 9
        ids = [int(v) for v in synth.integers(t, "ids", (n,), 100, 999)]
        k = t % n
        failed = sorted(set(1 + int(v) % (n - 1) for v in synth.integers(t, "failed", (k,), 0, 1000))) if k else []
        new_ids, new_index = P.renumber_workers(ids, failed)
        assert new_ids == oracle_renumber(ids, failed)
        assert [i for i, v in enumerate(new_index) if v < 0] == failed
        assert [new_ids[v] for v in new_index if v >= 0] == [w for i, w in enumerate(ids) if i not in failed]
    # one failure in the middle of a 4-stage pipeline: worker 1 asks for a unit of failed stage 2 -> index 2, now worker 13
    cur, new = [0, 3, 6, 9, 12], [0, 4, 8, 12]
    m_need, _ = P.redistribution_plan(new, cur, 2, 1, 1)
    ids, _ = P.renumber_workers([10, 11, 12, 13], [2])
    assert m_need == {2: [6, 7]} and ids[2] == 13
    for bad in ([0], [4], [1, 1], [-1]):
        with pytest.raises(RuntimeError):
            P.renumber_workers([10, 11, 12, 13], bad)


def test_repartition_schedule_and_capacities_match_oracle(P):
    from oracle.partition import repartition_due, repartition_capacities
    assert [b for b in range(0, 450) if P.repartition_due(b)] == [b for b in range(0, 450) if repartition_due(b)] == [10, 110, 210, 310, 410]
    rng = np.random.default_rng(5)
    for _ in range(200):
        L = int(rng.integers(3, 14)); n = int(rng.integers(1, min(L, 5) + 1))
        costs = rng.uniform(0.5, 9.0, L)
        cuts = sorted(rng.choice(np.arange(1, L), size=n - 1, replace=False).tolist()) if n > 1 else []
        bounds = [0] + cuts + [L]
        means = [None if rng.random() < 0.15 else float(rng.uniform(1.0, 50.0)) for _ in range(n)]
        got = P.repartition_capacities(means, costs, bounds)
        ref = repartition_capacities(means, list(costs), bounds)
        assert got == ref                                    # same float64 operations in the same order
    with pytest.raises(RuntimeError):
        P.repartition_capacities([1.0, 2.0], [1.0, 1.0, 1.0], [0, 1, 2])      # bounds do not cover the layers
    with pytest.raises(RuntimeError):
        P.repartition_due(-1)


def test_model_create_rejects_feature_maps_beyond_the_depthwise_offsets(P):
    """Host check, no GPU: the depthwise kernels form in-image offsets in 32 bits."""
    import paper_2110_02781_amd.binding as B
    unit = [dict(kind=B.UNIT_INVRES, cin=8, cout=8, stride=1, expand=6)]
    with pytest.raises(RuntimeError):
        P.model_create(unit, 8192, 4096, 8, P.BF16)          # H*W = 2^25
    with pytest.raises(RuntimeError):
        P.model_create(unit, 4096, 4000, 8 * 20, P.BF16)     # H*W*C*expand >= 2^31
    m = P.model_create(unit, 1024, 1024, 8, P.BF16)
    P.model_destroy(m)
