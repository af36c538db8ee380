"""GPU parity: the HIP library against the CPU oracle, element by element, on
the same seeded inputs, through the C ABI.  Tolerances: relative 1e-4 (fp32),
2e-2 (bf16) on activations, gradients and updated weights, measured per tensor
as max-abs error / max-abs reference AND relative L2 error."""
import numpy as np
import pytest

import synth
from oracle import layers as L
from oracle import models as OM
from oracle.partition import solve_partition as oracle_solve
from oracle.stage import one_f_one_b_order
from harness import Pair, TOL, CHAINED_BAR, unit_shapes, assert_close, rel_err, unitwise_check, unit_compare, chained_report, assert_chained

pytestmark = pytest.mark.gpu


def hip_models():
    import paper_2110_02781_amd as P
    return P.models


def conv_unit(cin, cout, kh, kw, stride, ph, pw, act):
    import paper_2110_02781_amd.binding as B
    return (OM.Unit('conv', cin, cout, kh, kw, stride, ph, pw, act=act),
            dict(kind=B.UNIT_CONV, cin=cin, cout=cout, kh=kh, kw=kw, stride=stride, pad_h=ph, pad_w=pw, act=act))


def invres_unit(cin, cout, stride, expand):
    import paper_2110_02781_amd.binding as B
    return (OM.Unit('invres', cin, cout, 3, 3, stride, 1, 1, expand=expand, act=L.ACT_RELU6),
            dict(kind=B.UNIT_INVRES, cin=cin, cout=cout, stride=stride, expand=expand))


def train_step_check(pair, seed, classes, tol, steps=2, lr=0.01, mu=0.9, wd=4e-5, want_dx=True, tol_bwd=None):
    """fwd + loss + bwd + update, `steps` times, everything compared."""
    tol_bwd = tol if tol_bwd is None else tol_bwd
    for step in range(steps):
        x = synth.normal(seed, f"x{step}", (pair.batch,) + tuple(pair.in_shape))
        labels = synth.labels(seed, f"labels{step}", pair.batch, classes)
        y, yo = pair.forward(0, x)
        assert_close(y, yo, tol, f"step {step} logits")
        lh, lo = pair.loss(0, labels)
        assert abs(lh - lo) <= tol * max(1.0, abs(lo)), (lh, lo)
        dx, dxo = pair.backward(0, None, want_dx=want_dx)
        if want_dx:
            assert_close(dx, dxo, tol_bwd, f"step {step} dx")
        e = pair.compare_unit_vectors("grads", tol_bwd, floor=1e-7)
        print(f"step {step}: worst grad error max-rel {e[0]:.2e} l2-rel {e[1]:.2e}; ties {pair.tie_reports[-1]}", flush=True)
        pair.compare_unit_vectors("bn", tol)
        pair.update(lr, mu, wd)
        pair.compare_unit_vectors("weights", tol)
        pair.compare_unit_vectors("momentum", tol_bwd, floor=1e-7)
        tol = max(tol, tol_bwd * lr * 10) if step == 0 else tol   # later steps start from perturbed weights


# ------------------------------------------------------------------ single units
SINGLE = [
    ("stem_s1", conv_unit(3, 32, 3, 3, 1, 1, 1, L.ACT_RELU6), (13, 11, 3), 5),
    ("stem_s2", conv_unit(3, 48, 3, 3, 2, 1, 1, L.ACT_RELU6), (15, 18, 3), 3),
    ("conv1d", conv_unit(16, 32, 1, 5, 1, 0, 2, L.ACT_RELU), (1, 37, 16), 4),
    ("conv1d_cin9", conv_unit(9, 32, 1, 5, 1, 0, 2, L.ACT_RELU), (1, 50, 9), 4),
    ("pw_head", conv_unit(40, 72, 1, 1, 1, 0, 0, L.ACT_RELU6), (5, 7, 40), 6),
    ("invres_t6_s1_res", invres_unit(16, 16, 1, 6), (9, 7, 16), 5),
    ("invres_t6_s2", invres_unit(16, 24, 2, 6), (9, 7, 16), 5),
    ("invres_t1", invres_unit(32, 16, 1, 1), (6, 6, 32), 4),
    ("invres_t1_res", invres_unit(16, 16, 1, 1), (6, 5, 16), 4),
    ("invres_wide", invres_unit(88, 136, 2, 6), (7, 7, 88), 3),
    # more than 2048 rows (the tiled / streaming kernels), with nothing a multiple of a tile: rows not of 128 or 32,
    # feature maps not of 8x16, channels of 8 only
    ("invres_ragged_big_s1_res", invres_unit(40, 40, 1, 6), (37, 29, 40), 3),
    ("invres_ragged_big_s2", invres_unit(24, 40, 2, 4), (75, 61, 24), 2),
    ("invres_ragged_mixed_s2", invres_unit(40, 72, 2, 6), (37, 29, 40), 3),
    ("pw_ragged_big", conv_unit(40, 72, 1, 1, 1, 0, 0, L.ACT_RELU6), (37, 61, 40), 2),
    ("stem_ragged_big_s2", conv_unit(3, 24, 3, 3, 2, 1, 1, L.ACT_RELU6), (75, 61, 3), 3),
    # reductions of 256 channels or more over more than 2048 rows (bfloat16: the long-reduction GEMM), ragged in every
    # extent: rows not a multiple of 64, reductions not of 64, output columns not of 32; with and without a view on
    # the input, with and without a residual
    ("invres_long_reduction_s1_res", invres_unit(48, 48, 1, 6), (27, 29, 48), 3),
    ("invres_long_reduction_wide", invres_unit(88, 136, 1, 6), (19, 19, 88), 6),
    ("pw_long_reduction_fwd", conv_unit(264, 72, 1, 1, 1, 0, 0, L.ACT_RELU6), (37, 61, 264), 1),
    ("pw_long_reduction_dgrad", conv_unit(40, 264, 1, 1, 1, 0, 0, L.ACT_RELU6), (37, 61, 40), 1),
    # images of more than 112 x 112 pixels with 144 / 48 depthwise channels (bfloat16: the depthwise weight gradient that
    # stages rows through an LDS ring), widths and heights that are no multiple of its column bands or row segments
    ("invres_row_ring_s2", invres_unit(24, 32, 2, 6), (113, 117, 24), 1),
    ("invres_row_ring_s1_res", invres_unit(8, 8, 1, 6), (115, 113, 8), 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name,unit,in_shape,batch", SINGLE, ids=[s[0] for s in SINGLE])
def test_single_unit_forward_backward(name, unit, in_shape, batch, dtype):
    print(f"case {name} {dtype} in_shape={in_shape} batch={batch}", flush=True)
    tol = TOL[dtype]
    # float: the oracle decides every activation alone; bfloat16: decisions inside the rounding band follow the library
    pair = Pair([unit[0]], [unit[1]], in_shape, batch, 0, 1, dtype, seed=3, ties="off" if dtype == "f32" else "bounded")
    try:
        x = synth.normal(11, "x", (batch,) + tuple(in_shape))
        y, yo = pair.forward(0, x)
        assert_close(y, yo, tol, "y")
        dy = synth.normal(11, "dy", yo.shape)
        dx, dxo = pair.backward(0, dy)
        assert_close(dx, dxo, tol, "dx")
        pair.compare_unit_vectors("grads", tol, floor=1e-6)
        pair.compare_unit_vectors("bn", tol)
        pair.update(0.05, 0.9, 4e-5)
        pair.compare_unit_vectors("weights", tol)
    finally:
        pair.close()


# ---------------------------------------------------------------------- config 1
def test_config1_cnn1d_train_steps():
    print("config 1: cnn1d batch 8 fp32", flush=True)
    pair = Pair(OM.cnn1d(), hip_models().cnn1d_units(), (1, 128, 9), 8, 0, 6, "f32", seed=1)
    try:
        train_step_check(pair, 1, 6, TOL["f32"], steps=3, wd=0.0)
    finally:
        pair.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_cnn1d_at_a_larger_batch(dtype):
    """The 1-D CNN at batch 40 (5120 positions per layer): the convolutions leave the short-problem kernels and
    run as patch matrix + row-streaming MFMA GEMM (forward, data gradient, weight gradient)."""
    print(f"cnn1d batch 40 {dtype}", flush=True)
    o, h = OM.cnn1d(), hip_models().cnn1d_units()
    if dtype == "f32":
        pair = Pair(o, h, (1, 128, 9), 40, 0, 6, "f32", seed=17, ties="bounded")      # 1.6 M activation decisions
        try:
            train_step_check(pair, 17, 6, TOL["f32"], steps=2, wd=0.0)
        finally:
            pair.close()
    else:
        from oracle.stage import bf16_round
        x = bf16_round(synth.normal(17, "x0", (40, 1, 128, 9)))
        unitwise_check(o, h, (1, 128, 9), 40, 0, 6, "bf16", 17, x, labels=synth.labels(17, "labels0", 40, 6))


def small_net():
    us = [conv_unit(3, 8, 3, 3, 1, 1, 1, L.ACT_RELU6), invres_unit(8, 8, 1, 1), invres_unit(8, 16, 2, 6),
          invres_unit(16, 16, 1, 6), invres_unit(16, 24, 1, 6), conv_unit(24, 32, 1, 1, 1, 0, 0, L.ACT_RELU6)]
    import paper_2110_02781_amd.binding as B
    o = [u[0] for u in us] + [OM.Unit('gap', 32, 32), OM.Unit('fc', 32, 10), OM.Unit('loss', 10, 10)]
    h = [u[1] for u in us] + [dict(kind=B.UNIT_GAP, cin=32, cout=32), dict(kind=B.UNIT_FC, cin=32, cout=10),
                              dict(kind=B.UNIT_LOSS, cin=10, cout=10)]
    return o, h


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_net_ragged_shapes(dtype):
    print(f"small net 9x11 batch 5 {dtype}", flush=True)
    o, h = small_net()
    x = synth.normal(2, "x0", (5, 9, 11, 3))
    labels = synth.labels(2, "labels0", 5, 10)
    if dtype == "f32":
        pair = Pair(o, h, (9, 11, 3), 5, 0, len(o), dtype, seed=2)
        try:
            train_step_check(pair, 2, 10, TOL[dtype], steps=2)
        finally:
            pair.close()
    else:
        from oracle.stage import bf16_round
        x = bf16_round(x)
        assert_chained(chained_report(o, h, (9, 11, 3), 5, 0, len(o), dtype, 2, x, labels=labels), "small_net")
        unitwise_check(o, h, (9, 11, 3), 5, 0, len(o), dtype, 2, x, labels=labels, storage="exact")
    unitwise_check(o, h, (9, 11, 3), 5, 0, len(o), dtype, 2, x, labels=labels)


def test_degenerate_tail_only_stage():
    """A stage that holds no convolution at all: [GAP, FC, loss] on a 2x2x32 boundary tensor."""
    print("tail-only stage: gap + fc + loss, batch 7", flush=True)
    o, h = small_net()
    a, b = len(o) - 3, len(o)
    pair = Pair(o, h, (9, 11, 3), 7, a, b, "f32", seed=13)
    try:
        x = synth.normal(13, "x", (7,) + tuple(pair.in_shape))
        labels = synth.labels(13, "labels", 7, 10)
        y, yo = pair.forward(0, x)
        assert_close(y, yo, TOL["f32"], "logits")
        lh, lo = pair.loss(0, labels)
        assert abs(lh - lo) <= TOL["f32"] * max(1.0, abs(lo))
        dx, dxo = pair.backward(0, None, want_dx=True)
        assert_close(dx, dxo, TOL["f32"], "dx")
        pair.compare_unit_vectors("grads", TOL["f32"], floor=1e-7)
        pair.update(0.01, 0.9, 0.0)
        pair.compare_unit_vectors("weights", TOL["f32"])
    finally:
        pair.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_tiny_feature_maps(dtype):
    """Batch 3 on a 12x10 input: the last blocks see 3x3 and 2x2 feature maps, BatchNorm over 27 and 12 values.
    (Over 2-3 values the input gradient of BatchNorm cancels to rounding noise: fp32 against the float64 oracle
    then differs by more than 1e-4 relative without either being wrong, so that case is not compared.)"""
    print(f"small net 12x10 batch 3 {dtype}", flush=True)
    us = [conv_unit(3, 8, 3, 3, 2, 1, 1, L.ACT_RELU6), invres_unit(8, 16, 2, 6), invres_unit(16, 16, 1, 6),
          invres_unit(16, 24, 2, 6)]
    import paper_2110_02781_amd.binding as B
    o = [u[0] for u in us] + [OM.Unit('gap', 24, 24), OM.Unit('fc', 24, 10), OM.Unit('loss', 10, 10)]
    h = [u[1] for u in us] + [dict(kind=B.UNIT_GAP, cin=24, cout=24), dict(kind=B.UNIT_FC, cin=24, cout=10),
                              dict(kind=B.UNIT_LOSS, cin=10, cout=10)]
    x = synth.normal(14, "x0", (3, 12, 10, 3))
    if dtype == "bf16":
        from oracle.stage import bf16_round
        x = bf16_round(x)
    unitwise_check(o, h, (12, 10, 3), 3, 0, len(o), dtype, 14, x, labels=synth.labels(14, "labels0", 3, 10))


# ---------------------------------------------------------------------- config 2
def test_config2_mobilenetv2_32_train_step():
    print("config 2: MobileNetV2 w1.0 32x32 batch 32 fp32", flush=True)
    pair = Pair(OM.mobilenet_v2(1.0, 10, 1), hip_models().mobilenet_v2_units(1.0, 10, 1), (32, 32, 3), 32, 0, 22,
                "f32", seed=4, ties="bounded")
    try:
        train_step_check(pair, 4, 10, TOL["f32"], steps=2, want_dx=False)
    finally:
        pair.close()


# ---------------------------------------------------------------------- config 3
def seeded_unit_costs(seed, n_units=22):
    """A fixed cost vector (integer nanoseconds) for the partition tests: the units a stage covers then do not
    change from run to run as they do with measured costs."""
    return synth.integers(seed, "unit_costs", (n_units,), 20000, 400000).astype(np.float64)


@pytest.mark.parametrize("costs_from", ["seeded", "profiled"])
def test_config3_heaviest_stage_one_f_one_b_with_stashing(costs_from):
    import paper_2110_02781_amd as P
    print(f"config 3: 3-way split on {costs_from} costs, heaviest stage, 4 micro-batches 1F1B", flush=True)
    o_units, h_units = OM.mobilenet_v2(1.0, 10, 1), P.models.mobilenet_v2_units(1.0, 10, 1)
    if costs_from == "profiled":
        model = P.model_create(h_units, 32, 32, 3, P.F32)
        costs, _ = P.profile_layers(model, 32, 10)
        P.model_destroy(model)
    else:
        costs = seeded_unit_costs(6)
    caps = [1.0, 3.0, 10.0]
    bounds, bott = P.solve_partition(costs, caps)
    ob, obott = oracle_solve(list(costs), caps)
    assert list(bounds) == ob and bott == obott
    loads = [costs[bounds[k]:bounds[k + 1]].sum() for k in range(3)]
    k = int(np.argmax(loads))
    a, b = int(bounds[k]), int(bounds[k + 1])
    print(f"bounds {list(bounds)} heaviest stage {k} = units [{a},{b})", flush=True)
    tol = TOL["f32"]
    pair = Pair(o_units, h_units, (32, 32, 3), 32, a, b, "f32", n_slots=3, seed=6, ties="bounded")
    try:
        nb = 4
        xs = [synth.normal(6, f"x{i}", (32,) + tuple(pair.in_shape)) for i in range(nb)]
        dys = [synth.normal(6, f"dy{i}", (32,) + tuple(pair.out_shape), std=1.0 / 32) for i in range(nb)]
        labels = [synth.labels(6, f"l{i}", 32, 10) for i in range(nb)]
        last = (b == 22)
        for op, i in one_f_one_b_order(k, 3, nb):
            if op == 'F':
                y, yo = pair.forward(i % 3, xs[i], snapshot=True)
                assert_close(y, yo, tol, f"F{i} y")
                if last:
                    pair.loss(i % 3, labels[i])
            else:
                dx, dxo = pair.backward(i % 3, None if last else dys[i], want_dx=(a > 0))
                if a > 0:
                    assert_close(dx, dxo, tol, f"B{i} dx")
                pair.compare_unit_vectors("grads", tol, floor=1e-7)
                pair.update(0.01, 0.9, 4e-5)
                pair.compare_unit_vectors("weights", tol)
                tol = max(tol, 3e-4)       # later versions start from weights that already differ by the tolerance
        pair.compare_unit_vectors("bn", tol)
        pair.compare_unit_vectors("momentum", tol, floor=1e-7)
    finally:
        pair.close()


def test_weight_aggregation_along_the_one_f_one_b_schedule():
    """Stage 0 of 3 with weight stashing and aggregation (section "Async Pipeline Training"): the schedule and
    the aggregation points come from the oracle's version trace (pinned to the paper's example); weights,
    momentum and gradients are compared after every update and after every aggregation."""
    from oracle.stage import version_trace
    print("weight aggregation: small net, stage 0 of 3, 9 micro-batches", flush=True)
    o, h = small_net()
    nb, depth = 9, 3
    pair = Pair(o, h, (9, 11, 3), 4, 0, len(o), "f32", seed=21, n_slots=depth)
    try:
        xs = [synth.normal(21, f"x{i}", (4, 9, 11, 3)) for i in range(nb)]
        ls = [synth.labels(21, f"l{i}", 4, 10) for i in range(nb)]
        tol, n_agg = TOL["f32"], 0
        for ev in version_trace(0, 3, nb, aggregate=True):
            if ev[0] == 'F':
                b = ev[1]
                pair.forward(b % depth, xs[b], snapshot=True)
                pair.loss(b % depth, ls[b])
            elif ev[0] == 'B':
                pair.backward(ev[1] % depth, None, want_dx=False)
                pair.update(0.01, 0.9, 4e-5)
                pair.compare_unit_vectors("weights", tol)
                tol = max(tol, 3e-4)       # later versions start from weights that already differ by the tolerance
            else:
                in_flight = sorted(pair.oracle_busy_slots())
                assert len(in_flight) == len(ev[1]) == depth
                before = pair.export_unit_vectors("weights")
                pair.aggregate(in_flight)
                pair.compare_unit_vectors("weights", tol)
                pair.compare_unit_vectors("momentum", tol, floor=1e-7)
                after = pair.export_unit_vectors("weights")
                assert any(not np.array_equal(a, b) for a, b in zip(before, after)), "aggregation changed nothing"
                n_agg += 1
        assert n_agg == 2
    finally:
        pair.close()


def test_weight_aggregation_is_exact_and_rejects_bad_slots():
    """The mean is computed in fp32 in the order given, so two versions give exactly (a + b) / 2 in fp32; slots
    without a snapshot, duplicates and n outside 1..8 are refused."""
    import paper_2110_02781_amd as P
    o, h = small_net()
    pair = Pair(o, h, (9, 11, 3), 4, 0, len(o), "f32", seed=22, n_slots=3)
    try:
        x = synth.normal(22, "x", (4, 9, 11, 3))
        labels = synth.labels(22, "l", 4, 10)
        pair.forward(0, x, snapshot=True); pair.loss(0, labels)
        w0 = pair.export_unit_vectors("weights")
        pair.backward(0, None, want_dx=False); pair.update(0.05, 0.9, 0.0)
        pair.forward(1, x, snapshot=True)                     # slot 1: version 1
        pair.forward(0, x, snapshot=False)                    # slot 0 busy again, but without a snapshot
        with pytest.raises(RuntimeError):
            P.stage_aggregate_weights(pair.stage, [0, 1], pair.stream)
        with pytest.raises(RuntimeError):
            P.stage_aggregate_weights(pair.stage, [1, 1], pair.stream)
        with pytest.raises(RuntimeError):
            P.stage_aggregate_weights(pair.stage, [], pair.stream)
        with pytest.raises(RuntimeError):
            P.stage_aggregate_weights(pair.stage, [7], pair.stream)
        w1 = pair.export_unit_vectors("weights")
        P.stage_snapshot_weights(pair.stage, 0, pair.stream)  # now slot 0 stashes version 1 as well
        P.stage_aggregate_weights(pair.stage, [0, 1], pair.stream)
        same = pair.export_unit_vectors("weights")
        assert all(np.array_equal(a, b) for a, b in zip(w1, same)), "mean of two equal versions must be that version"
        assert any(not np.array_equal(a, b) for a, b in zip(w0, w1))
    finally:
        pair.close()


def _two_stage_step(pa, pb, x, labels, tol, lr=0.01):
    """One synchronous step of a two-stage pipeline: each side's boundary tensors feed its own next stage."""
    ya, yao = pa.forward(0, x)
    assert_close(ya, yao, tol, "boundary activation")
    yb, ybo = pb.forward(0, ya)             # teacher-forced with the library's boundary tensor on both sides
    assert_close(yb, ybo, tol, "logits")
    pb.loss(0, labels)
    dxb, dxbo = pb.backward(0, None, want_dx=True)
    assert_close(dxb, dxbo, tol, "boundary gradient")
    pa.backward(0, dxb, want_dx=False)
    for p in (pa, pb):
        p.compare_unit_vectors("grads", tol, floor=1e-7)
        p.update(lr, 0.9, 4e-5)
        p.compare_unit_vectors("weights", tol)
        p.compare_unit_vectors("momentum", tol, floor=1e-7)
    return yb


def test_repartition_moves_units_between_stages_on_the_device():
    """Dynamic re-partition (section "Dynamic Model Partition"): two stages train, the cut moves, every worker
    works out what it is missing with the redistribution plan and takes it from its owner device-to-device,
    then training goes on.  Each step is compared with the oracle; after the move, so are the moved weights,
    momentum and BatchNorm running statistics."""
    import paper_2110_02781_amd as P
    print("re-partition: small net, cut 4 -> 6, two stages", flush=True)
    o, h = small_net()
    L = len(o)
    cur, new = [0, 4, L], [0, 6, L]
    tol = TOL["f32"]
    A = Pair(o, h, (9, 11, 3), 4, cur[0], cur[1], "f32", seed=31)
    B = Pair(o, h, (9, 11, 3), 4, cur[1], cur[2], "f32", seed=31, model_of=A)
    A2 = B2 = None
    try:
        xs = [synth.normal(31, f"x{i}", (4, 9, 11, 3)) for i in range(3)]
        ls = [synth.labels(31, f"l{i}", 4, 10) for i in range(3)]
        _two_stage_step(A, B, xs[0], ls[0], tol)
        _two_stage_step(A, B, xs[1], ls[1], 3 * tol)
        # new stages; every worker fetches what the plan says, from the stage that holds it now
        A2 = Pair(o, h, (9, 11, 3), 4, new[0], new[1], "f32", seed=99, model_of=A)      # other seed: nothing may survive
        B2 = Pair(o, h, (9, 11, 3), 4, new[1], new[2], "f32", seed=99, model_of=A)
        old = [A, B]
        for i_w, dst in enumerate([A2, B2]):
            m_need, local = P.redistribution_plan(new, cur, None, i_w, i_w)
            for u in local:
                dst.copy_units_from(old[i_w], u, u + 1)
            for src_w, units in m_need.items():
                for u in units:
                    dst.copy_units_from(old[src_w], u, u + 1)
        assert P.redistribution_plan(new, cur, None, 0, 0) == ({1: [4, 5]}, [0, 1, 2, 3])
        for p in (A2, B2):
            p.compare_unit_vectors("weights", 3 * tol)
            p.compare_unit_vectors("momentum", 3 * tol, floor=1e-7)
            p.compare_unit_vectors("bn", 3 * tol)
        # the moved state is the old state, bit for bit
        wa = {u: v for u, v in zip(range(cur[1], cur[2]), B.export_unit_vectors("weights"))}
        w2 = A2.export_unit_vectors("weights")
        assert np.array_equal(w2[4], wa[4]) and np.array_equal(w2[5], wa[5])
        _two_stage_step(A2, B2, xs[2], ls[2], 6 * tol)
        with pytest.raises(RuntimeError):
            P.stage_copy_units(A2.stage, B.stage, 0, 2, A2.stream)       # B never held units 0-1
    finally:
        for p in (B2, A2, B):
            if p is not None:
                p.close()
        A.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recomputation_along_the_one_f_one_b_schedule(dtype):
    """Slots that keep only their stage input and run the forward again in the backward (section "Synchronous
    Pipeline Parallelism Training"), under one-forward-one-backward with weight stashing: against the oracle to the
    usual tolerance, against a twin stage that keeps every intermediate bit for bit, and with less device memory."""
    import paper_2110_02781_amd as P
    print(f"recomputation: small net, stage 0 of 3, 6 micro-batches, {dtype}", flush=True)
    o, h = small_net()
    nb, depth = 6, 3
    # float: everything against the oracle (which decides every activation alone).  bfloat16: the run on its own
    # activations leaves the oracle's (see CHAINED_BAR), so there the oracle checks the loss of every forward and the
    # running statistics at the chained bar, and the weights are checked bit for bit against the twin that keeps
    # everything, whose own parity the other bfloat16 tests establish.
    pair = Pair(o, h, (9, 11, 3), 4, 0, len(o), dtype, seed=51, n_slots=depth, recompute=True)
    try:
        assert P.stage_device_bytes(pair.stage) < P.stage_device_bytes(pair.twin)
        xs = [synth.normal(51, f"x{i}", (4, 9, 11, 3)) for i in range(nb)]
        ls = [synth.labels(51, f"l{i}", 4, 10) for i in range(nb)]
        # bfloat16, six micro-batches with updates in between: loss within 1e-3, running statistics within 5e-3 (measured 1.1e-3)
        tol = TOL[dtype] if dtype == "f32" else 1e-3
        for op, b in one_f_one_b_order(0, 3, nb):
            if op == 'F':
                y, yo = pair.forward(b % depth, xs[b], snapshot=True)
                l, lo = pair.loss(b % depth, ls[b])
                assert abs(l - lo) <= tol * max(1.0, abs(lo)), (l, lo)
            else:
                pair.backward(b % depth, None, want_dx=False)
                if dtype == "f32":
                    pair.compare_unit_vectors("grads", tol, floor=1e-7)
                pair.update(0.01, 0.9, 4e-5)
                pair.assert_twin_identical()
                if dtype == "f32":
                    pair.compare_unit_vectors("weights", tol)
                    tol = max(tol, 3e-4)   # later versions start from weights that already differ by the tolerance
        pair.compare_unit_vectors("bn", tol if dtype == "f32" else 5e-3)        # the second forwards did not move the running statistics
    finally:
        pair.close()


def test_recomputation_on_a_two_stream_stage_is_bit_identical():
    """A stage large enough to run its weight gradients on the second stream (largest activation 58 MB), two
    micro-batches in flight: the recomputing stage's second forward runs in front of each backward while nothing
    of the previous backward is pending, so it must leave exactly the weights of the stage that keeps everything."""
    import torch
    import paper_2110_02781_amd as P
    print("recomputation, 224x224 w1.4 batch 16 bf16, two slots", flush=True)
    units = P.models.mobilenet_v2_units(1.4, 1000, 2)
    model = P.model_create(units, 224, 224, 3, P.BF16)
    L = P.model_num_units(model)
    params = P.models.init_unit_params(units, 71)
    stages = [P.stage_create(model, 0, L, 16, 2, f) for f in (0, P.STAGE_RECOMPUTE)]
    try:
        dev = torch.device("cuda:0")
        for st in stages:
            for i in range(L):
                P.stage_import_weights(st, i, params[i])
        xs = [torch.from_numpy(synth.normal(71, f"x{k}", (16, 224, 224, 3)).astype(np.float32)).to(dev).to(torch.bfloat16) for k in range(2)]
        ls = [torch.from_numpy(synth.labels(71, f"l{k}", 16, 1000).astype(np.int32)).to(dev) for k in range(2)]
        loss = torch.zeros(1, dtype=torch.float32, device=dev)
        sp = torch.cuda.current_stream().cuda_stream
        assert P.stage_device_bytes(stages[1]) < P.stage_device_bytes(stages[0])
        for rep in range(2):
            for st in stages:
                for k in range(2):
                    P.stage_forward(st, k, xs[k], None, sp)
                    P.stage_loss(st, k, ls[k], loss, sp)
                for k in range(2):
                    P.stage_backward(st, k, None, None, sp)
                P.stage_update(st, 0.005, 0.9, 4e-5, sp)
            torch.cuda.synchronize()
            for i in range(L):
                n = P.model_unit_param_count(model, i)
                if n:
                    assert np.array_equal(P.stage_export_weights(stages[0], i, n), P.stage_export_weights(stages[1], i, n)), \
                        f"mini-batch {rep}: unit {i} differs"
                nb = P.model_unit_bn_channels(model, i)
                if nb:
                    assert np.array_equal(P.stage_export_bn_stats(stages[0], i, 2 * nb), P.stage_export_bn_stats(stages[1], i, 2 * nb))
    finally:
        for st in stages:
            P.stage_destroy(st)
        P.model_destroy(model)


def test_recomputation_call_order_errors():
    """With recomputation the logits of a slot are gone once another slot has been forwarded."""
    import paper_2110_02781_amd as P
    o, h = small_net()
    pair = Pair(o, h, (9, 11, 3), 4, 0, len(o), "f32", seed=52, n_slots=2, recompute=True)
    try:
        x = synth.normal(52, "x", (4, 9, 11, 3))
        labels = synth.labels(52, "l", 4, 10)
        pair.forward(0, x); pair.forward(1, x)
        ld = pair.torch.from_numpy(np.asarray(labels, dtype=np.int32)).to(pair.dev)
        out = pair.torch.zeros(1, dtype=pair.torch.float32, device=pair.dev)
        with pytest.raises(RuntimeError):
            P.stage_loss(pair.stage, 0, ld, out, pair.stream)             # slot 1 owns the stash now
        with pytest.raises(RuntimeError):
            P.stage_export_conv_output(pair.stage, 0, 0, 0, 4 * 9 * 11 * 8)
        with pytest.raises(RuntimeError):
            P.stage_create(pair.model, 0, len(o), 4, 1, 0x80)             # unknown flag
        pair.loss(1, labels)
        pair.backward(1, None, want_dx=False)
        dy = synth.normal(52, "dy", (4,) + tuple(pair.out_shape))
        pair.backward(0, dy, want_dx=False)                               # recomputes slot 0; needs an explicit gradient
        pair.assert_twin_identical()
    finally:
        pair.close()


@pytest.mark.parametrize("case", ["one_stream_f32", "two_streams_bf16"])
def test_training_step_replays_from_a_hip_graph(case):
    """The compute calls only enqueue kernels and device-to-device copies (no allocation, no memset, no host
    synchronisation), so a whole step can be captured into a HIP graph, including the fork and join of the
    weight-gradient stream of a large stage.  Every replay, with eager work and synchronisations in between, must
    leave exactly the weights that the same step gives when it is launched eagerly on a second stage."""
    import torch
    import paper_2110_02781_amd as P
    print(f"graph replay {case}", flush=True)
    if case == "one_stream_f32":
        _, units = small_net()
        shape, batch, dt, tdt, classes = (9, 11, 3), 4, P.F32, torch.float32, 10
    else:
        units = P.models.mobilenet_v2_units(1.4, 1000, 2)          # largest activation 58 MB: the side stream is on
        shape, batch, dt, tdt, classes = (224, 224, 3), 16, P.BF16, torch.bfloat16, 1000
    dev = torch.device("cuda:0")
    model = P.model_create(units, *shape, dt)
    L = P.model_num_units(model)
    params = P.models.init_unit_params(units, 61)
    stages = [P.stage_create(model, 0, L, batch, 1) for _ in range(2)]
    try:
        for st in stages:
            for i in range(L):
                P.stage_import_weights(st, i, params[i])
        x = torch.from_numpy(synth.normal(61, "x", (batch,) + shape).astype(np.float32)).to(dev).to(tdt)
        labels = torch.from_numpy(synth.labels(61, "l", batch, classes).astype(np.int32)).to(dev)
        loss = [torch.zeros(1, dtype=torch.float32, device=dev) for _ in range(2)]
        stream = torch.cuda.Stream()
        sp = stream.cuda_stream

        def step(k):
            P.stage_forward(stages[k], 0, x, None, sp)
            P.stage_loss(stages[k], 0, labels, loss[k], sp)
            P.stage_backward(stages[k], 0, None, None, sp)
            P.stage_update(stages[k], 0.01, 0.9, 4e-5, sp)

        def weights(k):
            torch.cuda.synchronize()
            return [np.array(P.stage_export_weights(stages[k], i, P.model_unit_param_count(model, i)), copy=True)
                    for i in range(L) if P.model_unit_param_count(model, i)]

        step(0); step(1)                                  # first launches (code objects load) stay outside the capture
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step(1)
        step(0)                                           # the capture itself runs nothing: stage 1 is one step behind
        graph.replay()
        for a, b in zip(weights(0), weights(1)):
            assert np.array_equal(a, b), "first replay differs from the eager step"
        for rep in range(3):
            step(0)
            junk = torch.randn(1 << 16, device=dev).sum()           # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            assert np.isfinite(float(junk))
            for a, b in zip(weights(0), weights(1)):
                assert np.array_equal(a, b), f"replay {rep + 2} differs from the eager step"
            assert float(loss[0].item()) == float(loss[1].item())
        del graph
    finally:
        for st in stages:
            P.stage_destroy(st)
        P.model_destroy(model)


def test_online_execution_timing_feeds_the_capacity_estimate():
    """Execution profiling phase of the dynamic partition: the stage records forward+backward time per batch,
    the mean over the window and the profiled unit costs give the worker's capacity (about 1 on the device that
    did the profiling), and the solver accepts it.  Batches in flight at the read are left out."""
    import paper_2110_02781_amd as P
    print("online execution timing -> capacity -> partition", flush=True)
    o, h = small_net()
    L = len(o)
    pair = Pair(o, h, (9, 11, 3), 4, 0, L, "f32", seed=41, n_slots=2)
    try:
        costs, out_bytes = P.profile_layers(pair.model, 4, 3)
        assert len(costs) == L and all(c > 0 for c in costs)
        with pytest.raises(RuntimeError):
            P.stage_timing_read(pair.stage)                   # not enabled
        P.stage_timing(pair.stage, True)
        x = synth.normal(41, "x", (4, 9, 11, 3))
        labels = synth.labels(41, "l", 4, 10)
        for _ in range(5):
            pair.forward(0, x); pair.loss(0, labels)
            pair.backward(0, None, want_dx=False)
            pair.update(0.01, 0.9, 0.0)
        pair.forward(1, x)                                    # in flight: not a whole batch yet
        mean_ns, n = P.stage_timing_read(pair.stage)
        assert n == 5 and mean_ns > 0
        cap = P.estimate_capacity(mean_ns, costs, 0, L - 1)
        assert 0.05 < cap < 20.0, cap                         # same device as the profile: order one
        bounds, bottleneck = P.solve_partition(costs, [cap, 3.0 * cap])
        assert bounds[0] == 0 and bounds[-1] == L and bounds[1] > L // 2 - 1      # the faster device takes more
        mean2, n2 = P.stage_timing_read(pair.stage)
        assert n2 == 0 and mean2 == 0.0                       # new window, the in-flight batch was dropped
        pair.loss(1, labels); pair.backward(1, None, want_dx=False)
        with pytest.raises(RuntimeError):
            pair.forward(0, x); P.stage_timing(pair.stage, False)     # a batch is in flight
        pair.loss(0, labels); pair.backward(0, None, want_dx=False)
        P.stage_timing(pair.stage, False)
    finally:
        pair.close()


@pytest.mark.parametrize("case", ["one_stream_f32", "two_streams_bf16"])
def test_profiled_unit_costs_add_up_to_the_batch_time(case):
    """Model profiling phase against execution profiling phase on the same device: the per-unit costs of
    ftp_profile_layers add up to the forward+backward time that ftp_stage_timing measures on a live stage of the
    whole model, within a factor 1.3 (two separate measurements of a 1-10 ms step), so the capacity equation gives
    this device a capacity of about 1; also for a stage that runs its weight gradients on the second stream, where
    the per-unit times are taken without that overlap and then scaled."""
    import torch
    import paper_2110_02781_amd as P
    if case == "one_stream_f32":
        units, shape, batch, dt, tdt, classes = P.models.mobilenet_v2_units(1.0, 10, 1), (32, 32, 3), 32, P.F32, torch.float32, 10
    else:
        units, shape, batch, dt, tdt, classes = P.models.mobilenet_v2_units(1.0, 1000, 2), (224, 224, 3), 32, P.BF16, torch.bfloat16, 1000
    print(f"profile_layers vs stage_timing: {case}", flush=True)
    dev = torch.device("cuda:0")
    model = P.model_create(units, *shape, dt)
    L = P.model_num_units(model)
    stage = P.stage_create(model, 0, L, batch, 1)
    try:
        params = P.models.init_unit_params(units, 5)
        for i in range(L):
            P.stage_import_weights(stage, i, params[i])
        x = torch.from_numpy(synth.normal(5, "x", (batch,) + shape).astype(np.float32)).to(dev).to(tdt)
        labels = torch.from_numpy(synth.labels(5, "l", batch, classes).astype(np.int32)).to(dev)
        loss = torch.zeros(1, dtype=torch.float32, device=dev)
        sp = torch.cuda.current_stream().cuda_stream

        def step():
            P.stage_forward(stage, 0, x, None, sp)
            P.stage_loss(stage, 0, labels, loss, sp)
            P.stage_backward(stage, 0, None, None, sp)
            P.stage_update(stage, 0.001, 0.9, 0.0, sp)
        for _ in range(5):
            step()
        torch.cuda.synchronize()
        costs, _ = P.profile_layers(model, batch, 10)
        P.stage_timing(stage, True)
        for _ in range(10):
            step()
        mean_ns, n = P.stage_timing_read(stage)
        P.stage_timing(stage, False)
        assert n == 10
        ratio = costs.sum() / mean_ns
        cap = P.estimate_capacity(mean_ns, costs, 0, L - 1)
        print(f"  sum of unit costs {costs.sum() / 1e6:.3f} ms, batch time {mean_ns / 1e6:.3f} ms, ratio {ratio:.3f}, capacity {cap:.3f}", flush=True)
        assert 1 / 1.3 < ratio < 1.3 and 1 / 1.3 < cap < 1.3
    finally:
        P.stage_destroy(stage)
        P.model_destroy(model)


def test_a_failed_launch_plan_is_reported_once_and_per_thread():
    """A launcher that finds its plan outside its kernel's limits skips the launch and the stage call returns
    FTP_ERR_UNSUPPORTED; the mark belongs to the thread that set it and is cleared by the report."""
    import threading
    import paper_2110_02781_amd as P
    o, h = small_net()
    pair = Pair(o, h, (9, 11, 3), 4, 0, len(o), "f32", seed=8)
    try:
        P.diag_fail_next_launch_plan()
        seen = []
        t = threading.Thread(target=lambda: seen.append(P.stage_update(pair.stage, 0.0, 0.0, 0.0, pair.stream)))
        t.start(); t.join()
        assert seen == [None]                                  # another thread: not affected
        with pytest.raises(P.FtpError) as ei:
            P.stage_update(pair.stage, 0.0, 0.0, 0.0, pair.stream)
        assert ei.value.status == -3 and "launch plan" in str(ei.value)
        P.stage_update(pair.stage, 0.0, 0.0, 0.0, pair.stream)   # reported once
    finally:
        pair.close()


def test_weight_stashing_matters_on_gpu():
    """Without the snapshot the backward uses the newer weights: results must differ from the stashed run."""
    o, h = small_net()
    res = []
    for snap in (True, False):
        pair = Pair(o, h, (8, 8, 3), 4, 0, 5, "f32", n_slots=2, seed=8)
        try:
            x0, x1 = synth.normal(8, "x0", (4, 8, 8, 3)), synth.normal(8, "x1", (4, 8, 8, 3))
            dy = synth.normal(8, "dy", (4,) + tuple(pair.out_shape))
            pair.forward(0, x0, snapshot=snap)
            pair.forward(1, x1, snapshot=snap)
            pair.backward(0, dy, want_dx=False)
            pair.update(0.1, 0.9, 0.0)
            pair.backward(1, dy, want_dx=False)
            e = pair.compare_unit_vectors("grads", TOL["f32"], floor=1e-7)
            import paper_2110_02781_amd as P
            res.append(P.stage_export_grads(pair.stage, 2, P.model_unit_param_count(pair.model, 2)))
        finally:
            pair.close()
    assert np.abs(res[0] - res[1]).max() > 1e-6


# ------------------------------------------------------------------------ solver
def test_solver_bit_exact_on_1000_capacity_vectors():
    import paper_2110_02781_amd as P
    costs = synth.integers(5, "costs", (22,), 1000, 5000000)
    for t in range(1000):
        caps = synth.uniform(5, f"caps{t}", (4,), 1.0, 10.0)
        b, bott = P.solve_partition(costs, caps)
        ob, obott = oracle_solve(list(costs), list(caps))
        assert list(b) == ob and bott == obott, t
    D = synth.integers(5, "D", (22,), 1000, 9000000)
    for t in range(200):
        caps = synth.uniform(6, f"caps{t}", (3,), 1.0, 10.0)
        bw = synth.uniform(6, f"bw{t}", (2,), 0.1, 20.0)
        b, bott = P.solve_partition(costs, caps, D, bw)
        ob, obott = oracle_solve(list(costs), list(caps), list(D), list(bw))
        assert list(b) == ob and bott == obott, t


def test_config1_solver_on_six_units():
    import paper_2110_02781_amd as P
    model = P.model_create(P.models.cnn1d_units(), 1, 128, 9, P.F32)
    costs, out_bytes = P.profile_layers(model, 8, 10)
    P.model_destroy(model)
    assert costs.shape == (6,) and np.all(costs >= 1) and np.all(costs == np.floor(costs))
    assert list(out_bytes) == [8 * 128 * 32 * 4, 8 * 128 * 64 * 4, 8 * 128 * 64 * 4, 8 * 64 * 4, 8 * 6 * 4, 8 * 6 * 4]
    b, bott = P.solve_partition(costs, [1.0, 3.0, 10.0])
    ob, obott = oracle_solve(list(costs), [1.0, 3.0, 10.0])
    assert list(b) == ob and bott == obott


# ---------------------------------------------------------------------- config 4
@pytest.mark.parametrize("costs_from", ["seeded", "profiled"])
def test_config4_middle_stage_of_4way_split_bf16(costs_from):
    """MobileNetV2 w1.0 at 224x224, batch 64, bf16: stage 1 of the 4-way split that solve_partition makes at
    capacities 1:2:5:10, once from a fixed seeded cost vector (the same units every run) and once from
    profile_layers' costs.  The stage's training step on its own activations is measured against the rounding and
    the exact oracle (forward output, input gradient, every weight gradient, updated weights, running statistics);
    then every unit alone, teacher-forced, at the 2e-2 bar against both."""
    import paper_2110_02781_amd as P
    print(f"config 4: 224x224 batch 64 bf16, stage 1 of 4, {costs_from} costs", flush=True)
    batch = 64
    o_units, h_units = OM.mobilenet_v2(1.0, 1000, 2), P.models.mobilenet_v2_units(1.0, 1000, 2)
    if costs_from == "profiled":
        model = P.model_create(h_units, 224, 224, 3, P.BF16)
        costs, out_bytes = P.profile_layers(model, batch, 3)
        P.model_destroy(model)
    else:
        costs = seeded_unit_costs(9)
    caps = [1.0, 2.0, 5.0, 10.0]
    bounds, bott = P.solve_partition(costs, caps)
    ob, obott = oracle_solve(list(costs), caps)
    assert list(bounds) == ob and bott == obott
    a, b = int(bounds[1]), int(bounds[2])
    print(f"costs(us) {[round(c / 1e3) for c in costs]} bounds {list(bounds)} stage 1 = units [{a},{b})", flush=True)
    from oracle.stage import bf16_round
    shapes = unit_shapes(o_units, (224, 224, 3))
    x = bf16_round(synth.normal(9, "x", (batch,) + tuple(shapes[a])))
    dy = bf16_round(synth.normal(9, "dy", (batch,) + tuple(shapes[b]), std=1.0 / batch))
    if costs_from == "seeded":
        assert_chained(chained_report(o_units, h_units, (224, 224, 3), batch, a, b, "bf16", 9, x, dy=dy), "config4")
    # the 2e-2 bar proper: every unit of the stage alone, at its real shape
    rep = []
    unitwise_check(o_units, h_units, (224, 224, 3), batch, a, b, "bf16", 9, x, dy=dy, report=rep)
    for r in rep:
        print("  ", r, flush=True)
    if costs_from == "seeded":
        rep = []
        unitwise_check(o_units, h_units, (224, 224, 3), batch, a, b, "bf16", 9, x, dy=dy, report=rep, storage="exact")
        for r in rep:
            print("  ", r, flush=True)


# ---------------------------------------------------------------------- config 5
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_config5_shapes_at_reduced_batch(dtype):
    """MobileNetV2 w1.4, 224x224, 1000 classes, whole model as one stage; batch 4 (float: 6) instead of
    128 so that the float64 oracle finishes in seconds (same spatial and channel shapes).  At batch 6 in float the
    largest activation is 43 MB: the stage runs its weight gradients on the second stream, as at full size, and the
    whole step (a mix of forked layers and layers too short to fork) is compared with the oracle.  bfloat16: the
    whole step on its own activations is measured against both oracles, then every unit teacher-forced at 2e-2."""
    batch = 6 if dtype == "f32" else 4
    print(f"config 5 shapes, batch {batch}, {dtype}", flush=True)
    o_units, h_units = OM.mobilenet_v2(1.4, 1000, 2), hip_models().mobilenet_v2_units(1.4, 1000, 2)
    if dtype == "f32":
        pair = Pair(o_units, h_units, (224, 224, 3), batch, 0, 22, dtype, seed=10, ties="bounded")
        try:
            train_step_check(pair, 10, 1000, TOL[dtype], steps=1, want_dx=False)
        finally:
            pair.close()
        return
    from oracle.stage import bf16_round
    x = bf16_round(synth.normal(10, "x0", (4, 224, 224, 3)))
    labels = synth.labels(10, "labels0", 4, 1000)
    assert_chained(chained_report(o_units, h_units, (224, 224, 3), 4, 0, 22, dtype, 10, x, labels=labels), "config5")
    rep = []
    unitwise_check(o_units, h_units, (224, 224, 3), 4, 0, 22, dtype, 10, x, labels=labels, report=rep)
    for r in rep:
        print("  ", r, flush=True)
    unitwise_check(o_units, h_units, (224, 224, 3), 4, 0, 22, dtype, 10, x, labels=labels, storage="exact")


FULL_BATCH_GROUPS = [(0, 1), (1, 2), (2, 3), (3, 5), (5, 8), (8, 15), (15, 22)]


@pytest.mark.parametrize("lo,hi", FULL_BATCH_GROUPS, ids=[f"units{lo}-{hi - 1}" for lo, hi in FULL_BATCH_GROUPS])
def test_config5_full_batch_every_unit_against_the_oracle(lo, hi):
    """Batch 128, the shapes bench.py times (1.6 M rows at 112x112, 462 MB tensors, the row-range loops of the
    streaming GEMM, the persistent depthwise weight-gradient blocks).  The float64 oracle cannot hold a step of that
    size, so the batch is 8 copies of a seeded batch of 16: the batch statistics of such a batch are those of one
    copy, every forward tensor and data gradient is the tiled small one and the weight gradients are equal (see
    Pair(tile=...)), and every element of the full-size outputs is compared with the oracle's, unit by unit,
    teacher-forced on seeded inputs of the unit's real shape, at 2e-2."""
    print(f"config 5 at batch 128 = 8 x 16, units [{lo},{hi})", flush=True)
    from oracle.stage import bf16_round
    o_units, h_units = OM.mobilenet_v2(1.4, 1000, 2), hip_models().mobilenet_v2_units(1.4, 1000, 2)
    shapes = unit_shapes(o_units, (224, 224, 3))
    labels = synth.labels(12, "labels", 16, 1000)
    for i in range(lo, hi):
        kind = o_units[i].kind
        print(f"  unit {i} ({kind}) in {shapes[i]} out {shapes[i + 1]}", flush=True)
        pair = Pair(o_units, h_units, (224, 224, 3), 128, i, i + 1, "bf16", seed=12, ties="bounded", tile=8)
        try:
            x = bf16_round(synth.normal(12, f"x{i}", (16,) + tuple(shapes[i])))
            dy = bf16_round(synth.normal(12, f"dy{i}", (16,) + tuple(shapes[i + 1]), std=1.0 / 16))
            rep = []
            unit_compare(pair, i, kind, x, dy, labels, TOL["bf16"], rep)
            print("   ", rep[0][2:], flush=True)
        finally:
            pair.close()


def test_config5_full_batch_sampled_outputs_and_invariants():
    """Batch 128 in the configuration bench.py times.  The oracle cannot run the whole step at
    this size in reasonable time, so: (i) sampled outputs of the stem convolution are recomputed
    one by one from the definition; (ii) properties that hold at any size are checked on every
    BatchNorm: the normalised output has mean beta and variance gamma^2 var/(var+eps) per channel,
    i.e. scale*mean + shift = beta; (iii) gradients are finite, d(beta) of the last BatchNorm
    before a normalised consumer vanishes, and rows of the logits gradient sum to zero through FC
    bias: d(b) sums to ~0."""
    import torch
    import paper_2110_02781_amd as P
    print("config 5 full batch 128 bf16", flush=True)
    batch = 128
    h_units = P.models.mobilenet_v2_units(1.4, 1000, 2)
    model = P.model_create(h_units, 224, 224, 3, P.BF16)
    stage = P.stage_create(model, 0, 22, batch, 1)
    try:
        hp = P.models.init_unit_params(h_units, 12)
        for i in range(22):
            P.stage_import_weights(stage, i, hp[i])
        x = synth.normal(12, "x", (batch, 224, 224, 3)).astype(np.float32)
        xd = torch.from_numpy(x).cuda().to(torch.bfloat16)
        labels = torch.from_numpy(synth.labels(12, "labels", batch, 1000)).cuda()
        loss = torch.zeros(1, device="cuda")
        logits = torch.empty(batch, 1000, dtype=torch.bfloat16, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        P.stage_forward(stage, 0, xd, logits, st)
        P.stage_loss(stage, 0, labels, loss, st)
        torch.cuda.synchronize()
        # (i) sampled stem outputs from the definition (float64) on the bf16-rounded operands
        xr = xd.float().cpu().numpy().astype(np.float64)
        w = torch.from_numpy(hp[0][:48 * 27]).to(torch.bfloat16).float().numpy().astype(np.float64).reshape(48, 3, 3, 3)
        z = P.stage_export_conv_output(stage, 0, 0, 0, batch * 112 * 112 * 48).reshape(batch, 112, 112, 48)
        idx = synth.bits(12, "sample", 600) % np.uint64(batch * 112 * 112)
        worst = 0.0
        for t in idx:
            t = int(t)
            n, r = divmod(t, 112 * 112)
            ho, wo = divmod(r, 112)
            acc = np.zeros(48)
            for i in range(3):
                for j in range(3):
                    hi, wi = 2 * ho + i - 1, 2 * wo + j - 1
                    if 0 <= hi < 224 and 0 <= wi < 224:
                        acc += w[:, i, j, :] @ xr[n, hi, wi, :]
            worst = max(worst, np.abs(z[n, ho, wo] - acc).max() / max(np.abs(acc).max(), 1e-6))
        print(f"sampled stem outputs: worst rel err {worst:.2e}", flush=True)
        assert worst <= TOL["bf16"]
        # (ii) BatchNorm invariants on every convolution of a few units (full tensors, float64 on host)
        for (u, k, C, n) in [(0, 0, 48, batch * 112 * 112 * 48), (2, 2, 32, batch * 56 * 56 * 32), (17, 0, 1344, batch * 7 * 7 * 1344),
                             (18, 0, 1792, batch * 7 * 7 * 1792)]:
            zz = P.stage_export_conv_output(stage, 0, u, k, n).reshape(-1, C).astype(np.float64)
            s = P.stage_export_bn_batch_stats(stage, 0, u, k, 4 * C).astype(np.float64)
            mean, var = zz.mean(0), zz.var(0)
            assert_close(s[:C], mean, 1e-4, f"unit {u} conv {k} batch mean", scale_ref=np.sqrt(var + mean ** 2))
            assert_close(s[C:2 * C], 1 / np.sqrt(var + 1e-5), 1e-4, f"unit {u} conv {k} invstd")
            ynorm = zz * s[2 * C:3 * C] + s[3 * C:]
            assert np.abs(ynorm.mean(0)).max() < 1e-4 and np.abs(ynorm.var(0) - var / (var + 1e-5)).max() < 1e-3
        lval = float(loss.item())
        print(f"loss {lval:.4f}", flush=True)
        assert np.isfinite(lval) and 5.0 < lval < 12.0
        # (iii) backward invariants
        P.stage_backward(stage, 0, None, None, st)
        torch.cuda.synchronize()
        for i in range(22):
            n = P.model_unit_param_count(model, i)
            if n:
                g = P.stage_export_grads(stage, i, n)
                assert np.all(np.isfinite(g)), f"unit {i} gradient not finite"
        gfc = P.stage_export_grads(stage, 20, 1792 * 1000 + 1000)
        assert abs(gfc[-1000:].sum()) < 1e-2          # rows of (softmax - onehot)/B sum to zero (bf16-rounded)
        g19 = P.stage_export_grads(stage, 19 - 1, P.model_unit_param_count(model, 18))
        assert np.abs(g19).max() > 0
    finally:
        P.stage_destroy(stage)
        P.model_destroy(model)
