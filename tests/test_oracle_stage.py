"""Pins for the oracle's stage step: the same network assembled from PyTorch CPU
operators with autograd and torch.optim.SGD (library pin), finite differences
of the scalar loss through the whole 1-D CNN, split invariance, and the
paper's worked one-forward-one-backward / weight-stashing example."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle import layers as L
from oracle import models as M
from oracle.stage import Stage, one_f_one_b_order

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_stage(units, in_shape, a, b, seed, n_slots=1):
    st = Stage(units, in_shape, a, b, n_slots)
    P = M.init_params(units, seed)
    for i in range(a, b):
        st.set_params(i, P[i])
    return st


# ------------------------------------------------------------ library network
def torch_forward(units, params, x, labels):
    """The same network from library operators (NCHW, float64, autograd)."""
    def cba(h, w, g, b, stride, pad, groups, act):
        h = F.conv2d(h, w.permute(0, 3, 1, 2), None, stride=stride, padding=pad, groups=groups)
        h = F.batch_norm(h, None, None, g, b, True, 0.1, L.BN_EPS)
        return F.relu6(h) if act == L.ACT_RELU6 else F.relu(h) if act == L.ACT_RELU else h
    h = x
    for u, P in zip(units, params):
        if u.kind == 'conv':
            h = cba(h, P[0], P[1], P[2], u.stride, (u.pad_h, u.pad_w), 1, u.act)
        elif u.kind == 'invres':
            inp, k = h, 0
            ce = u.cin * u.expand
            if u.expand != 1:
                h = cba(h, P[0], P[1], P[2], 1, 0, 1, L.ACT_RELU6); k = 3
            h = cba(h, P[k], P[k + 1], P[k + 2], u.stride, 1, ce, L.ACT_RELU6)
            h = cba(h, P[k + 3], P[k + 4], P[k + 5], 1, 0, 1, L.ACT_NONE)
            if u.stride == 1 and u.cin == u.cout:
                h = h + inp
        elif u.kind == 'gap':
            h = h.mean(dim=(2, 3))
        elif u.kind == 'fc':
            h = F.linear(h, P[0], P[1])
        elif u.kind == 'loss':
            return F.cross_entropy(h, labels)
    return h


def small_mbv2():
    """Reduced block list with every block variant: t=1, stride 2, residual, plain."""
    return [M.Unit('conv', 3, 8, 3, 3, 1, 1, 1, act=L.ACT_RELU6),
            M.Unit('invres', 8, 8, 3, 3, 1, 1, 1, expand=1, act=L.ACT_RELU6),
            M.Unit('invres', 8, 16, 3, 3, 2, 1, 1, expand=6, act=L.ACT_RELU6),
            M.Unit('invres', 16, 16, 3, 3, 1, 1, 1, expand=6, act=L.ACT_RELU6),
            M.Unit('invres', 16, 24, 3, 3, 1, 1, 1, expand=6, act=L.ACT_RELU6),
            M.Unit('conv', 24, 32, 1, 1, 1, 0, 0, act=L.ACT_RELU6),
            M.Unit('gap', 32, 32), M.Unit('fc', 32, 10), M.Unit('loss', 10, 10)]


@pytest.mark.parametrize("name", ["cnn1d", "small_mbv2", "mbv2_full"])
def test_stage_step_matches_library_autograd(name):
    if name == "cnn1d":
        units, in_shape, batch, classes = M.cnn1d(), (1, 128, 9), 8, 6
    elif name == "small_mbv2":
        units, in_shape, batch, classes = small_mbv2(), (9, 9, 3), 4, 10
    else:
        units, in_shape, batch, classes = M.mobilenet_v2(1.0, 10, 1), (32, 32, 3), 4, 10
    seed = 7
    x = synth.normal(seed, "x", (batch,) + in_shape)
    labels = synth.labels(seed, "labels", batch, classes)
    st = make_stage(units, in_shape, 0, len(units), seed)
    lr, mu, wd = 0.01, 0.9, 4e-5
    tparams = [[torch.from_numpy(p.copy()).requires_grad_() for p in st.params[i]] for i in range(len(units))]
    flat = [p for ps in tparams for p in ps]
    opt = torch.optim.SGD(flat, lr=lr, momentum=mu, weight_decay=wd)
    xt = torch.from_numpy(x.transpose(0, 3, 1, 2).copy()).requires_grad_()
    lt = torch.from_numpy(labels).long()
    for step in range(2):
        st.forward(0, x)
        loss = st.loss(0, labels)
        grads_before = None
        dx = st.backward(0)
        opt.zero_grad()
        xt.grad = None
        tl = torch_forward(units, tparams, xt, lt)
        tl.backward()
        assert abs(loss - tl.item()) < 1e-10 * max(1, abs(loss))
        np.testing.assert_allclose(dx, xt.grad.numpy().transpose(0, 2, 3, 1), rtol=1e-6, atol=1e-10)
        for i in range(len(units)):
            for k, p in enumerate(tparams[i]):
                g = st.grads[i][k]
                scale = max(np.abs(p.grad.numpy()).max(), 1e-30)
                assert np.abs(g - p.grad.numpy()).max() <= 1e-8 * scale + 1e-12, (i, k)
        st.update(lr, mu, wd)
        opt.step()
        for i in range(len(units)):
            for k, p in enumerate(tparams[i]):
                np.testing.assert_allclose(st.params[i][k], p.detach().numpy(), rtol=1e-9, atol=1e-12)


def test_finite_differences_through_whole_cnn1d():
    units, in_shape = M.cnn1d(), (1, 32, 9)
    seed = 3
    x = synth.normal(seed, "x", (4,) + in_shape)
    labels = synth.labels(seed, "labels", 4, 6)
    st = make_stage(units, in_shape, 0, 6, seed)

    def loss_of():
        st.slots[0] = None
        st.forward(0, x)
        return st.loss(0, labels)
    loss_of()
    dx = st.backward(0)
    h = 1e-6
    for (i, k, idx) in [(0, 0, (3, 0, 2, 4)), (1, 0, (10, 0, 0, 7)), (2, 1, (5,)), (4, 0, (2, 11)), (4, 1, (3,)), (1, 2, (9,))]:
        p = st.params[i][k]
        old = p[idx]
        p[idx] = old + h; lp = loss_of()
        p[idx] = old - h; lm = loss_of()
        p[idx] = old
        assert abs((lp - lm) / (2 * h) - st.grads[i][k][idx]) < 1e-7, (i, k, idx)
    for idx in [(0, 0, 0, 0), (3, 0, 17, 5)]:
        old = x[idx]
        x[idx] = old + h; lp = loss_of()
        x[idx] = old - h; lm = loss_of()
        x[idx] = old
        assert abs((lp - lm) / (2 * h) - dx[idx]) < 1e-7


def test_split_invariance():
    """Chaining the stages of any contiguous split equals the whole model."""
    units, in_shape = small_mbv2(), (9, 9, 3)
    seed = 11
    x = synth.normal(seed, "x", (4,) + in_shape)
    labels = synth.labels(seed, "labels", 4, 10)
    whole = make_stage(units, in_shape, 0, len(units), seed)
    whole.forward(0, x)
    loss = whole.loss(0, labels)
    dx = whole.backward(0)
    for bounds in ([0, 2, 5, 9], [0, 1, 3, 4, 9], [0, 8, 9]):
        stages = [make_stage(units, in_shape, bounds[k], bounds[k + 1], seed) for k in range(len(bounds) - 1)]
        h = x
        for s in stages:
            h = s.forward(0, h)
        l2 = stages[-1].loss(0, labels)
        assert abs(l2 - loss) < 1e-13
        d = None
        for s in reversed(stages):
            d = s.backward(0, d)
        np.testing.assert_allclose(d, dx, rtol=1e-12, atol=1e-15)
        for s in stages:
            for i in range(s.a, s.b):
                for k in range(len(s.grads[i])):
                    np.testing.assert_allclose(s.grads[i][k], whole.grads[i][k], rtol=1e-11, atol=1e-15)


def read_trace():
    rows = []
    for line in open(os.path.join(GOLDEN, "onef1b_versions.txt")):
        if line.strip() and not line.startswith("#"):
            op, b, v = line.split()
            rows.append((op, int(b), int(v)))
    return rows


def test_one_f_one_b_order_and_versions_match_paper_example():
    trace = read_trace()
    order = one_f_one_b_order(0, 3, 6)
    assert order[:len(trace)] == [(op, b) for op, b, _ in trace]
    # replay on a real stage: the version a pass uses is identified by the weights it sees
    units, in_shape = M.cnn1d(channels=(8, 8, 8)), (1, 16, 9)
    seed = 5
    st = make_stage(units, in_shape, 0, 3, seed, n_slots=3)
    versions = {0: [p.copy() for p in st.params[0]]}
    fwd_version, version = {}, 0
    for op, b, v in trace:
        x = synth.normal(seed, f"x{b}", (2,) + in_shape)
        if op == 'F':
            st.forward(b % 3, x)
            fwd_version[b] = version
            assert version == v
            assert all(np.array_equal(p, q) for p, q in zip(st.slots[b % 3]['params'][0], versions[v]))
        else:
            assert fwd_version[b] == v
            assert all(np.array_equal(p, q) for p, q in zip(st.slots[b % 3]['params'][0], versions[v]))
            st.backward(b % 3, synth.normal(seed, f"dy{b}", (2, 1, 16, 8)))
            st.update(0.01, 0.9, 0.0)
            version += 1
            versions[version] = [p.copy() for p in st.params[0]]
    assert one_f_one_b_order(0, 3, 4) == [('F', 0), ('F', 1), ('F', 2), ('B', 0), ('F', 3), ('B', 1), ('B', 2), ('B', 3)]
    assert one_f_one_b_order(2, 3, 3) == [('F', 0), ('B', 0), ('F', 1), ('B', 1), ('F', 2), ('B', 2)]


def test_weight_stashing_differs_from_current_weights_and_lr0_equals_sync():
    units, in_shape = M.cnn1d(channels=(8, 8, 8)), (1, 16, 9)
    seed = 9
    xs = [synth.normal(seed, f"x{b}", (2,) + in_shape) for b in range(4)]
    dys = [synth.normal(seed, f"dy{b}", (2, 1, 16, 8)) for b in range(4)]

    def run(lr, stash, sync):
        st = make_stage(units, in_shape, 0, 3, seed, n_slots=3)
        tot = None
        for op, b in one_f_one_b_order(0, 3, 4):
            if op == 'F':
                st.forward(b % 3, xs[b], stash_weights=stash)
            else:
                st.backward(b % 3, dys[b])
                if not sync:
                    g = [x.copy() for x in st.grads[0]]
                    tot = g if tot is None else [a + c for a, c in zip(tot, g)]
                    st.update(lr, 0.9, 0.0)
        return st, (st.grads[0] if sync else tot)
    _, g_async0 = run(0.0, True, False)
    _, g_sync = run(0.0, True, True)
    for p, q in zip(g_async0, g_sync):
        np.testing.assert_allclose(p, q, rtol=1e-12, atol=1e-15)
    a, _ = run(0.05, True, False)
    c, _ = run(0.05, False, False)
    assert np.abs(a.params[0][0] - c.params[0][0]).max() > 1e-6


def test_bf16_rounding_matches_library_conversion():
    from oracle.stage import bf16_round
    v = np.concatenate([synth.normal(1, "r", (4096,)) * 10.0 ** synth.integers(1, "e", (4096,), -6, 6),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, -2.5e-40])])
    ref = torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16).float().numpy().astype(np.float64)
    np.testing.assert_array_equal(bf16_round(v), ref)
    # ties go to the even mantissa: 1 + 2^-8 is half way between 1 and 1 + 2^-7
    assert bf16_round(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert bf16_round(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6


def test_bf16_storage_mode_stays_close_to_exact_and_rounds_stored_tensors():
    from oracle.stage import bf16_round
    units, in_shape = small_mbv2(), (9, 9, 3)
    x = bf16_round(synth.normal(2, "x", (4,) + in_shape))
    labels = synth.labels(2, "labels", 4, 10)
    P = M.init_params(units, 2)
    out = []
    for storage in (None, 'bf16'):
        st = Stage(units, in_shape, 0, len(units), 1, storage=storage)
        for i in range(len(units)):
            st.set_params(i, P[i])
        y = st.forward(0, x)
        loss = st.loss(0, labels)
        st.backward(0)
        out.append((y, loss, st.grads[2][0]))
        if storage == 'bf16':
            np.testing.assert_array_equal(y, bf16_round(y))
    assert abs(out[0][1] - out[1][1]) < 0.05 * abs(out[0][1])
    assert np.abs(out[0][2] - out[1][2]).max() < 0.5 * np.abs(out[0][2]).max()


class _StoreBF16(torch.autograd.Function):
    """A tensor stored in bfloat16: the value is rounded on the way forward and its gradient on the way back
    (the library's own conversion, round to nearest even, does both roundings)."""
    @staticmethod
    def forward(ctx, t):
        return t.to(torch.bfloat16).to(t.dtype)

    @staticmethod
    def backward(ctx, g):
        return g.to(torch.bfloat16).to(g.dtype)


class _WorkingCopyBF16(torch.autograd.Function):
    """The bfloat16 working copy of a weight: rounded forward; the weight gradient stays in full precision."""
    @staticmethod
    def forward(ctx, t):
        return t.to(torch.bfloat16).to(t.dtype)

    @staticmethod
    def backward(ctx, g):
        return g


def torch_forward_bf16_storage(units, params, x, labels):
    """The network of torch_forward with every tensor that mixed-precision training stores in bfloat16 passed
    through _StoreBF16: the working copy of conv / FC weights, every convolution output, every BatchNorm +
    activation output, block outputs, pooled features, logits; BatchNorm statistics, gamma, beta and the loss stay
    in float64."""
    R, Rw = _StoreBF16.apply, _WorkingCopyBF16.apply

    def cba(h, w, g, b, stride, pad, groups, act):
        z = R(F.conv2d(h, Rw(w).permute(0, 3, 1, 2), None, stride=stride, padding=pad, groups=groups))
        y = F.batch_norm(z, None, None, g, b, True, 0.1, L.BN_EPS)
        return R(F.relu6(y) if act == L.ACT_RELU6 else F.relu(y) if act == L.ACT_RELU else y)
    h = x
    for u, P in zip(units, params):
        if u.kind == 'conv':
            h = cba(h, P[0], P[1], P[2], u.stride, (u.pad_h, u.pad_w), 1, u.act)
        elif u.kind == 'invres':
            inp, k = h, 0
            ce = u.cin * u.expand
            if u.expand != 1:
                h = cba(h, P[0], P[1], P[2], 1, 0, 1, L.ACT_RELU6); k = 3
            h = cba(h, P[k], P[k + 1], P[k + 2], u.stride, 1, ce, L.ACT_RELU6)
            h = cba(h, P[k + 3], P[k + 4], P[k + 5], 1, 0, 1, L.ACT_NONE)
            if u.stride == 1 and u.cin == u.cout:
                h = h + inp
            h = R(h)
        elif u.kind == 'gap':
            h = R(h.mean(dim=(2, 3)))
        elif u.kind == 'fc':
            h = R(F.linear(h, Rw(P[0]), P[1]))
        elif u.kind == 'loss':
            return F.cross_entropy(h, labels), h
    return h, h


@pytest.mark.parametrize("name", ["cnn1d", "small_mbv2"])
def test_bf16_storage_mode_rounds_exactly_at_the_stated_points(name):
    """Pin of the storage='bf16' oracle: the same step from library operators and autograd in float64, with the
    library's own bfloat16 conversion inserted at the storage points (forward value and backward gradient), must give
    the same logits, loss, input gradient and weight gradients to float64 accuracy.  A rounding that the oracle
    misses, adds or puts elsewhere shows up at the 1e-3 level."""
    from oracle.stage import bf16_round
    if name == "cnn1d":
        units, in_shape, batch, classes = M.cnn1d(), (1, 128, 9), 8, 6
    else:
        units, in_shape, batch, classes = small_mbv2(), (9, 9, 3), 4, 10
    seed = 23
    x = bf16_round(synth.normal(seed, "x", (batch,) + in_shape))
    labels = synth.labels(seed, "labels", batch, classes)
    st = Stage(units, in_shape, 0, len(units), 1, storage='bf16')
    P = M.init_params(units, seed)
    for i in range(len(units)):
        st.set_params(i, [p.astype(np.float32).astype(np.float64) for p in P[i]])
    logits = st.forward(0, x)
    loss = st.loss(0, labels)
    dx = st.backward(0)
    tparams = [[torch.from_numpy(p.copy()).requires_grad_() for p in st.params[i]] for i in range(len(units))]
    xt = torch.from_numpy(x.transpose(0, 3, 1, 2).copy()).requires_grad_()
    tl, tlogits = torch_forward_bf16_storage(units, tparams, xt, torch.from_numpy(labels).long())
    tl.backward()
    np.testing.assert_array_equal(logits.reshape(batch, -1), tlogits.detach().numpy())       # stored values: identical
    assert abs(loss - tl.item()) < 1e-12 * max(1, abs(loss))
    # the gradient that reaches the input is a stored tensor too: the oracle returns it rounded
    want_dx = bf16_round(xt.grad.numpy().transpose(0, 2, 3, 1))
    flips = (dx != want_dx).mean()
    assert flips <= 1e-3 and np.abs(dx - want_dx).max() <= 2.0 ** -7 * np.abs(want_dx).max(), flips
    for i in range(len(units)):
        for k, p in enumerate(tparams[i]):
            g, ref = st.grads[i][k], p.grad.numpy()
            assert np.abs(g - ref).max() <= 1e-9 * max(np.abs(ref).max(), 1e-30) + 1e-14, (i, k, np.abs(g - ref).max(), np.abs(ref).max())


def test_tie_breaks_only_act_inside_the_band():
    """Decisions handed to backward are adopted only within the rounding band around a
    kink; elsewhere the oracle keeps its own and counts the disagreement."""
    units, in_shape = M.cnn1d(channels=(8, 8, 8)), (1, 16, 9)
    x = synth.normal(4, "x", (2,) + in_shape)
    dy = synth.normal(4, "dy", (2, 1, 16, 8))
    P = M.init_params(units, 4)

    def run(ties, guard):
        st = Stage(units, in_shape, 0, 1)
        st.set_params(0, P[0])
        st.forward(0, x)
        y = st.slots[0]['caches'][0][0]['y']
        d = st.backward(0, dy, tie_breaks=None if ties is None else {(0, 0): ties(y)}, guard=guard)
        return d, st.tie_report, y
    base, _, y = run(None, 0.0)
    same, rep, _ = run(lambda y: y > 0, 1e-5)
    np.testing.assert_array_equal(base, same)
    assert rep['disagree'] == 0 and rep['adopted'] == 0
    # flipping everything: outside the band nothing changes and every element is reported
    flipped, rep, _ = run(lambda y: y <= 0, 1e-9)
    assert rep['disagree'] + rep['adopted'] == y.size and rep['adopted'] == rep['ties']
    if rep['ties'] == 0:
        np.testing.assert_array_equal(base, flipped)
    # a huge band adopts the caller's decisions, which changes the gradient
    adopted, rep, _ = run(lambda y: y <= 0, 1e3)
    assert rep['adopted'] == y.size and np.abs(adopted - base).max() > 1e-3


def test_version_trace_with_aggregation_matches_paper_example():
    """Pin: the version numbers the paper prints for its three-device example, aggregation included."""
    from oracle.stage import version_trace
    want = []
    for line in open(os.path.join(GOLDEN, "onef1b_aggregation.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        if f[0] == 'A':
            want.append(('A', tuple(int(x) for x in f[1].split(',')), int(f[2])))
        else:
            want.append((f[0], int(f[1]), int(f[2])))
    got = version_trace(0, 3, 9, aggregate=True)
    assert got[:len(want)] == want
    # without aggregation the trace is the plain stashing example
    plain = version_trace(0, 3, 6)
    assert plain[:10] == [('F', 0, 0), ('F', 1, 0), ('F', 2, 0), ('B', 0, 0), ('F', 3, 1), ('B', 1, 0), ('F', 4, 2),
                          ('B', 2, 0), ('F', 5, 3), ('B', 3, 1)]
    # the last stage holds one version at a time: aggregating one version changes nothing but the counter
    last = version_trace(2, 3, 3, aggregate=True)
    assert [e for e in last if e[0] == 'A'] == [('A', (1,), 2), ('A', (3,), 4)]


def test_aggregate_is_the_mean_of_the_stashed_versions():
    """Pins: mean of identical versions is that version; mean of two versions is their midpoint; momentum and
    gradients untouched; a stage whose slots all hold the live weights is unchanged."""
    units = M.cnn1d()
    st = Stage(units, (1, 16, 9), 0, len(units), n_slots=3)
    st.params = M.init_params(units, 7)
    x = synth.normal(7, "x", (4, 1, 16, 9))
    labels = synth.labels(7, "l", 4, 6)
    w0 = [[p.copy() for p in st.params[i]] for i in range(len(units))]
    st.forward(0, x); st.loss(0, labels)
    st.forward(1, x)
    st.aggregate([0, 1])                      # both slots stashed the same version
    assert all(np.array_equal(p, q) for i in range(len(units)) for p, q in zip(st.params[i], w0[i]))
    st.backward(0); st.update(0.05, 0.9, 0.0)       # version 1
    w1 = [[p.copy() for p in st.params[i]] for i in range(len(units))]
    mom = [[m.copy() for m in st.mom[i]] for i in range(len(units))]
    st.forward(0, x)                           # slot 0 stashes version 1, slot 1 still version 0
    st.aggregate([0, 1])
    for i in range(len(units)):
        for p, a, b in zip(st.params[i], w0[i], w1[i]):
            np.testing.assert_allclose(p, (a.astype(np.float64) + b.astype(np.float64)) / 2, rtol=0, atol=1e-7)
    assert all(np.array_equal(m, n) for i in range(len(units)) for m, n in zip(st.mom[i], mom[i]))


# ------------------------------------------------------------ recomputation
def _run_1f1b(recompute, storage=None, n_batches=5):
    units, in_shape, seed = small_mbv2(), (8, 8, 3), 23
    st = Stage(units, in_shape, 0, len(units), n_slots=3, storage=storage, recompute=recompute)
    P = M.init_params(units, seed)
    for i in range(len(units)):
        st.set_params(i, P[i])
    xs = [synth.normal(seed, f"x{b}", (4,) + in_shape) for b in range(n_batches)]
    ls = [synth.labels(seed, f"l{b}", 4, 10) for b in range(n_batches)]
    losses, held = [], []
    for op, b in one_f_one_b_order(0, 3, n_batches):
        if op == 'F':
            st.forward(b % 3, xs[b])
            losses.append(st.loss(b % 3, ls[b]))
            held.append(st.slots[b % 3]['caches'] is None)
        else:
            st.backward(b % 3)
            st.update(0.05, 0.9, 4e-5)
    return st, losses, held


@pytest.mark.parametrize("storage", [None, "bf16"])
def test_recomputation_gives_the_same_training_run(storage):
    """Throwing the intermediates away and running the forward again from the stashed
    input and the stashed weight version changes nothing: weights, momentum, running
    statistics and losses along a one-forward-one-backward run are identical."""
    a, la, held_a = _run_1f1b(False, storage)
    b, lb, held_b = _run_1f1b(True, storage)
    assert not any(held_a) and all(held_b)          # the recomputing slots really hold no intermediates
    assert la == lb
    for i in range(len(a.units)):
        for p, q in zip(a.params[i], b.params[i]):
            assert np.array_equal(p, q)
        for p, q in zip(a.mom[i], b.mom[i]):
            assert np.array_equal(p, q)
        for (m0, v0), (m1, v1) in zip(a.bn_run[i], b.bn_run[i]):
            assert np.array_equal(m0, m1) and np.array_equal(v0, v1)


def test_recomputation_moves_running_statistics_once_per_batch():
    """Closed form: K training forwards of the same batch with fixed weights leave the
    running mean at (1 - 0.9^K) * mean and the running variance at 0.9^K + (1 - 0.9^K) * var
    (unbiased); a recomputation that counted as a training forward would give 0.9^(2K)."""
    units, in_shape, seed, K = small_mbv2(), (8, 8, 3), 29, 3
    st = Stage(units, in_shape, 0, 1, recompute=True)
    st.set_params(0, M.init_params(units, seed)[0])
    x = synth.normal(seed, "x", (4,) + in_shape)
    dy = synth.normal(seed, "dy", (4, 8, 8, 8))
    z = L.conv2d_fwd(x, st.params[0][0], 1, 1, 1, 1).reshape(-1, 8)
    for _ in range(K):
        st.forward(0, x)
        st.backward(0, dy)
    rm, rv = st.bn_run[0][0]
    f = 0.9 ** K
    np.testing.assert_allclose(rm, (1 - f) * z.mean(0), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(rv, f + (1 - f) * z.var(0, ddof=1), rtol=1e-12, atol=1e-14)
