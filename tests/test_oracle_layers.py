"""Pins for the oracle's layer functions: a library routine (PyTorch CPU ops and
autograd, float64), closed forms, adjoint identities and central finite
differences.  None of these re-uses the oracle's own formula."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layers as L

rng = np.random.default_rng(1234)


def t_nchw(x):
    return torch.from_numpy(np.ascontiguousarray(x.transpose(0, 3, 1, 2)))


def t_w(w):  # [Cout,kh,kw,Cg] -> [Cout,Cg,kh,kw]
    return torch.from_numpy(np.ascontiguousarray(w.transpose(0, 3, 1, 2)))


CONV_CASES = [
    # N,H,W,Cin,Cout,kh,kw,s,ph,pw,groups
    (2, 7, 6, 3, 5, 3, 3, 1, 1, 1, 1),
    (2, 9, 8, 3, 4, 3, 3, 2, 1, 1, 1),
    (2, 8, 8, 6, 6, 3, 3, 1, 1, 1, 6),      # depthwise
    (2, 9, 7, 6, 6, 3, 3, 2, 1, 1, 6),      # depthwise stride 2, odd sizes
    (3, 1, 17, 4, 7, 1, 5, 1, 0, 2, 1),     # conv1d as H=1
    (2, 5, 5, 8, 12, 1, 1, 1, 0, 0, 1),     # pointwise
    (2, 6, 6, 4, 6, 3, 3, 1, 1, 1, 2),      # grouped
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matches_library_forward_and_backward(case):
    N, H, W, Cin, Cout, kh, kw, s, ph, pw, g = case
    x = rng.standard_normal((N, H, W, Cin))
    w = rng.standard_normal((Cout, kh, kw, Cin // g))
    y = L.conv2d_fwd(x, w, s, ph, pw, g)
    xt, wt = t_nchw(x).requires_grad_(), t_w(w).requires_grad_()
    yt = F.conv2d(xt, wt, None, stride=s, padding=(ph, pw), groups=g)
    np.testing.assert_allclose(y, yt.detach().numpy().transpose(0, 2, 3, 1), rtol=1e-12, atol=1e-12)
    dy = rng.standard_normal(y.shape)
    yt.backward(t_nchw(dy))
    dx, dw = L.conv2d_bwd(x, w, dy, s, ph, pw, g)
    np.testing.assert_allclose(dx, xt.grad.numpy().transpose(0, 2, 3, 1), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw, wt.grad.numpy().transpose(0, 2, 3, 1), rtol=1e-12, atol=1e-12)


def test_conv_delta_kernel_is_shift():
    x = rng.standard_normal((2, 6, 7, 3))
    for (i, j) in [(1, 1), (0, 1), (2, 2), (1, 0)]:
        w = np.zeros((3, 3, 3, 1))
        w[:, i, j, 0] = 1.0
        y = L.conv2d_fwd(x, w, 1, 1, 1, groups=3)
        ref = np.zeros_like(x)
        for h in range(6):
            for ww in range(7):
                hs, ws = h + i - 1, ww + j - 1
                if 0 <= hs < 6 and 0 <= ws < 7:
                    ref[:, h, ww] = x[:, hs, ws]
        np.testing.assert_array_equal(y, ref)


def test_conv_ones_counts_in_bounds_taps():
    x = np.ones((1, 5, 6, 2))
    w = np.ones((1, 3, 3, 2))
    y = L.conv2d_fwd(x, w, 1, 1, 1)[0, :, :, 0]
    assert y[0, 0] == 8 and y[0, 2] == 12 and y[2, 2] == 18 and y[4, 5] == 8
    y2 = L.conv2d_fwd(x, w, 2, 1, 1)[0, :, :, 0]
    np.testing.assert_array_equal(y2, y[::2, ::2])


def test_pointwise_is_matrix_product():
    x = rng.standard_normal((2, 3, 4, 5))
    w = rng.standard_normal((7, 1, 1, 5))
    y = L.conv2d_fwd(x, w, 1, 0, 0)
    ref = np.einsum('nhwc,oc->nhwo', x, w[:, 0, 0, :])
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)


def test_depthwise_equals_block_diagonal_dense():
    x = rng.standard_normal((2, 6, 6, 4))
    wd = rng.standard_normal((4, 3, 3, 1))
    dense = np.zeros((4, 3, 3, 4))
    for c in range(4):
        dense[c, :, :, c] = wd[c, :, :, 0]
    for s in (1, 2):
        np.testing.assert_allclose(L.conv2d_fwd(x, wd, s, 1, 1, 4), L.conv2d_fwd(x, dense, s, 1, 1, 1), atol=1e-13)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_adjoint_identities(case):
    N, H, W, Cin, Cout, kh, kw, s, ph, pw, g = case
    x = rng.standard_normal((N, H, W, Cin))
    w = rng.standard_normal((Cout, kh, kw, Cin // g))
    y = L.conv2d_fwd(x, w, s, ph, pw, g)
    dy = rng.standard_normal(y.shape)
    dx, dw = L.conv2d_bwd(x, w, dy, s, ph, pw, g)
    lhs = (y * dy).sum()
    assert abs(lhs - (x * dx).sum()) < 1e-10 * max(1, abs(lhs))
    assert abs(lhs - (w * dw).sum()) < 1e-10 * max(1, abs(lhs))


def _fd(f, x, idx, h=1e-6):
    xp, xm = x.copy(), x.copy()
    xp[idx] += h
    xm[idx] -= h
    return (f(xp) - f(xm)) / (2 * h)


def test_conv_finite_differences():
    x = rng.standard_normal((2, 5, 5, 3))
    w = rng.standard_normal((4, 3, 3, 3))
    r = rng.standard_normal((2, 3, 3, 4))
    dx, dw = L.conv2d_bwd(x, w, r, 2, 1, 1)
    for idx in [(0, 0, 0, 0), (1, 4, 4, 2), (0, 2, 3, 1)]:
        assert abs(_fd(lambda v: (L.conv2d_fwd(v, w, 2, 1, 1) * r).sum(), x, idx) - dx[idx]) < 1e-6
    for idx in [(0, 0, 0, 0), (3, 2, 2, 2), (1, 1, 2, 0)]:
        assert abs(_fd(lambda v: (L.conv2d_fwd(x, v, 2, 1, 1) * r).sum(), w, idx) - dw[idx]) < 1e-6


def test_bn_forward_closed_forms_and_library():
    z = rng.standard_normal((4, 3, 5, 6)) * 3 + 2
    g, b = rng.standard_normal(6), rng.standard_normal(6)
    y1, mean, invstd, var = L.bn_fwd(z, np.ones(6), np.zeros(6))
    np.testing.assert_allclose(y1.mean(axis=(0, 1, 2)), 0, atol=1e-13)
    np.testing.assert_allclose(y1.var(axis=(0, 1, 2)), var / (var + L.BN_EPS), rtol=1e-12)
    zc = z.copy(); zc[..., 2] = 7.5
    yc = L.bn_fwd(zc, g, b)[0]
    np.testing.assert_allclose(yc[..., 2], b[2], atol=1e-12)
    ysh = L.bn_fwd(z * 4 + 11, g, b)[0]
    np.testing.assert_allclose(ysh, L.bn_fwd(z, g, b)[0], atol=1e-5)
    # library: training-mode batch_norm incl. running statistics
    rm, rv = torch.zeros(6, dtype=torch.float64), torch.ones(6, dtype=torch.float64)
    yt = F.batch_norm(t_nchw(z), rm, rv, torch.from_numpy(g), torch.from_numpy(b), True, L.BN_MOMENTUM, L.BN_EPS)
    np.testing.assert_allclose(L.bn_fwd(z, g, b)[0], yt.numpy().transpose(0, 2, 3, 1), rtol=1e-11, atol=1e-11)
    nrm, nrv = L.bn_running_update(np.zeros(6), np.ones(6), mean, var, 4 * 3 * 5)
    np.testing.assert_allclose(nrm, rm.numpy(), rtol=1e-12)
    np.testing.assert_allclose(nrv, rv.numpy(), rtol=1e-12)


def test_bn_backward_invariants_library_and_fd():
    z = rng.standard_normal((3, 4, 4, 5)) * 2 + 1
    g, b = rng.standard_normal(5), rng.standard_normal(5)
    dy = rng.standard_normal(z.shape)
    y, mean, invstd, var = L.bn_fwd(z, g, b)
    dx, dg, db = L.bn_bwd(dy, z, mean, invstd, g)
    xhat = (z - mean) * invstd
    np.testing.assert_allclose(dx.sum(axis=(0, 1, 2)), 0, atol=1e-12)
    # sum(xhat^2) = M*var/(var+eps), so the second invariant holds up to the eps term
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 1, 2)), g * invstd * dg * L.BN_EPS * invstd ** 2,
                               rtol=1e-6, atol=1e-12)
    assert np.abs((dx * xhat).sum(axis=(0, 1, 2))).max() < 1e-4
    zt = t_nchw(z).requires_grad_()
    gt, bt = torch.from_numpy(g).requires_grad_(), torch.from_numpy(b).requires_grad_()
    yt = F.batch_norm(zt, None, None, gt, bt, True, 0.1, L.BN_EPS)
    yt.backward(t_nchw(dy))
    np.testing.assert_allclose(dx, zt.grad.numpy().transpose(0, 2, 3, 1), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(dg, gt.grad.numpy(), rtol=1e-11)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-11)
    f = lambda v: (L.bn_fwd(v, g, b)[0] * dy).sum()
    for idx in [(0, 0, 0, 0), (2, 3, 1, 4)]:
        assert abs(_fd(f, z, idx) - dx[idx]) < 1e-6


def test_activations_and_gap_closed_forms():
    y = np.array([-1.0, 0.0, 0.5, 6.0, 7.0])
    np.testing.assert_array_equal(L.act_fwd(y, L.ACT_RELU6), [0, 0, 0.5, 6, 6])
    np.testing.assert_array_equal(L.act_fwd(y, L.ACT_RELU), [0, 0, 0.5, 6, 7])
    np.testing.assert_array_equal(L.act_bwd(np.ones(5), y, L.ACT_RELU6), [0, 0, 1, 0, 0])
    np.testing.assert_array_equal(L.act_bwd(np.ones(5), y, L.ACT_RELU), [0, 0, 1, 1, 1])
    np.testing.assert_array_equal(L.act_bwd(np.ones(5), y, L.ACT_NONE), np.ones(5))
    x = np.full((2, 3, 4, 5), 2.5)
    np.testing.assert_array_equal(L.gap_fwd(x), np.full((2, 5), 2.5))
    x = rng.standard_normal((2, 3, 4, 5))
    np.testing.assert_allclose(L.gap_fwd(x)[1, 2], x[1, :, :, 2].sum() / 12)
    d = rng.standard_normal((2, 5))
    dx = L.gap_bwd(d, 3, 4)
    assert dx.shape == (2, 3, 4, 5)
    np.testing.assert_allclose(dx[1, 2, 3], d[1] / 12)


def test_fc_matches_library():
    x, w, b = rng.standard_normal((4, 7)), rng.standard_normal((3, 7)), rng.standard_normal(3)
    xt, wt, bt = [torch.from_numpy(v).requires_grad_() for v in (x, w, b)]
    yt = F.linear(xt, wt, bt)
    np.testing.assert_allclose(L.fc_fwd(x, w, b), yt.detach().numpy(), rtol=1e-13)
    dy = rng.standard_normal((4, 3))
    yt.backward(torch.from_numpy(dy))
    dx, dw, db = L.fc_bwd(x, w, dy)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-12)


def test_softmax_ce_closed_forms_library_and_fd():
    loss, d = L.softmax_ce(np.zeros((4, 6)), np.array([0, 5, 2, 2]))
    assert abs(loss - np.log(6)) < 1e-14
    z = rng.standard_normal((5, 7)) * 3
    lab = np.array([0, 6, 3, 3, 1])
    loss, d = L.softmax_ce(z, lab)
    np.testing.assert_allclose(d.sum(axis=1), 0, atol=1e-15)
    zt = torch.from_numpy(z).requires_grad_()
    lt = F.cross_entropy(zt, torch.from_numpy(lab).long())
    lt.backward()
    assert abs(loss - lt.item()) < 1e-13
    np.testing.assert_allclose(d, zt.grad.numpy(), rtol=1e-11, atol=1e-14)
    for idx in [(0, 0), (4, 1), (2, 6)]:
        assert abs(_fd(lambda v: L.softmax_ce(v, lab)[0], z, idx) - d[idx]) < 1e-8
    big = L.softmax_ce(np.array([[1000.0, 0.0]]), np.array([1]))[0]
    assert abs(big - 1000.0) < 1e-9


def test_sgd_closed_forms_and_library():
    w0 = rng.standard_normal(5)
    g = rng.standard_normal(5)
    lr, mu = 0.01, 0.9
    w, v = w0.copy(), np.zeros(5)
    acc = np.zeros(5)
    for k in range(1, 8):
        w, v = L.sgd_momentum(w, g, v, lr, mu, 0.0)
        np.testing.assert_allclose(v, g * (1 - mu ** k) / (1 - mu), rtol=1e-12)
        acc += g * (1 - mu ** k) / (1 - mu)
        np.testing.assert_allclose(w, w0 - lr * acc, rtol=1e-12, atol=1e-14)
    w, v = L.sgd_momentum(w0, g, np.zeros(5), lr, 0.0, 0.0)
    np.testing.assert_allclose(w, w0 - lr * g, rtol=1e-14)
    w = w0.copy(); v = np.zeros(5)
    for k in range(1, 5):
        w, v = L.sgd_momentum(w, np.zeros(5), v, lr, 0.0, 0.1)
        np.testing.assert_allclose(w, w0 * (1 - lr * 0.1) ** k, rtol=1e-13)
    # library optimiser, three steps with changing gradients, momentum and weight decay
    wt = torch.from_numpy(w0.copy()).requires_grad_()
    opt = torch.optim.SGD([wt], lr=lr, momentum=mu, weight_decay=4e-5)
    w, v = w0.copy(), np.zeros(5)
    for k in range(3):
        gk = rng.standard_normal(5)
        wt.grad = torch.from_numpy(gk.copy())
        opt.step()
        w, v = L.sgd_momentum(w, gk, v, lr, mu, 4e-5)
        np.testing.assert_allclose(w, wt.detach().numpy(), rtol=1e-13)
