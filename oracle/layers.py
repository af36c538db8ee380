"""Layer definitions of the oracle (test infrastructure; see package docstring).

The paper trains MobileNetV2 with SGD, momentum 0.9 and weight decay 4e-5
(section "Experiment Setup") and leaves the layers themselves to the deep
learning library it uses, so each function below is the standard definition of
the layer, its exact gradient, or the optimiser recurrence.

Layouts: activations [N, H, W, C] (channels fastest); convolution weights
[Cout, kh, kw, Cin/groups]; fully connected weights [out, in].
No blocking, fusion or reordering: one loop over kernel taps, one library
matrix product (or elementwise product for depthwise) per tap.
"""
import numpy as np


def conv_out_size(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


def _pad(x, ph, pw):
    N, H, W, C = x.shape
    xp = np.zeros((N, H + 2 * ph, W + 2 * pw, C), dtype=x.dtype)
    xp[:, ph:ph + H, pw:pw + W, :] = x
    return xp


def conv2d_fwd(x, w, stride, ph, pw, groups=1):
    """y[n,ho,wo,co] = sum_{i,j,ci} xpad[n, ho*s+i, wo*s+j, ci] * w[co,i,j,ci]."""
    N, H, W, Cin = x.shape
    Cout, kh, kw, Cg = w.shape
    assert Cin == Cg * groups and Cout % groups == 0
    Ho, Wo = conv_out_size(H, kh, stride, ph), conv_out_size(W, kw, stride, pw)
    xp = _pad(x, ph, pw)
    y = np.zeros((N, Ho, Wo, Cout), dtype=x.dtype)
    Og = Cout // groups
    for i in range(kh):
        for j in range(kw):
            patch = xp[:, i:i + (Ho - 1) * stride + 1:stride, j:j + (Wo - 1) * stride + 1:stride, :]
            if groups == 1:
                y += patch @ w[:, i, j, :].T
            elif Cg == 1 and Og == 1:                       # depthwise
                y += patch * w[:, i, j, 0]
            else:
                for g in range(groups):
                    y[..., g * Og:(g + 1) * Og] += patch[..., g * Cg:(g + 1) * Cg] @ w[g * Og:(g + 1) * Og, i, j, :].T
    return y


def conv2d_bwd(x, w, dy, stride, ph, pw, groups=1):
    """Exact adjoints of conv2d_fwd: returns (dx, dw)."""
    N, H, W, Cin = x.shape
    Cout, kh, kw, Cg = w.shape
    _, Ho, Wo, _ = dy.shape
    xp = _pad(x, ph, pw)
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    Og = Cout // groups
    for i in range(kh):
        for j in range(kw):
            sl = (slice(None), slice(i, i + (Ho - 1) * stride + 1, stride),
                  slice(j, j + (Wo - 1) * stride + 1, stride), slice(None))
            patch = xp[sl]
            if groups == 1:
                dw[:, i, j, :] = dy.reshape(-1, Cout).T @ patch.reshape(-1, Cin)
                dxp[sl] += dy @ w[:, i, j, :]
            elif Cg == 1 and Og == 1:
                dw[:, i, j, 0] = (dy * patch).sum(axis=(0, 1, 2))
                dxp[sl] += dy * w[:, i, j, 0]
            else:
                for g in range(groups):
                    dyg = dy[..., g * Og:(g + 1) * Og]
                    pg = patch[..., g * Cg:(g + 1) * Cg]
                    dw[g * Og:(g + 1) * Og, i, j, :] = dyg.reshape(-1, Og).T @ pg.reshape(-1, Cg)
                    dxp[sl[0], sl[1], sl[2], g * Cg:(g + 1) * Cg] += dyg @ w[g * Og:(g + 1) * Og, i, j, :]
    dx = dxp[:, ph:ph + H, pw:pw + W, :]
    return np.ascontiguousarray(dx), dw


BN_EPS = 1e-5
BN_MOMENTUM = 0.1


def bn_fwd(z, gamma, beta, eps=BN_EPS):
    """Training-mode batch norm over all axes but the last.
    Returns y, mean, invstd, biased variance."""
    ax = tuple(range(z.ndim - 1))
    mean = z.mean(axis=ax)
    var = ((z - mean) ** 2).mean(axis=ax)
    invstd = 1.0 / np.sqrt(var + eps)
    y = (z - mean) * invstd * gamma + beta
    return y, mean, invstd, var


def bn_running_update(rm, rv, mean, var, count, momentum=BN_MOMENTUM):
    """Exponential running statistics; the variance fed in is the unbiased one."""
    unbiased = var * (count / (count - 1.0)) if count > 1 else var
    return (1 - momentum) * rm + momentum * mean, (1 - momentum) * rv + momentum * unbiased


def bn_bwd(dy, z, mean, invstd, gamma):
    """dx = gamma*invstd*(dy - dbeta/M - xhat*dgamma/M); returns dx, dgamma, dbeta."""
    ax = tuple(range(z.ndim - 1))
    M = z.size // z.shape[-1]
    xhat = (z - mean) * invstd
    dbeta = dy.sum(axis=ax)
    dgamma = (dy * xhat).sum(axis=ax)
    dx = gamma * invstd * (dy - dbeta / M - xhat * dgamma / M)
    return dx, dgamma, dbeta


ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2


def act_fwd(y, act):
    if act == ACT_NONE:
        return y
    if act == ACT_RELU:
        return np.maximum(y, 0)
    return np.minimum(np.maximum(y, 0), 6)


def act_bwd(da, y, act):
    """Derivative is 1 strictly inside the linear region, 0 at and beyond the kinks."""
    if act == ACT_NONE:
        return da
    if act == ACT_RELU:
        return da * (y > 0)
    return da * ((y > 0) & (y < 6))


def gap_fwd(x):
    return x.mean(axis=(1, 2))


def gap_bwd(dy, H, W):
    N, C = dy.shape
    return np.broadcast_to((dy / (H * W))[:, None, None, :], (N, H, W, C)).copy()


def fc_fwd(x, w, b):
    return x @ w.T + b


def fc_bwd(x, w, dy):
    return dy @ w, dy.T @ x, dy.sum(axis=0)


def softmax_ce(logits, labels):
    """Mean cross-entropy over the batch and its gradient w.r.t. the logits."""
    B = logits.shape[0]
    s = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(s)
    p = e / e.sum(axis=1, keepdims=True)
    logp = s - np.log(e.sum(axis=1, keepdims=True))
    loss = -logp[np.arange(B), labels].mean()
    d = p.copy()
    d[np.arange(B), labels] -= 1.0
    return loss, d / B


def sgd_momentum(w, g, v, lr, momentum, weight_decay):
    """g <- g + wd*w ; v <- mu*v + g ; w <- w - lr*v  (v starts at 0, no dampening, no Nesterov)."""
    g = g + weight_decay * w
    v = momentum * v + g
    return w - lr * v, v
