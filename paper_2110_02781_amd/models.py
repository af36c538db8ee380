"""Unit lists (ftp_unit_desc dictionaries) of the two networks, and the layout of
a unit's parameter vector for initialisation.

MobileNetV2 follows the public block table of that architecture (the paper only
names the network, section "Experiment Setup"): 3x3 stem, groups
(t, c, n, s) = (1,16,1,1) (6,24,2,2) (6,32,3,2) (6,64,4,2) (6,96,3,1) (6,160,3,2)
(6,320,1,1), 1x1 head, global average pool, FC, loss; channel counts scaled by
the width multiplier and rounded to multiples of 8."""
import numpy as np

from . import binding as B


def _round8(v):
    r = max(8, (int(v + 4) // 8) * 8)
    return r + 8 if r < 0.9 * v else r


_MBV2_GROUPS = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1))


def mobilenet_v2_units(width=1.0, classes=10, stem_stride=1):
    c = _round8(32 * width)
    units = [dict(kind=B.UNIT_CONV, cin=3, cout=c, kh=3, kw=3, stride=stem_stride, pad_h=1, pad_w=1, act=B.ACT_RELU6)]
    for t, ch, n, s in _MBV2_GROUPS:
        co = _round8(ch * width)
        for i in range(n):
            units.append(dict(kind=B.UNIT_INVRES, cin=c, cout=co, stride=s if i == 0 else 1, expand=t))
            c = co
    head = _round8(1280 * max(1.0, width))
    units.append(dict(kind=B.UNIT_CONV, cin=c, cout=head, kh=1, kw=1, stride=1, act=B.ACT_RELU6))
    units.append(dict(kind=B.UNIT_GAP, cin=head, cout=head))
    units.append(dict(kind=B.UNIT_FC, cin=head, cout=classes))
    units.append(dict(kind=B.UNIT_LOSS, cin=classes, cout=classes))
    return units


def cnn1d_units(cin=9, channels=(32, 64, 64), classes=6, k=5):
    """conv1d(k, same padding)+BN+ReLU x3, GAP, FC, loss; a window is [N, 1, T, C]."""
    units, c = [], cin
    for co in channels:
        units.append(dict(kind=B.UNIT_CONV, cin=c, cout=co, kh=1, kw=k, stride=1, pad_h=0, pad_w=k // 2, act=B.ACT_RELU))
        c = co
    units += [dict(kind=B.UNIT_GAP, cin=c, cout=c), dict(kind=B.UNIT_FC, cin=c, cout=classes),
              dict(kind=B.UNIT_LOSS, cin=classes, cout=classes)]
    return units


def unit_param_layout(u):
    """[(name, count, fan_in)] in the order of the unit's parameter vector
    (fan_in 0: BatchNorm gamma (init 1), -1: beta / bias (init 0))."""
    k = u["kind"]
    if k == B.UNIT_CONV:
        fan = u["kh"] * u["kw"] * u["cin"]
        return [("w", u["cout"] * fan, fan), ("gamma", u["cout"], 0), ("beta", u["cout"], -1)]
    if k == B.UNIT_INVRES:
        ce = u["cin"] * u["expand"]
        out = []
        if u["expand"] != 1:
            out += [("w1", ce * u["cin"], u["cin"]), ("gamma1", ce, 0), ("beta1", ce, -1)]
        out += [("wd", ce * 9, 9), ("gamma2", ce, 0), ("beta2", ce, -1),
                ("w3", u["cout"] * ce, ce), ("gamma3", u["cout"], 0), ("beta3", u["cout"], -1)]
        return out
    if k == B.UNIT_FC:
        return [("w", u["cout"] * u["cin"], u["cin"]), ("b", u["cout"], -1)]
    return []


def init_unit_params(units, seed):
    """He-normal weights (std sqrt(2/fan_in)), gamma 1, beta/bias 0: one flat
    float32 vector per unit, drawn from the shared seeded generator."""
    import synth
    out = []
    for ui, u in enumerate(units):
        parts = []
        for name, n, fan in unit_param_layout(u):
            if fan > 0:
                parts.append(synth.normal(seed, f"w:{ui}:{name}", (n,), std=float(np.sqrt(2.0 / fan))))
            elif fan == 0:
                parts.append(np.ones(n))
            else:
                parts.append(np.zeros(n))
        out.append(np.concatenate(parts).astype(np.float32) if parts else np.zeros(0, np.float32))
    return out
