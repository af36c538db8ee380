"""Partition-unit lists of the two networks the oracle trains (test infrastructure).

The paper trains MobileNetV2 (section "Experiment Setup") without describing
its layers, and motivates sensor-window workloads; the unit lists below follow
the public MobileNetV2 block table and a three-convolution 1-D CNN.  A
partition unit is what the paper's profiling and partition sections call a
"layer": the smallest piece a stage boundary may fall between, so a residual
connection is never cut.
"""
from dataclasses import dataclass
import numpy as np
from . import layers as L
import synth


@dataclass(frozen=True)
class Unit:
    kind: str                 # 'conv' | 'invres' | 'gap' | 'fc' | 'loss'
    cin: int = 0
    cout: int = 0
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad_h: int = 0
    pad_w: int = 0
    expand: int = 1
    act: int = L.ACT_NONE


def make_divisible(v, divisor=8):
    """Round to the nearest multiple of 8, never dropping below 90 % of v."""
    new_v = max(divisor, int(v + divisor / 2) // divisor * divisor)
    if new_v < 0.9 * v:
        new_v += divisor
    return new_v


def mobilenet_v2(width=1.0, classes=10, stem_stride=1):
    """stem, 17 inverted-residual blocks, head 1x1 conv, GAP, FC, loss = 22 units."""
    groups = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
              (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
    c = make_divisible(32 * width)
    units = [Unit('conv', 3, c, 3, 3, stem_stride, 1, 1, act=L.ACT_RELU6)]
    for t, ch, n, s in groups:
        co = make_divisible(ch * width)
        for i in range(n):
            units.append(Unit('invres', c, co, 3, 3, s if i == 0 else 1, 1, 1, expand=t, act=L.ACT_RELU6))
            c = co
    head = make_divisible(1280 * max(1.0, width))
    units.append(Unit('conv', c, head, 1, 1, 1, 0, 0, act=L.ACT_RELU6))
    units.append(Unit('gap', head, head))
    units.append(Unit('fc', head, classes))
    units.append(Unit('loss', classes, classes))
    return units


def cnn1d(cin=9, channels=(32, 64, 64), classes=6, k=5):
    """Three conv1d(k=5, same padding)+BN+ReLU units, GAP, FC, loss = 6 units.
    A window of T steps is the tensor [N, 1, T, C]."""
    units, c = [], cin
    for co in channels:
        units.append(Unit('conv', c, co, 1, k, 1, 0, k // 2, act=L.ACT_RELU))
        c = co
    units += [Unit('gap', c, c), Unit('fc', c, classes), Unit('loss', classes, classes)]
    return units


def param_specs(u):
    """[(name, shape, kind, fan_in)] in the order the weights of a unit are laid
    out; kind is 'he' (normal, std sqrt(2/fan_in)), 'one' or 'zero'."""
    if u.kind == 'conv':
        return [('w', (u.cout, u.kh, u.kw, u.cin), 'he', u.kh * u.kw * u.cin),
                ('gamma', (u.cout,), 'one', 0), ('beta', (u.cout,), 'zero', 0)]
    if u.kind == 'invres':
        ce = u.cin * u.expand
        s = []
        if u.expand != 1:
            s += [('w1', (ce, 1, 1, u.cin), 'he', u.cin), ('gamma1', (ce,), 'one', 0), ('beta1', (ce,), 'zero', 0)]
        s += [('wd', (ce, 3, 3, 1), 'he', 9), ('gamma2', (ce,), 'one', 0), ('beta2', (ce,), 'zero', 0),
              ('w3', (u.cout, 1, 1, ce), 'he', ce), ('gamma3', (u.cout,), 'one', 0), ('beta3', (u.cout,), 'zero', 0)]
        return s
    if u.kind == 'fc':
        return [('w', (u.cout, u.cin), 'he', u.cin), ('b', (u.cout,), 'zero', 0)]
    return []


def bn_channels(u):
    """Channel count of each batch-norm in the unit, in order."""
    if u.kind == 'conv':
        return [u.cout]
    if u.kind == 'invres':
        ce = u.cin * u.expand
        return ([ce] if u.expand != 1 else []) + [ce, u.cout]
    return []


def init_params(units, seed, dtype=np.float64):
    """He-normal convolution / FC weights, gamma 1, beta 0, bias 0 — one list of
    arrays per unit, drawn from stream 'w:<unit>:<name>'."""
    out = []
    for ui, u in enumerate(units):
        ps = []
        for name, shape, kind, fan in param_specs(u):
            if kind == 'he':
                ps.append(synth.normal(seed, f"w:{ui}:{name}", shape, std=float(np.sqrt(2.0 / fan))).astype(dtype))
            elif kind == 'one':
                ps.append(np.ones(shape, dtype))
            else:
                ps.append(np.zeros(shape, dtype))
        out.append(ps)
    return out


def unit_out_shape(u, shape):
    """Output (H, W, C) of a unit for input (H, W, C); after GAP H=W=1."""
    H, W, C = shape
    if u.kind == 'conv':
        return (L.conv_out_size(H, u.kh, u.stride, u.pad_h), L.conv_out_size(W, u.kw, u.stride, u.pad_w), u.cout)
    if u.kind == 'invres':
        return (L.conv_out_size(H, 3, u.stride, 1), L.conv_out_size(W, 3, u.stride, 1), u.cout)
    if u.kind == 'gap':
        return (1, 1, C)
    if u.kind == 'fc':
        return (1, 1, u.cout)
    return (1, 1, C)
