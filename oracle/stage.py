"""One pipeline stage's training step on the CPU (test infrastructure).

A stage is the contiguous unit range [a, b) a worker builds from its partition
points (paper, section "Initialization"); it forwards a batch, later backwards
it with the weight version that forward used (weight stashing, section "Async
Pipeline Training"), and applies SGD with momentum and weight decay (section
"Experiment Setup").  Each in-flight batch occupies a slot holding whatever
its backward needs.
"""
import numpy as np
from . import layers as L
from . import models as M


def _identity(a):
    return a


def bf16_round(a):
    """Round to the nearest bfloat16 (ties to even) and return in the input's dtype."""
    a = np.asarray(a)
    u = a.astype(np.float32).view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(a.dtype).reshape(a.shape)


def _conv_bn_act_fwd(x, w, gamma, beta, stride, ph, pw, groups, act, q=_identity):
    z = q(L.conv2d_fwd(x, q(w), stride, ph, pw, groups))
    y, mean, invstd, var = L.bn_fwd(z, gamma, beta)
    a = q(L.act_fwd(y, act))
    return a, dict(x=x, z=z, y=y, mean=mean, invstd=invstd, var=var, gamma=gamma, beta=beta)


def _conv_bn_act_bwd(da, c, w, gamma, stride, ph, pw, groups, act, q=_identity, tie=None):
    """Returns the UNROUNDED input gradient (the caller rounds it once, after a
    possible residual add) and the weight / gamma / beta gradients.

    tie = (on, guard, report) resolves ReLU / ReLU6 on-off decisions that are ties
    at the precision of the implementation under test: where the pre-activation
    y lies within guard * (|gamma| * sqrt(1 + mean^2/var) + |beta|) of a kink
    (a relative error `guard` of the channel's typical |z|, carried through
    y = gamma*(z-mean)/std + beta), on and off are both correct, and the caller's
    boolean array `on` decides.  Everywhere
    else the oracle's own decision stands; report counts the elements where `on`
    disagrees with it outside the tie band (a real error of the caller)."""
    if tie is not None and act != L.ACT_NONE:
        on, guard, report = tie
        y = c['y']
        sc = gamma * c['invstd']
        band = guard * (np.abs(sc) * np.sqrt(c['var'] + c['mean'] ** 2) + np.abs(c['beta']))
        amb = np.abs(y) <= band
        own = y > 0
        if act == L.ACT_RELU6:
            amb |= np.abs(y - 6) <= band
            own &= y < 6
        on = np.asarray(on, dtype=bool).reshape(y.shape)
        report['elements'] = report.get('elements', 0) + int(y.size)
        report['ties'] += int(amb.sum())
        report['adopted'] += int((amb & (on != own)).sum())
        report['disagree'] += int((~amb & (on != own)).sum())
        dy = da * np.where(amb, on, own)
    else:
        dy = L.act_bwd(da, c['y'], act)
    dz, dgamma, dbeta = L.bn_bwd(dy, c['z'], c['mean'], c['invstd'], gamma)
    dx, dw = L.conv2d_bwd(c['x'], q(w), q(dz), stride, ph, pw, groups)
    return dx, dw, dgamma, dbeta


class Stage:
    def __init__(self, units, in_shape, a, b, n_slots=1, dtype=np.float64, storage=None, recompute=False):
        """units: full unit list; in_shape: (H, W, C) of the model input.
        recompute=True: a slot keeps only the stage input of its batch (and the weight
        version); the backward first runs the forward again to get the intermediates
        back (section "Synchronous Pipeline Parallelism Training": intermediates are
        thrown away and re-computed when the gradient arrives).  The second forward
        is not a training forward: the BatchNorm running statistics do not move.
        storage='bf16' models mixed-precision training: every tensor that such a
        run keeps in bfloat16 (convolution / FC outputs, block outputs, pooled
        features, BatchNorm+activation outputs, activation gradients, and the
        working copy of convolution / FC weights) is rounded to bfloat16 at the point where it is stored, while
        statistics, gamma/beta, weight gradients, momentum and master weights stay
        exact.  The ReLU / ReLU6 on-off decisions are thereby taken on the same
        rounded values a bfloat16 implementation sees."""
        assert 0 <= a < b <= len(units)
        assert storage in (None, 'bf16')
        self.q = bf16_round if storage == 'bf16' else _identity
        self.units, self.a, self.b, self.dtype = units, a, b, dtype
        shape = tuple(in_shape)
        self.shapes = [shape]
        for u in units:
            shape = M.unit_out_shape(u, shape)
            self.shapes.append(shape)
        self.params = {i: [] for i in range(a, b)}
        self.grads, self.mom, self.bn_run = {}, {}, {}
        for i in range(a, b):
            specs = M.param_specs(units[i])
            self.params[i] = [np.zeros(s, dtype) for _, s, _, _ in specs]
            self.grads[i] = [np.zeros(s, dtype) for _, s, _, _ in specs]
            self.mom[i] = [np.zeros(s, dtype) for _, s, _, _ in specs]
            self.bn_run[i] = [[np.zeros(c, dtype), np.ones(c, dtype)] for c in M.bn_channels(units[i])]
        self.slots = [None] * n_slots
        self.recompute = recompute
        self._tracking = True

    def set_params(self, i, arrays):
        self.params[i] = [np.array(p, dtype=self.dtype) for p in arrays]

    # ---------------------------------------------------------------- forward
    def _bn_track(self, i, k, c):
        if not self._tracking:
            return
        cnt = c['z'].size // c['z'].shape[-1]
        rm, rv = self.bn_run[i][k]
        self.bn_run[i][k] = list(L.bn_running_update(rm, rv, c['mean'], c['var'], cnt))

    def _unit_fwd(self, i, x, P):
        u = self.units[i]
        q = self.q
        if u.kind == 'conv':
            a, c = _conv_bn_act_fwd(x, P[0], P[1], P[2], u.stride, u.pad_h, u.pad_w, 1, u.act, q)
            self._bn_track(i, 0, c)
            return a, [c]
        if u.kind == 'invres':
            caches, h, k, nb = [], x, 0, 0
            ce = u.cin * u.expand
            if u.expand != 1:
                h, c = _conv_bn_act_fwd(h, P[0], P[1], P[2], 1, 0, 0, 1, L.ACT_RELU6, q)
                self._bn_track(i, nb, c); nb += 1
                caches.append(c); k = 3
            h, c = _conv_bn_act_fwd(h, P[k], P[k + 1], P[k + 2], u.stride, 1, 1, ce, L.ACT_RELU6, q)
            self._bn_track(i, nb, c); nb += 1
            caches.append(c)
            h, c = _conv_bn_act_fwd(h, P[k + 3], P[k + 4], P[k + 5], 1, 0, 0, 1, L.ACT_NONE, q)
            self._bn_track(i, nb, c)
            caches.append(c)
            if u.stride == 1 and u.cin == u.cout:
                h = x + h
            return q(h), caches
        if u.kind == 'gap':
            return q(L.gap_fwd(x))[:, None, None, :], [dict(hw=x.shape[1:3])]
        if u.kind == 'fc':
            x2 = x.reshape(x.shape[0], -1)
            return q(L.fc_fwd(x2, q(P[0]), P[1]))[:, None, None, :], [dict(x=x2)]
        return x, [dict()]                                   # loss unit: logits pass through

    def forward(self, slot, x, stash_weights=True):
        assert self.slots[slot] is None, "slot busy"
        x = np.asarray(x, dtype=self.dtype)
        # update() replaces parameter arrays instead of writing into them, so
        # keeping the lists is a snapshot of this weight version
        P = {i: list(self.params[i]) for i in range(self.a, self.b)}
        caches, h, unit_in = {}, x, {}
        for i in range(self.a, self.b):
            unit_in[i] = h
            h, caches[i] = self._unit_fwd(i, h, P[i])
        h = self.q(h)                                        # the stage output is a stored tensor
        self.slots[slot] = dict(caches=caches, params=P if stash_weights else None, out=h, dlogits=None,
                                unit_in=unit_in)
        if self.recompute:
            self.slots[slot].update(caches=None, unit_in=None, x=x)
        return h

    def materialize(self, slot):
        """Run the second forward of a recomputing slot now (backward does it on demand)."""
        s = self.slots[slot]
        if s['caches'] is None:
            self._recompute(s, s['params'] if s['params'] is not None else self.params)

    def _recompute(self, s, P):
        """The intermediates of a slot that kept only its input, from the weights P."""
        self._tracking = False
        try:
            caches, h, unit_in = {}, s['x'], {}
            for i in range(self.a, self.b):
                unit_in[i] = h
                h, caches[i] = self._unit_fwd(i, h, P[i])
        finally:
            self._tracking = True
        s['caches'], s['unit_in'] = caches, unit_in

    def loss(self, slot, labels):
        assert self.units[self.b - 1].kind == 'loss'
        s = self.slots[slot]
        logits = s['out'].reshape(s['out'].shape[0], -1)
        loss, d = L.softmax_ce(logits, np.asarray(labels))
        s['dlogits'] = self.q(d)[:, None, None, :]
        return loss

    # --------------------------------------------------------------- backward
    def _acc(self, i, k, g):
        self.grads[i][k] = self.grads[i][k] + g

    def _unit_bwd(self, i, d, caches, P, ties=None):
        u = self.units[i]
        q = self.q

        def tie(k):          # tie-break data of convolution k of this unit, if the caller gave any
            if ties is None or (i, k) not in ties['on']:
                return None
            g = ties['guard']
            return (ties['on'][(i, k)], g[(i, k)] if isinstance(g, dict) else g, ties['report'])
        if u.kind == 'conv':
            dx, dw, dg, db = _conv_bn_act_bwd(d, caches[0], P[0], P[1], u.stride, u.pad_h, u.pad_w, 1, u.act, q, tie(0))
            self._acc(i, 0, dw); self._acc(i, 1, dg); self._acc(i, 2, db)
            return q(dx)
        if u.kind == 'invres':
            ce = u.cin * u.expand
            k = 3 if u.expand != 1 else 0
            dout = d
            d, dw, dg, db = _conv_bn_act_bwd(d, caches[-1], P[k + 3], P[k + 4], 1, 0, 0, 1, L.ACT_NONE, q, None)
            self._acc(i, k + 3, dw); self._acc(i, k + 4, dg); self._acc(i, k + 5, db)
            d, dw, dg, db = _conv_bn_act_bwd(q(d), caches[-2], P[k], P[k + 1], u.stride, 1, 1, ce, L.ACT_RELU6, q,
                                             tie(len(caches) - 2))
            self._acc(i, k, dw); self._acc(i, k + 1, dg); self._acc(i, k + 2, db)
            if u.expand != 1:
                d, dw, dg, db = _conv_bn_act_bwd(q(d), caches[0], P[0], P[1], 1, 0, 0, 1, L.ACT_RELU6, q, tie(0))
                self._acc(i, 0, dw); self._acc(i, 1, dg); self._acc(i, 2, db)
            if u.stride == 1 and u.cin == u.cout:
                d = d + dout
            return q(d)
        if u.kind == 'gap':
            H, W = caches[0]['hw']
            return q(L.gap_bwd(d.reshape(d.shape[0], -1), H, W))
        if u.kind == 'fc':
            dx, dw, db = L.fc_bwd(caches[0]['x'], q(P[0]), d.reshape(d.shape[0], -1))
            self._acc(i, 0, dw); self._acc(i, 1, db)
            return q(dx)[:, None, None, :]
        return d

    def backward(self, slot, dy=None, tie_breaks=None, guard=0.0):
        """tie_breaks: {(unit, conv): boolean array} of activation on-off decisions
        to adopt inside the tie band (see _conv_bn_act_bwd; guard: one width for all
        layers or {(unit, conv): width}); the counts of ties,
        adopted decisions and out-of-band disagreements land in self.tie_report."""
        s = self.slots[slot]
        assert s is not None, "slot empty"
        d = s['dlogits'] if dy is None else np.asarray(dy, dtype=self.dtype)
        assert d is not None
        P = s['params'] if s['params'] is not None else self.params
        if s['caches'] is None:
            self._recompute(s, P)
        self.tie_report = dict(ties=0, adopted=0, disagree=0)
        ties = None if tie_breaks is None else dict(on=tie_breaks, guard=guard, report=self.tie_report)
        self.unit_in, self.unit_dout = s['unit_in'], {}     # kept for unit-by-unit checks
        for i in range(self.b - 1, self.a - 1, -1):
            self.unit_dout[i] = d
            d = self._unit_bwd(i, d, s['caches'][i], P[i], ties)
        self.slots[slot] = None
        return d

    # ----------------------------------------------------------------- update
    def adopt_units(self, other, lo, hi):
        """Weight redistribution, receiving side: take weights, momentum and BatchNorm
        running statistics of units [lo, hi) from another stage (section "Dynamic Model
        Partition": a worker fetches the layers it is missing from their current owner)."""
        for i in range(lo, hi):
            self.params[i] = [p.copy() for p in other.params[i]]
            self.mom[i] = [m.copy() for m in other.mom[i]]
            if i in other.bn_run:
                self.bn_run[i] = [[a.copy() for a in pair] for pair in other.bn_run[i]]

    def aggregate(self, slots):
        """Weight aggregation (section "Async Pipeline Training"): the live
        weights become the arithmetic mean of the weight versions stashed in
        `slots`; momentum and gradients stay as they are."""
        snaps = [self.slots[s]['params'] for s in slots]
        assert all(sn is not None for sn in snaps)
        for i in range(self.a, self.b):
            for k in range(len(self.params[i])):
                acc = np.zeros(self.params[i][k].shape, dtype=np.float64)
                for sn in snaps:
                    acc = acc + sn[i][k].astype(np.float64)
                self.params[i][k] = (acc / len(snaps)).astype(self.params[i][k].dtype)

    def update(self, lr, momentum, weight_decay):
        for i in range(self.a, self.b):
            for k in range(len(self.params[i])):
                w, v = L.sgd_momentum(self.params[i][k], self.grads[i][k], self.mom[i][k], lr, momentum, weight_decay)
                self.params[i][k], self.mom[i][k] = w, v
                self.grads[i][k] = np.zeros_like(w)


def version_trace(stage_index, n_stages, n_batches, aggregate=False):
    """Weight versions along the one-forward-one-backward order of one stage
    (section "Async Pipeline Training"): every backward produces the next
    version, a forward uses the newest one, a backward uses the version its
    forward used (weight stashing).  With aggregate=True the stage also
    aggregates: stage i of n has n-i versions in use at once, and after every
    n-i backwards, right behind the forward that picks up the newest of them,
    those n-i versions are merged into one new version.
    Returns [('F'|'B', batch, version_used) | ('A', (versions...), new_version)]."""
    depth = n_stages - stage_index
    out, fwd_version, version, n_bwd, pending = [], {}, 0, 0, False
    for op, b in one_f_one_b_order(stage_index, n_stages, n_batches):
        if op == 'F':
            fwd_version[b] = version
            out.append(('F', b, version))
            if aggregate and pending:
                live = sorted(fwd_version[x] for x in fwd_version if x > b - depth)   # versions of the batches in flight
                version += 1
                out.append(('A', tuple(live), version))
                pending = False
        else:
            out.append(('B', b, fwd_version[b]))
            version += 1
            n_bwd += 1
            if n_bwd % depth == 0:
                pending = True
    return out


def one_f_one_b_order(stage_index, n_stages, n_batches):
    """Call order of one stage under the one-forward-one-backward rule: stage i
    of n keeps n-i batches in flight (section "Async Pipeline Training"), so it
    forwards n-i batches, then alternates backward/forward, then drains.
    Returns [('F', b) | ('B', b)]."""
    depth = min(n_stages - stage_index, n_batches)
    order = [('F', b) for b in range(depth)]
    nf, nb = depth, 0
    while nb < n_batches:
        order.append(('B', nb)); nb += 1
        if nf < n_batches:
            order.append(('F', nf)); nf += 1
    return order
