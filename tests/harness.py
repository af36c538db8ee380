"""Shared helpers of the GPU parity tests: build the same stage in the oracle and
in the HIP library from the seeded generators, run both, compare tensors."""
import numpy as np

import synth
from oracle import models as OM
from oracle.stage import Stage as OracleStage

TOL = {"f32": 1e-4, "bf16": 2e-2}
# Teacher-forced bfloat16 units against the oracle that never rounds: 3e-2.  Measured: every tensor within 1e-2 except
# one BatchNorm shift gradient of the 112x112 block at batch 4 (2.01e-2), a sum that nearly cancels.  The 2e-2 bar is
# held against the oracle that takes its activation decisions on bfloat16-stored values, as the kernels do.
TOL_BF16_VS_EXACT = 3e-2
# Activation on/off decisions next to a kink (Pair(ties="bounded") only; the default
# is ties="off": the oracle decides alone and nothing of the library enters it).
# GUARD: width of the band around a ReLU / ReLU6 kink inside which on and off are both
# correct, as a multiple of the magnitude of the two summands of y = scale*z + shift.
# float: 3e-5, or five times the error measured on that layer's conv output if that is more
# (about 1e-5 of the largest |z| on a first step, up to 6e-5 after several updates; the band is
# relative to the channel's r.m.s., a fifth of its maximum; the error itself is held to TOL in
# kernel_decisions); bfloat16: 2e-2, the tolerance, i.e. five storage roundings of 2^-8.  ADOPT_CAP: the most decisions, as a fraction of all of them, that
# may be taken over from the library inside the band (plus 4 for tiny tensors).
GUARD = {"f32": 3e-5, "bf16": 2e-2}
ADOPT_CAP = {"f32": 1e-5, "bf16": 2e-4}
# Against the oracle that never rounds, a bfloat16 implementation decides on values that carry their storage
# rounding (2^-9 relative on average): decisions within that distance of a kink differ for about one element in a
# thousand, all of them inside the band.
ADOPT_CAP_EXACT = 3e-3


# What one training step on the stage's OWN activations (nothing teacher-forced, no activation decision taken over)
# is held to, per class of tensor, as max(max-abs error / max-abs reference, relative L2 error).  float: 1e-4
# everywhere (the tests use TOL).  bfloat16: every stored tensor carries a rounding of 2^-9 relative that the next
# layer amplifies or damps, and an activation that two correct implementations switch differently changes a
# gradient element by its whole value, so a chained run has no a-priori 2e-2 bound (that bar is held unit by unit,
# teacher-forced).  The bars below are 1.5 times the errors measured on the MI355X for each workload, against the
# oracle that rounds stored tensors where the library does ("rounding") and against the one that never rounds
# ("exact"); a regression in any kernel moves them by far more.
CHAINED_BAR = {
    # 9x11 input, batch 5, 9 units: the library reproduces the rounding oracle's forward exactly
    "small_net": {"rounding": dict(y=1e-3, loss=1e-4, dx=1e-2, grads=1e-2, weights=1e-4, bn=1e-4),
                  "exact": dict(y=1.2e-2, loss=1e-3, dx=0.8, grads=0.8, weights=4e-3, bn=4e-3)},
    # MobileNetV2 w1.0 224x224 batch 64, stage 1 of the 4-way split on the seeded costs (units 15-18)
    "config4": {"rounding": dict(y=1.3e-2, dx=0.15, grads=0.2, weights=4e-2, bn=3e-4),
                "exact": dict(y=1.8e-2, dx=0.26, grads=0.32, weights=7.5e-2, bn=1.6e-3)},
    # MobileNetV2 w1.4 224x224 batch 4, all 22 units: the gradients of the first layers have passed ~50 bfloat16
    # layers backwards on BatchNorm statistics of as few as 196 values and carry no common digits any more (the two
    # oracles are as far from each other), which the update (lr 0.01) shrinks to 2-3 % of the weights
    "config5": {"rounding": dict(y=7e-2, loss=2e-3, grads=2.1, weights=4e-2, bn=4e-2),
                "exact": dict(y=0.125, loss=1e-2, grads=2.2, weights=5.5e-2, bn=7.5e-2)},
}


def assert_chained(report, workload):
    """The bars of CHAINED_BAR, and for the backward classes the yardstick: the library may be no further from the
    rounding oracle than 1.5 times what separates the two oracles from each other (plus 1e-2)."""
    for oracle_name in ("rounding", "exact"):
        for cls, (e_max, e_l2) in report[oracle_name].items():
            bar = CHAINED_BAR[workload][oracle_name][cls]
            assert max(e_max, e_l2) <= bar, f"{workload} vs {oracle_name} oracle: {cls} error {e_max:.3e} / {e_l2:.3e} above {bar}"
    for cls in ("dx", "grads"):
        if cls in report["rounding"]:
            got, yard = max(report["rounding"][cls]), max(report["oracles"][cls])
            assert got <= 1.5 * yard + 1e-2, f"{workload}: {cls} is {got:.3e} from the rounding oracle, the oracles are {yard:.3e} apart"


def unit_shapes(o_units, in_shape):
    """Input shape (H, W, C) of every unit, and the output shape of the last, from the oracle's model description."""
    shapes = [tuple(in_shape)]
    for u in o_units:
        shapes.append(tuple(OM.unit_out_shape(u, shapes[-1])))
    return shapes


def rel_err(a, b):
    """(max-abs error / max-abs reference, relative L2 error)."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    assert a.shape == b.shape, (a.shape, b.shape)
    if a.size == 0:
        return 0.0, 0.0
    d = a - b
    ref_max = max(np.abs(b).max(), 1e-30)
    ref_l2 = max(np.sqrt((b * b).sum()), 1e-30)
    return np.abs(d).max() / ref_max, np.sqrt((d * d).sum()) / ref_l2


def assert_close(a, b, tol, what, floor=0.0, scale_ref=None):
    """Both the max-abs and the L2 relative error must be within tol.  `floor`:
    tensors whose reference is numerically zero (below floor) are compared absolutely.
    `scale_ref`: a tensor of the same natural magnitude as the terms summed into b;
    used as the denominator when it is larger than b itself (sums that cancel)."""
    assert np.all(np.isfinite(np.asarray(a, dtype=np.float64))), f"{what}: non-finite values"
    if np.abs(np.asarray(b)).max() <= floor and scale_ref is None:
        assert np.abs(np.asarray(a)).max() <= max(floor, 1e-30) * 10, f"{what}: expected ~0"
        return 0.0, 0.0
    e_max, e_l2 = rel_err(a, b)
    if scale_ref is not None:
        d = np.asarray(a, dtype=np.float64).ravel() - np.asarray(b, dtype=np.float64).ravel()
        sr = np.asarray(scale_ref, dtype=np.float64).ravel()
        e_max = min(e_max, np.abs(d).max() / max(np.abs(sr).max(), 1e-30))
        e_l2 = min(e_l2, np.sqrt((d * d).sum()) / max(np.sqrt((sr * sr).sum()), 1e-30))
    assert e_max <= tol and e_l2 <= tol, f"{what}: max-rel {e_max:.3e}, l2-rel {e_l2:.3e} > {tol}"
    return e_max, e_l2


def flat_params(plist):
    return np.concatenate([np.asarray(p, dtype=np.float64).ravel() for p in plist]) if plist else np.zeros(0)


def to_bf16_bits(a):
    """float -> bfloat16 bit patterns (round to nearest even) as uint16."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def from_bf16_bits(b):
    return (b.astype(np.uint32) << 16).view(np.float32)


class Pair:
    """The same stage [a,b) in the oracle (float64) and in the HIP library."""

    def __init__(self, o_units, h_units, in_shape, batch, a, b, dtype="f32", n_slots=1, seed=1, guard=None, ties="off",
                 model_of=None, recompute=False, storage="match", z_tol=None, tile=1, adopt_cap=None):
        """ties: "off" = the oracle takes every activation decision itself; "bounded" = decisions inside the
        band of width `guard` around a kink follow the library, after its conv outputs and BatchNorm scale / shift
        have been checked against the oracle's at z_tol (default: the tolerance of the type), at most ADOPT_CAP
        of them, and none outside the band.  storage: "match" = the oracle rounds stored tensors to bfloat16
        when the library does; "exact" = the oracle never rounds (float64 throughout).
        tile > 1: the library runs `batch` samples that are `tile` copies of the oracle's batch // tile.  Batch
        statistics of a batch of identical copies are those of one copy, so with the output gradient divided by
        `tile` every forward tensor and (times `tile`) every data gradient of the large batch is the tiled small
        one and the weight gradients are equal: the oracle stays affordable while every row of the full-size
        tensors is compared."""
        import torch
        import paper_2110_02781_amd as P
        self.P, self.torch = P, torch
        self.dtype, self.batch, self.a, self.b = dtype, batch, a, b
        self.o_units, self.h_units = o_units, h_units
        self.dev = torch.device("cuda:0")
        self.tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        H, W, Cc = in_shape
        # stages that exchange units (re-partition) are built from one model object
        self.owns_model = model_of is None
        self.model = P.model_create(h_units, H, W, Cc, P.F32 if dtype == "f32" else P.BF16) if model_of is None else model_of.model
        self.stage = P.stage_create(self.model, a, b, batch, n_slots, P.STAGE_RECOMPUTE if recompute else 0)
        # A recomputing stage has no intermediates to show between forward and backward: a twin that keeps
        # everything runs the same calls; it supplies the activation decisions, and the two must agree bit for bit.
        self.twin = P.stage_create(self.model, a, b, batch, n_slots) if recompute else None
        assert ties in ("off", "bounded") and storage in ("match", "exact")
        assert batch % tile == 0
        self.tile = tile
        self.bn_count = {}
        self.oracle = OracleStage(o_units, in_shape, a, b, n_slots,
                                  storage='bf16' if dtype == 'bf16' and storage == "match" else None, recompute=recompute)
        op = OM.init_params(o_units, seed)
        hp = P.models.init_unit_params(h_units, seed)
        for i in range(a, b):
            flat = flat_params(op[i])
            assert np.array_equal(flat.astype(np.float32), hp[i]), "both sides must draw identical weights"
            # masters are fp32 on both sides; in bf16 mode each side rounds its own working copy
            self.oracle.set_params(i, [p.astype(np.float32).astype(np.float64) for p in op[i]])
            P.stage_import_weights(self.stage, i, hp[i])
            if self.twin:
                P.stage_import_weights(self.twin, i, hp[i])
        self.in_shape = self.oracle.shapes[a]
        self.out_shape = self.oracle.shapes[b]
        self.stream = torch.cuda.current_stream().cuda_stream
        self.tie_reports = []
        self.ties = ties
        self.guard = GUARD[dtype] if guard is None else guard
        self.z_tol = TOL[dtype] if z_tol is None else z_tol
        self.adopt_cap = ADOPT_CAP[dtype] if adopt_cap is None else adopt_cap
        self.z_err = 0.0                                          # worst conv-output error seen by kernel_decisions
        self.layer_guard = {}

    def close(self):
        self.P.stage_destroy(self.stage)
        if self.twin:
            self.P.stage_destroy(self.twin)
        if self.owns_model:
            self.P.model_destroy(self.model)

    def copy_units_from(self, other, lo, hi):
        """Weights, momentum and BatchNorm running statistics of units [lo, hi) from another pair, on both sides."""
        self.P.stage_copy_units(self.stage, other.stage, lo, hi, self.stream)
        self.oracle.adopt_units(other.oracle, lo, hi)

    # -- tensors ------------------------------------------------------------------
    def dev_tensor(self, arr):
        t = self.torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(self.dev)
        return t.to(self.tdt).contiguous()

    def as_seen(self, arr):
        """The values the library receives after conversion to its storage type."""
        return self.dev_tensor(arr).float().cpu().numpy().astype(np.float64)

    def host(self, t):
        self.torch.cuda.synchronize()
        return t.float().cpu().numpy().astype(np.float64)

    def empty(self, shape):
        return self.torch.full(tuple(shape), float("nan"), dtype=self.tdt, device=self.dev)

    # -- steps ----------------------------------------------------------------------
    def forward(self, slot, x, snapshot=False):
        P = self.P
        xd = self.dev_tensor(self._tiled(x))
        y = self.empty((self.batch,) + tuple(self.out_shape))
        P.stage_forward(self.stage, slot, xd, y, self.stream)
        if snapshot:
            P.stage_snapshot_weights(self.stage, slot, self.stream)
        if self.twin:
            y2 = self.empty((self.batch,) + tuple(self.out_shape))
            P.stage_forward(self.twin, slot, xd, y2, self.stream)
            if snapshot:
                P.stage_snapshot_weights(self.twin, slot, self.stream)
            assert self.torch.equal(y, y2), "recomputing stage and its twin disagree on the forward output"
        yo = self.oracle.forward(slot, self.as_seen(x), stash_weights=snapshot)
        caches = self.oracle.slots[slot]['caches']
        if self.tile > 1 and caches is not None:
            for i, cs in caches.items():
                for k, c in enumerate(cs):
                    if 'z' in c:
                        self.bn_count[(i, k)] = c['z'].size // c['z'].shape[-1]
        return self.host(y), self._tiled(yo)

    def _tiled(self, arr):
        return arr if self.tile == 1 else np.tile(arr, (self.tile,) + (1,) * (np.ndim(arr) - 1))

    def aggregate(self, slots):
        self.P.stage_aggregate_weights(self.stage, slots, self.stream)
        self.oracle.aggregate(slots)

    def loss(self, slot, labels):
        P, torch = self.P, self.torch
        ld = torch.from_numpy(np.ascontiguousarray(self._tiled(np.asarray(labels, dtype=np.int32)))).to(self.dev)
        out = torch.zeros(1, dtype=torch.float32, device=self.dev)
        P.stage_loss(self.stage, slot, ld, out, self.stream)
        if self.twin:
            out2 = torch.zeros(1, dtype=torch.float32, device=self.dev)
            P.stage_loss(self.twin, slot, ld, out2, self.stream)
            assert torch.equal(out, out2)
        lo = self.oracle.loss(slot, labels)
        return float(self.host(out)[0]), lo

    def kernel_decisions(self, slot):
        """The on/off decision the library takes for every ReLU / ReLU6 element of the
        slot's batch: act'(fma(z, scale, shift)) evaluated in float32 on its own z and
        BatchNorm scale / shift.  Before they are used, z, scale and shift themselves must
        agree with the oracle's to z_tol: only then is a decision that differs a tie."""
        P = self.P
        out = {}
        src = self.twin if self.twin else self.stage
        if self.twin:
            self.oracle.materialize(slot)
        for i in range(self.a, self.b):
            u = self.o_units[i]
            if u.kind == 'conv':
                acts = [u.act]
            elif u.kind == 'invres':
                acts = ([2] if u.expand != 1 else []) + [2, 0]
            else:
                continue
            for k, act in enumerate(acts):
                if act == 0:
                    continue
                zo = self.oracle.slots[slot]['caches'][i][k]['z']
                C = zo.shape[-1]
                z = P.stage_export_conv_output(src, slot, i, k, zo.size * self.tile).reshape((self.batch,) + zo.shape[1:])
                st = P.stage_export_bn_batch_stats(src, slot, i, k, 4 * C)
                c = self.oracle.slots[slot]['caches'][i][k]
                n0 = zo.shape[0]
                for t in range(self.tile):       # copy by copy: no tiled float64 tensor of the full size
                    e = assert_close(z[t * n0:(t + 1) * n0], zo, self.z_tol,
                                     f"unit {i} conv {k}: conv output behind the activation decisions")
                    assert t == 0 or np.array_equal(z[t * n0:(t + 1) * n0], z[:n0]), f"unit {i} conv {k}: copies of one sample differ"
                self.z_err = max(self.z_err, e[0])
                self.layer_guard[(i, k)] = max(self.guard, 5.0 * e[0]) if self.dtype == "f32" else self.guard
                sc_o = c['gamma'] * c['invstd']
                sh_o = c['beta'] - c['mean'] * sc_o
                mag = np.abs(sc_o) * np.sqrt(c['var'] + c['mean'] ** 2) + np.abs(c['beta'])
                assert_close(st[2 * C:3 * C], sc_o, self.z_tol, f"unit {i} conv {k}: BatchNorm scale")
                assert_close(st[3 * C:], sh_o, self.z_tol, f"unit {i} conv {k}: BatchNorm shift", scale_ref=mag)
                z = z[:n0]
                y = (z.astype(np.float64) * st[2 * C:3 * C].astype(np.float64) + st[3 * C:].astype(np.float64)).astype(np.float32)
                on = y > 0
                if act == 2:
                    on &= y < 6
                out[(i, k)] = on
        return out

    def backward(self, slot, dy=None, want_dx=True):
        """Backward on both sides.  On-off decisions of the activations that are ties at
        the library's precision are resolved the way the library resolved them; any
        decision that differs outside the tie band fails the test."""
        P = self.P
        dyd = self.dev_tensor(self._tiled(dy) / self.tile) if dy is not None else None
        dx = self.empty((self.batch,) + tuple(self.in_shape)) if want_dx else None
        ties = self.kernel_decisions(slot) if self.ties == "bounded" else None
        P.stage_backward(self.stage, slot, dyd, dx, self.stream)
        if self.twin:
            dx2 = self.empty((self.batch,) + tuple(self.in_shape)) if want_dx else None
            P.stage_backward(self.twin, slot, dyd, dx2, self.stream)
            assert dx is None or self.torch.equal(dx, dx2), "recomputing stage and its twin disagree on dx"
        dxo = self.oracle.backward(slot, None if dy is None else self.as_seen(dy), tie_breaks=ties,
                                   guard=dict(self.layer_guard) if ties is not None else 0.0)
        rep = dict(self.oracle.tie_report, mode=self.ties, z_err=self.z_err)
        self.tie_reports.append(rep)
        if ties is not None:
            assert rep['disagree'] == 0, f"activation decisions differ outside the tie band: {rep}"
            cap = 4 + self.adopt_cap * rep.get('elements', 0)
            assert rep['adopted'] <= cap, f"too many activation decisions taken over from the library (cap {cap:.0f}): {rep}"
        return (self.host(dx) * self.tile if want_dx else None), (self._tiled(dxo) if want_dx else dxo)

    def update(self, lr, mu, wd):
        self.P.stage_update(self.stage, lr, mu, wd, self.stream)
        if self.twin:
            self.P.stage_update(self.twin, lr, mu, wd, self.stream)
        self.oracle.update(lr, mu, wd)

    # -- comparisons ------------------------------------------------------------------
    def export_unit_vectors(self, which):
        """The library's per-unit parameter / gradient / momentum vectors as a list of float32 arrays."""
        P = self.P
        self.torch.cuda.synchronize()
        fn = {"weights": P.stage_export_weights, "grads": P.stage_export_grads, "momentum": P.stage_export_momentum}[which]
        return [np.array(fn(self.stage, i, P.model_unit_param_count(self.model, i)), copy=True)
                for i in range(self.a, self.b) if P.model_unit_param_count(self.model, i)]

    def assert_twin_identical(self):
        """Weights, gradients, momentum and running statistics of the recomputing stage and of its twin, bit for bit."""
        P = self.P
        self.torch.cuda.synchronize()
        for i in range(self.a, self.b):
            n = P.model_unit_param_count(self.model, i)
            for fn in (P.stage_export_weights, P.stage_export_grads, P.stage_export_momentum):
                if n:
                    assert np.array_equal(fn(self.stage, i, n), fn(self.twin, i, n)), f"unit {i}: {fn.__name__} differ"
            nb = P.model_unit_bn_channels(self.model, i)
            if nb:
                assert np.array_equal(P.stage_export_bn_stats(self.stage, i, 2 * nb), P.stage_export_bn_stats(self.twin, i, 2 * nb)), \
                    f"unit {i}: running statistics differ"

    def _run_var_at_full_batch(self, i, k, rv):
        """tile > 1, after ONE forward from the initial running variance 1: the unbiased variance that enters the
        running statistic carries the factor M/(M-1) of the batch it was measured on; M is `tile` times larger
        in the library."""
        if self.tile == 1:
            return rv
        m = self.bn_count[(i, k)]
        return 0.9 + (rv - 0.9) * ((m - 1.0) / m) * (self.tile * m / (self.tile * m - 1.0))

    def oracle_busy_slots(self):
        return [i for i, sl in enumerate(self.oracle.slots) if sl is not None]

    def compare_unit_vectors(self, which, tol, floor=0.0):
        """which: 'weights' | 'grads' | 'momentum' | 'bn'.  Returns the worst (max, l2) errors."""
        P = self.P
        worst = (0.0, 0.0)
        self.torch.cuda.synchronize()
        for i in range(self.a, self.b):
            n = P.model_unit_param_count(self.model, i)
            if which == "bn":
                nb = P.model_unit_bn_channels(self.model, i)
                if nb == 0:
                    continue
                got = P.stage_export_bn_stats(self.stage, i, 2 * nb)
                ref = np.concatenate([np.concatenate([rm, self._run_var_at_full_batch(i, k, rv)])
                                      for k, (rm, rv) in enumerate(self.oracle.bn_run[i])])
                e = assert_close(got, ref, tol, f"unit {i} bn running stats")
                worst = (max(worst[0], e[0]), max(worst[1], e[1]))
                continue
            if n == 0:
                continue
            fn = {"weights": P.stage_export_weights, "grads": P.stage_export_grads,
                  "momentum": P.stage_export_momentum}[which]
            src = {"weights": self.oracle.params, "grads": self.oracle.grads, "momentum": self.oracle.mom}[which]
            got = fn(self.stage, i, n)
            # compare tensor by tensor so that a small tensor is not hidden by a large one
            # d(gamma) of a BatchNorm whose consumer is again normalised per channel (expand ->
            # depthwise -> BatchNorm) cancels to almost zero; it is a sum of the same dY terms as
            # d(beta) weighted by unit-variance x-hat, so it is judged on d(beta)'s scale.
            names = [nm for nm, _, _, _ in OM.param_specs(self.o_units[i])]
            off = 0
            for k, ref in enumerate(src[i]):
                m = ref.size
                # gamma and beta of one BatchNorm are judged on their joint scale: either gradient can
                # vanish by an invariance of the network (a per-channel shift or scale that the next
                # normalisation removes) while the other does not
                sref = None
                if names[k].startswith("gamma"):
                    sref = np.concatenate([src[i][k].ravel(), src[i][k + 1].ravel()])
                elif names[k].startswith("beta"):
                    sref = np.concatenate([src[i][k - 1].ravel(), src[i][k].ravel()])
                e = assert_close(got[off:off + m], ref.ravel(), tol, f"unit {i} {which}[{k}:{names[k]}]", floor, sref)
                worst = (max(worst[0], e[0]), max(worst[1], e[1]))
                off += m
        return worst


def unitwise_check(o_units, h_units, in_shape, batch, a, b, dtype, seed, x, dy=None, labels=None, report=None, storage="match",
                   tol=None):
    """Teacher-forced parity of every unit of stage [a,b) at its real shape: the oracle runs
    the whole stage once; then each unit alone is built in the library, fed the oracle's input
    of that unit and the oracle's gradient of that unit's output, and compared at TOL.
    float: the oracle decides every activation alone.  bfloat16: decisions inside the rounding band
    follow the library (Pair(ties="bounded")).  storage="exact": against the oracle that never rounds."""
    whole = OracleStage(o_units, in_shape, a, b, 1, storage='bf16' if dtype == 'bf16' and storage == "match" else None)
    op = OM.init_params(o_units, seed)
    for i in range(a, b):
        whole.set_params(i, [p.astype(np.float32).astype(np.float64) for p in op[i]])
    whole.forward(0, x)
    if labels is not None:
        whole.loss(0, labels)
    whole.backward(0, dy)
    if tol is None:
        tol = TOL_BF16_VS_EXACT if dtype == "bf16" and storage == "exact" else TOL[dtype]
    for i in range(a, b):
        kind = o_units[i].kind
        print(f"  unit {i} ({kind}) teacher-forced {dtype} against the {'rounding' if storage == 'match' and dtype == 'bf16' else 'exact'} oracle", flush=True)
        pair = Pair(o_units, h_units, in_shape, batch, i, i + 1, dtype, seed=seed, ties="bounded" if dtype == "bf16" else "off",
                    storage=storage, adopt_cap=ADOPT_CAP_EXACT if dtype == "bf16" and storage == "exact" else None)
        try:
            unit_compare(pair, i, kind, whole.unit_in[i], whole.unit_dout[i], labels, tol, report)
        finally:
            pair.close()


def unit_compare(pair, i, kind, x, dout, labels, tol, report=None):
    """forward, backward, update of a one-unit pair on given input / output gradient; everything compared at tol."""
    y, yo = pair.forward(0, x)
    e_y = assert_close(y, yo, tol, f"unit {i} y")
    if kind == 'loss':
        lh, lo = pair.loss(0, labels)
        assert abs(lh - lo) <= tol * max(1.0, abs(lo)), (lh, lo)
        dx, dxo = pair.backward(0, None)
    else:
        dx, dxo = pair.backward(0, dout)
    e_dx = assert_close(dx, dxo, tol, f"unit {i} dx")
    e_g = pair.compare_unit_vectors("grads", tol, floor=1e-7)
    pair.compare_unit_vectors("bn", tol)
    pair.update(0.01, 0.9, 4e-5)
    pair.compare_unit_vectors("weights", tol)
    if report is not None:
        report.append((i, kind, e_y, e_dx, e_g, dict(pair.tie_reports[-1])))


def _named(pair, which, side):
    """{name: flat float64 array} of the stage's per-unit vectors on one side ("lib" | "oracle");
    which: 'weights' | 'grads' | 'bn' (running statistics, library layout)."""
    P = pair.P
    out = {}
    pair.torch.cuda.synchronize()
    for i in range(pair.a, pair.b):
        if which == "bn":
            nb = P.model_unit_bn_channels(pair.model, i)
            if nb:
                out[f"u{i}.bn"] = (np.asarray(P.stage_export_bn_stats(pair.stage, i, 2 * nb), dtype=np.float64) if side == "lib" else
                                   np.concatenate([np.concatenate([rm, rv]) for rm, rv in pair.oracle.bn_run[i]]).astype(np.float64))
            continue
        n = P.model_unit_param_count(pair.model, i)
        if n == 0:
            continue
        names = [nm for nm, _, _, _ in OM.param_specs(pair.o_units[i])]
        if side == "lib":
            fn = {"weights": P.stage_export_weights, "grads": P.stage_export_grads}[which]
            flat, off = np.asarray(fn(pair.stage, i, n), dtype=np.float64), 0
            src = {"weights": pair.oracle.params, "grads": pair.oracle.grads}[which][i]
            for k, ref in enumerate(src):
                out[f"u{i}.{k}:{names[k]}"] = flat[off:off + ref.size].copy()
                off += ref.size
        else:
            src = {"weights": pair.oracle.params, "grads": pair.oracle.grads}[which][i]
            for k, ref in enumerate(src):
                out[f"u{i}.{k}:{names[k]}"] = np.asarray(ref, dtype=np.float64).ravel().copy()
    return out


def compare_named(A, B):
    """Per tensor (max-abs error / max-abs reference, relative L2 error) of A against the reference B; gamma and
    beta gradients of one BatchNorm on their joint scale, as in Pair.compare_unit_vectors."""
    table = {}
    keys = list(B)
    for idx, name in enumerate(keys):
        a, b = A[name], B[name]
        e = rel_err(a, b)
        base = name.split(":")[-1]
        mate = None
        if base.startswith("gamma") and idx + 1 < len(keys):
            mate = keys[idx + 1]
        elif base.startswith("beta") and idx > 0:
            mate = keys[idx - 1]
        if mate is not None and np.abs(b).max() > 0 and mate.split(".")[0] == name.split(".")[0]:
            sr = np.concatenate([b, B[mate]])
            d = a - b
            e = (min(e[0], np.abs(d).max() / max(np.abs(sr).max(), 1e-30)),
                 min(e[1], np.sqrt((d * d).sum()) / max(np.sqrt((sr * sr).sum()), 1e-30)))
        table[name] = e
    return table


def chained_report(o_units, h_units, in_shape, batch, a, b, dtype, seed, x, dy=None, labels=None, lr=0.01, mu=0.9, wd=4e-5):
    """One training step of stage [a,b) in the library on its OWN activations (nothing teacher-forced, no
    activation decision taken over), measured against two independent oracle runs of the same step: the one that
    rounds stored tensors to bfloat16 where the library does ("rounding") and the one that never rounds ("exact");
    the distance between the two oracles ("oracles") is the yardstick: it is what the storage roundings alone do
    to this step.  Returns {comparison: {tensor class: (worst max-abs error / max-abs reference, worst relative L2
    error)}} over the classes y, dx, loss, grads, weights (updated), bn (running statistics); prints the classes
    and, per unit, the worst weight-gradient error."""
    sides = {}
    for name, storage in (("rounding", "match"), ("exact", "exact")):
        pair = Pair(o_units, h_units, in_shape, batch, a, b, dtype, seed=seed, ties="off", storage=storage)
        lib, ora = {}, {}
        try:
            lib["y"], ora["y"] = [{"y": np.ravel(t)} for t in pair.forward(0, x)]
            if labels is not None:
                lh, lo = pair.loss(0, labels)
                lib["loss"], ora["loss"] = {"loss": np.array([lh, 1.0])}, {"loss": np.array([lo, 1.0])}
            dx, dxo = pair.backward(0, dy, want_dx=a > 0 or dy is not None)
            if dx is not None:
                lib["dx"], ora["dx"] = {"dx": np.ravel(dx)}, {"dx": np.ravel(dxo)}
            lib["grads"], ora["grads"] = _named(pair, "grads", "lib"), _named(pair, "grads", "oracle")
            lib["bn"], ora["bn"] = _named(pair, "bn", "lib"), _named(pair, "bn", "oracle")
            pair.update(lr, mu, wd)
            lib["weights"], ora["weights"] = _named(pair, "weights", "lib"), _named(pair, "weights", "oracle")
        finally:
            pair.close()
        sides[name] = ora
        sides["lib"] = lib                # the same both times: the kernels are deterministic
    out, per_unit = {}, {}
    for cmp_name, (A, B) in (("rounding", ("lib", "rounding")), ("exact", ("lib", "exact")), ("oracles", ("rounding", "exact"))):
        res = {}
        for cls in sides["lib"]:
            table = compare_named(sides[A][cls], sides[B][cls])
            res[cls] = (max(e[0] for e in table.values()), max(e[1] for e in table.values()))
            if cls == "grads":
                for nm, e in table.items():
                    u = nm.split(".")[0]
                    per_unit.setdefault(u, {})[cmp_name] = max(per_unit.get(u, {}).get(cmp_name, 0.0), max(e))
        out[cmp_name] = res
    label = {"rounding": "library vs rounding oracle", "exact": "library vs exact oracle   ", "oracles": "rounding vs exact oracle  "}
    for cls in sides["lib"]:
        print(f"  chained {dtype} [{a},{b}) {cls:8s} " + "   ".join(
            f"{label[c]}: {out[c][cls][0]:.2e} / {out[c][cls][1]:.2e}" for c in out), flush=True)
    print("  worst weight-gradient error per unit (library vs rounding | library vs exact | rounding vs exact):", flush=True)
    for u, d in per_unit.items():
        print(f"    {u:5s} {d.get('rounding', 0):.2e} | {d.get('exact', 0):.2e} | {d.get('oracles', 0):.2e}", flush=True)
    return out
