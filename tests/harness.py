"""Shared helpers of the GPU parity tests: build the same stage in the oracle and
in the HIP library from the seeded generators, run both, compare tensors."""
import numpy as np

import synth
from oracle import models as OM
from oracle.stage import Stage as OracleStage

TOL = {"f32": 1e-4, "bf16": 2e-2}


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


def assert_close(a, b, tol, what, floor=0.0):
    """Both the max-abs and the L2 relative error must be within tol.  `floor`:
    tensors whose reference is numerically zero (below floor) are compared absolutely."""
    assert np.all(np.isfinite(np.asarray(a, dtype=np.float64))), f"{what}: non-finite values"
    if np.abs(np.asarray(b)).max() <= floor:
        assert np.abs(np.asarray(a)).max() <= max(floor, 1e-30) * 10, f"{what}: expected ~0"
        return 0.0, 0.0
    e_max, e_l2 = rel_err(a, b)
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

    def __init__(self, o_units, h_units, in_shape, batch, a, b, dtype="f32", n_slots=1, seed=1):
        import torch
        import paper_2110_02781_amd as P
        self.P, self.torch = P, torch
        self.dtype, self.batch, self.a, self.b = dtype, batch, a, b
        self.o_units, self.h_units = o_units, h_units
        self.dev = torch.device("cuda:0")
        self.tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        H, W, Cc = in_shape
        self.model = P.model_create(h_units, H, W, Cc, P.F32 if dtype == "f32" else P.BF16)
        self.stage = P.stage_create(self.model, a, b, batch, n_slots)
        self.oracle = OracleStage(o_units, in_shape, a, b, n_slots, storage='bf16' if dtype == 'bf16' else None)
        op = OM.init_params(o_units, seed)
        hp = P.models.init_unit_params(h_units, seed)
        for i in range(a, b):
            flat = flat_params(op[i])
            assert np.array_equal(flat.astype(np.float32), hp[i]), "both sides must draw identical weights"
            # masters are fp32 on both sides; in bf16 mode each side rounds its own working copy
            self.oracle.set_params(i, [p.astype(np.float32).astype(np.float64) for p in op[i]])
            P.stage_import_weights(self.stage, i, hp[i])
        self.in_shape = self.oracle.shapes[a]
        self.out_shape = self.oracle.shapes[b]
        self.stream = torch.cuda.current_stream().cuda_stream

    def close(self):
        self.P.stage_destroy(self.stage)
        self.P.model_destroy(self.model)

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
        xd = self.dev_tensor(x)
        y = self.empty((self.batch,) + tuple(self.out_shape))
        P.stage_forward(self.stage, slot, xd, y, self.stream)
        if snapshot:
            P.stage_snapshot_weights(self.stage, slot, self.stream)
        yo = self.oracle.forward(slot, self.as_seen(x), stash_weights=snapshot)
        return self.host(y), yo

    def loss(self, slot, labels):
        P, torch = self.P, self.torch
        ld = torch.from_numpy(np.asarray(labels, dtype=np.int32)).to(self.dev)
        out = torch.zeros(1, dtype=torch.float32, device=self.dev)
        P.stage_loss(self.stage, slot, ld, out, self.stream)
        lo = self.oracle.loss(slot, labels)
        return float(self.host(out)[0]), lo

    def backward(self, slot, dy=None, want_dx=True):
        P = self.P
        dyd = self.dev_tensor(dy) if dy is not None else None
        dx = self.empty((self.batch,) + tuple(self.in_shape)) if want_dx else None
        P.stage_backward(self.stage, slot, dyd, dx, self.stream)
        dxo = self.oracle.backward(slot, None if dy is None else self.as_seen(dy))
        return (self.host(dx) if want_dx else None), dxo

    def update(self, lr, mu, wd):
        self.P.stage_update(self.stage, lr, mu, wd, self.stream)
        self.oracle.update(lr, mu, wd)

    # -- comparisons ------------------------------------------------------------------
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
                ref = np.concatenate([np.concatenate([rm, rv]) for rm, rv in self.oracle.bn_run[i]])
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
            off = 0
            for k, ref in enumerate(src[i]):
                m = ref.size
                e = assert_close(got[off:off + m], ref.ravel(), tol, f"unit {i} {which}[{k}]", floor)
                worst = (max(worst[0], e[0]), max(worst[1], e[1]))
                off += m
        return worst
