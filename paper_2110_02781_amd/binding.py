"""ctypes binding of include/ftp.h.  Argument marshalling only: every function
here has the name of the C entry point without the ftp_ prefix, converts
arguments, calls it and raises FtpError on a negative status.  Device buffers
are passed as integer addresses (e.g. torch_tensor.data_ptr()), streams as the
raw hipStream_t (e.g. torch.cuda.current_stream().cuda_stream).

There is no fallback: if libftp_hip.so has not been built, importing this module
raises."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libftp_hip.so")

F32, BF16 = 0, 1
UNIT_CONV, UNIT_INVRES, UNIT_GAP, UNIT_FC, UNIT_LOSS = range(5)
ACT_NONE, ACT_RELU, ACT_RELU6 = range(3)


class FtpError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"ftp status {status}: {msg}")
        self.status = status


class UnitDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("kind", "cin", "cout", "kh", "kw", "stride", "pad_h", "pad_w", "expand", "act")]


class KtraceRow(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("alg_bytes", C.c_double), ("flops", C.c_double)]


class Sgd(C.Structure):
    _fields_ = [("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float)]


def _load():
    # Callers hand us PyTorch device pointers and streams, so the library must bind to
    # the HIP runtime PyTorch has loaded (its wheel bundles one whose soname our
    # library's dependency resolves to once it is in the process).  Loading ours first
    # would put a second, separate runtime into the process.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2110_02781_amd.build` "
                          "(or __graft_entry__.build()) first; there is no CPU fallback")
    return C.CDLL(_LIB_PATH)


lib = _load()
_vp, _i, _sz = C.c_void_p, C.c_int, C.c_size_t
_fp = C.POINTER(C.c_float)
_dp = C.POINTER(C.c_double)
_SIGS = {
    "ftp_last_error": (C.c_char_p, []),
    "ftp_model_create": (_i, [C.POINTER(UnitDesc), _i, _i, _i, _i, _i, C.POINTER(_vp)]),
    "ftp_model_destroy": (None, [_vp]),
    "ftp_model_num_units": (_i, [_vp]),
    "ftp_model_unit_in_shape": (_i, [_vp, _i, C.POINTER(_i), C.POINTER(_i), C.POINTER(_i)]),
    "ftp_model_unit_param_count": (_i, [_vp, _i, C.POINTER(_sz)]),
    "ftp_model_unit_bn_channels": (_i, [_vp, _i, C.POINTER(_sz)]),
    "ftp_stage_create": (_i, [_vp, _i, _i, _i, _i, C.POINTER(_vp)]),
    "ftp_stage_create_ex": (_i, [_vp, _i, _i, _i, _i, C.c_uint, C.POINTER(_vp)]),
    "ftp_stage_device_bytes": (_i, [_vp, C.POINTER(_sz)]),
    "ftp_stage_destroy": (None, [_vp]),
    "ftp_stage_import_weights": (_i, [_vp, _i, _fp, _sz]),
    "ftp_stage_export_weights": (_i, [_vp, _i, _fp, _sz]),
    "ftp_stage_export_grads": (_i, [_vp, _i, _fp, _sz]),
    "ftp_stage_export_momentum": (_i, [_vp, _i, _fp, _sz]),
    "ftp_stage_export_bn_stats": (_i, [_vp, _i, _fp, _sz]),
    "ftp_stage_export_conv_output": (_i, [_vp, _i, _i, _i, _fp, _sz]),
    "ftp_stage_export_bn_batch_stats": (_i, [_vp, _i, _i, _i, _fp, _sz]),
    "ftp_stage_forward": (_i, [_vp, _i, _vp, _vp, _vp]),
    "ftp_stage_loss": (_i, [_vp, _i, _vp, _vp, _vp]),
    "ftp_softmax_ce_static": (_i, [_vp, _vp, _i, _i, _i, _vp, _vp, _vp]),
    "ftp_stage_snapshot_weights": (_i, [_vp, _i, _vp]),
    "ftp_stage_aggregate_weights": (_i, [_vp, C.POINTER(C.c_int), _i, _vp]),
    "ftp_stage_backward": (_i, [_vp, _i, _vp, _vp, _vp]),
    "ftp_stage_update": (_i, [_vp, C.POINTER(Sgd), _vp]),
    "ftp_profile_layers": (_i, [_vp, _i, _i, _dp, C.POINTER(C.c_int64), _vp]),
    "ftp_solve_partition": (_i, [_dp, _i, _dp, _i, _dp, _dp, C.POINTER(C.c_int32), _dp]),
    "ftp_estimate_capacity": (_i, [C.c_double, _dp, _i, _i, _i, _dp]),
    "ftp_repartition_due": (_i, [C.c_int64, C.POINTER(_i)]),
    "ftp_repartition_capacities": (_i, [_dp, _dp, _i, C.POINTER(C.c_int32), _i, _dp]),
    "ftp_redistribution_plan": (_i, [C.POINTER(C.c_int32), _i, C.POINTER(C.c_int32), _i, _i, _i, _i, C.POINTER(C.c_int32)]),
    "ftp_renumber_workers": (_i, [C.POINTER(C.c_int32), _i, C.POINTER(C.c_int32), _i, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                  C.POINTER(_i)]),
    "ftp_stage_copy_units": (_i, [_vp, _vp, _i, _i, _vp]),
    "ftp_stage_timing": (_i, [_vp, _i]),
    "ftp_stage_timing_read": (_i, [_vp, _dp, C.POINTER(C.c_int)]),
    "ftp_calibration_copy": (_i, [_vp, _vp, _sz, _vp]),
    "ftp_diag_fail_next_launch_plan": (_i, []),
    "ftp_ktrace_begin": (_i, [_i]),
    "ftp_ktrace_end": (_i, [C.POINTER(KtraceRow), _i, C.POINTER(_i)]),
}
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args


def last_error():
    return lib.ftp_last_error().decode()


def _chk(rc):
    if rc < 0:
        raise FtpError(rc, last_error())
    return rc


def _ptr(p):
    """tensor / int / None -> void*"""
    if p is None:
        return None
    if hasattr(p, "data_ptr"):
        return C.c_void_p(p.data_ptr())
    return C.c_void_p(int(p))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_fp)


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


# ---- model ---------------------------------------------------------------------
def model_create(units, in_h, in_w, in_c, act_dtype=F32):
    """units: sequence of dicts / UnitDesc with the fields of ftp_unit_desc."""
    arr = (UnitDesc * len(units))()
    for i, u in enumerate(units):
        if isinstance(u, UnitDesc):
            arr[i] = u
        else:
            for f, _ in UnitDesc._fields_:
                setattr(arr[i], f, int(u.get(f, 0)))
    out = _vp()
    _chk(lib.ftp_model_create(arr, len(units), in_h, in_w, in_c, act_dtype, C.byref(out)))
    return out


def model_destroy(model):
    lib.ftp_model_destroy(model)


def model_num_units(model):
    return _chk(lib.ftp_model_num_units(model))


def model_unit_in_shape(model, u):
    h, w, c = _i(), _i(), _i()
    _chk(lib.ftp_model_unit_in_shape(model, u, C.byref(h), C.byref(w), C.byref(c)))
    return h.value, w.value, c.value


def model_unit_param_count(model, u):
    n = _sz()
    _chk(lib.ftp_model_unit_param_count(model, u, C.byref(n)))
    return n.value


def model_unit_bn_channels(model, u):
    n = _sz()
    _chk(lib.ftp_model_unit_bn_channels(model, u, C.byref(n)))
    return n.value


# ---- stage ---------------------------------------------------------------------
STAGE_RECOMPUTE = 1


def stage_create(model, a, b, batch, n_slots=1, flags=0):
    out = _vp()
    if flags:
        _chk(lib.ftp_stage_create_ex(model, a, b, batch, n_slots, flags, C.byref(out)))
    else:
        _chk(lib.ftp_stage_create(model, a, b, batch, n_slots, C.byref(out)))
    return out


def stage_device_bytes(stage):
    n = _sz(0)
    _chk(lib.ftp_stage_device_bytes(stage, C.byref(n)))
    return int(n.value)


def stage_destroy(stage):
    lib.ftp_stage_destroy(stage)


def stage_import_weights(stage, unit, host_w):
    a, p = _f32(host_w)
    _chk(lib.ftp_stage_import_weights(stage, unit, p, a.size))


def _export(fn, stage, unit, n):
    out = np.empty(n, dtype=np.float32)
    _chk(fn(stage, unit, out.ctypes.data_as(_fp), n))
    return out


def stage_export_weights(stage, unit, n):
    return _export(lib.ftp_stage_export_weights, stage, unit, n)


def stage_export_grads(stage, unit, n):
    return _export(lib.ftp_stage_export_grads, stage, unit, n)


def stage_export_momentum(stage, unit, n):
    return _export(lib.ftp_stage_export_momentum, stage, unit, n)


def stage_export_bn_stats(stage, unit, n):
    return _export(lib.ftp_stage_export_bn_stats, stage, unit, n)


def stage_export_conv_output(stage, slot, unit, conv, n):
    out = np.empty(n, dtype=np.float32)
    _chk(lib.ftp_stage_export_conv_output(stage, slot, unit, conv, out.ctypes.data_as(_fp), n))
    return out


def stage_export_bn_batch_stats(stage, slot, unit, conv, n):
    out = np.empty(n, dtype=np.float32)
    _chk(lib.ftp_stage_export_bn_batch_stats(stage, slot, unit, conv, out.ctypes.data_as(_fp), n))
    return out


def stage_forward(stage, slot, x_dev, y_dev=None, stream=None):
    _chk(lib.ftp_stage_forward(stage, slot, _ptr(x_dev), _ptr(y_dev), _ptr(stream)))


def stage_loss(stage, slot, labels_dev, loss_dev, stream=None):
    _chk(lib.ftp_stage_loss(stage, slot, _ptr(labels_dev), _ptr(loss_dev), _ptr(stream)))


STATIC_LOSS_MAX_BATCH = 65536


def softmax_ce_static(logits_dev, labels_dev, batch, classes, dtype, dlogits_dev, loss_dev, stream=None):
    _chk(lib.ftp_softmax_ce_static(_ptr(logits_dev), _ptr(labels_dev), batch, classes, dtype, _ptr(dlogits_dev), _ptr(loss_dev),
                                   _ptr(stream)))


def stage_snapshot_weights(stage, slot, stream=None):
    _chk(lib.ftp_stage_snapshot_weights(stage, slot, _ptr(stream)))


def stage_aggregate_weights(stage, slots, stream=None):
    arr = (C.c_int * len(slots))(*[int(s) for s in slots])
    _chk(lib.ftp_stage_aggregate_weights(stage, arr, len(slots), _ptr(stream)))


def stage_backward(stage, slot, dy_dev=None, dx_dev=None, stream=None):
    _chk(lib.ftp_stage_backward(stage, slot, _ptr(dy_dev), _ptr(dx_dev), _ptr(stream)))


def stage_update(stage, lr, momentum, weight_decay, stream=None):
    opt = Sgd(lr, momentum, weight_decay)
    _chk(lib.ftp_stage_update(stage, C.byref(opt), _ptr(stream)))


# ---- profiling and partition -----------------------------------------------------
def profile_layers(model, batch, reps=10, stream=None):
    L = model_num_units(model)
    t = np.zeros(L, dtype=np.float64)
    ob = np.zeros(L, dtype=np.int64)
    _chk(lib.ftp_profile_layers(model, batch, reps, t.ctypes.data_as(_dp),
                                ob.ctypes.data_as(C.POINTER(C.c_int64)), _ptr(stream)))
    return t, ob


def solve_partition(layer_costs, device_capacities, out_bytes=None, bandwidth=None):
    c, cp = _f64(layer_costs)
    k, kp = _f64(device_capacities)
    dp = bp = None
    if out_bytes is not None and bandwidth is not None:
        d, dp = _f64(out_bytes)
        b, bp = _f64(bandwidth)
    bounds = np.zeros(k.size + 1, dtype=np.int32)
    bott = C.c_double()
    _chk(lib.ftp_solve_partition(cp, c.size, kp, k.size, dp, bp,
                                 bounds.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(bott)))
    return bounds, bott.value


def estimate_capacity(stage_time, layer_costs, start, end):
    c, cp = _f64(layer_costs)
    out = C.c_double()
    _chk(lib.ftp_estimate_capacity(stage_time, cp, c.size, start, end, C.byref(out)))
    return out.value


# ---- diagnostics ---------------------------------------------------------------------
def ktrace_begin(max_launches=65536):
    _chk(lib.ftp_ktrace_begin(max_launches))


def ktrace_end():
    """-> list of dicts: name, launches, total_ms, alg_bytes, flops (one per kernel family)."""
    rows = (KtraceRow * 512)()
    n = _i()
    _chk(lib.ftp_ktrace_end(rows, 512, C.byref(n)))
    return [dict(name=rows[i].name.decode(), launches=rows[i].launches, total_ms=rows[i].total_ms,
                 alg_bytes=rows[i].alg_bytes, flops=rows[i].flops) for i in range(n.value)]


def diag_fail_next_launch_plan():
    _chk(lib.ftp_diag_fail_next_launch_plan())


def calibration_copy(dst_dev, src_dev, nbytes, stream=None):
    _chk(lib.ftp_calibration_copy(_ptr(dst_dev), _ptr(src_dev), nbytes, _ptr(stream)))


def repartition_due(batches_done):
    due = _i(0)
    _chk(lib.ftp_repartition_due(int(batches_done), C.byref(due)))
    return bool(due.value)


def repartition_capacities(mean_times, layer_costs, bounds_cur):
    """mean_times: per worker, None (or nan) where nothing was reported."""
    m, mp = _f64([float("nan") if v is None else float(v) for v in mean_times])
    c, cp = _f64(layer_costs)
    b = (C.c_int32 * len(bounds_cur))(*[int(v) for v in bounds_cur])
    n = len(bounds_cur) - 1
    out = np.zeros(n, dtype=np.float64)
    _chk(lib.ftp_repartition_capacities(mp, cp, len(c), b, n, out.ctypes.data_as(_dp)))
    return [float(v) for v in out]


def redistribution_plan(bounds_new, bounds_cur, i_fail, i_cur, i_new):
    """Returns (M_need, L_local) like the paper's algorithm: {worker index in the new numbering: [units]}, [units held]."""
    bn = (C.c_int32 * len(bounds_new))(*[int(v) for v in bounds_new])
    bc = (C.c_int32 * len(bounds_cur))(*[int(v) for v in bounds_cur])
    n = int(bounds_new[i_new + 1]) - int(bounds_new[i_new]) if 0 <= i_new < len(bounds_new) - 1 else 1
    src = (C.c_int32 * max(n, 1))()
    _chk(lib.ftp_redistribution_plan(bn, len(bounds_new) - 1, bc, len(bounds_cur) - 1, -1 if i_fail is None else int(i_fail),
                                     int(i_cur), int(i_new), src))
    m_need, local = {}, []
    for j in range(n):
        unit = int(bounds_new[i_new]) + j
        if src[j] < 0:
            local.append(unit)
        else:
            m_need.setdefault(int(src[j]), []).append(unit)
    return m_need, local


def renumber_workers(worker_ids, failed):
    """-> (new worker list, old index -> new index with -1 for the failed)."""
    ids = np.ascontiguousarray(worker_ids, dtype=np.int32)
    fl = np.ascontiguousarray(failed, dtype=np.int32)
    out = np.zeros(max(len(ids), 1), dtype=np.int32)
    idx = np.zeros(max(len(ids), 1), dtype=np.int32)
    n_new = C.c_int(0)
    i32p = C.POINTER(C.c_int32)
    _chk(lib.ftp_renumber_workers(ids.ctypes.data_as(i32p), len(ids), fl.ctypes.data_as(i32p), len(fl),
                                  out.ctypes.data_as(i32p), idx.ctypes.data_as(i32p), C.byref(n_new)))
    return [int(v) for v in out[:n_new.value]], [int(v) for v in idx[:len(ids)]]


def stage_copy_units(dst, src, unit_lo, unit_hi, stream=None):
    _chk(lib.ftp_stage_copy_units(dst, src, unit_lo, unit_hi, _ptr(stream)))


def stage_timing(stage, enable):
    _chk(lib.ftp_stage_timing(stage, 1 if enable else 0))


def stage_timing_read(stage):
    """Returns (mean forward+backward nanoseconds per batch, number of batches) since the last read."""
    mean, n = C.c_double(0.0), C.c_int(0)
    _chk(lib.ftp_stage_timing_read(stage, C.byref(mean), C.byref(n)))
    return mean.value, n.value
