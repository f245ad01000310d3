"""ctypes binding of include/daris.h.  Function names and argument order follow the C ABI one to one;
the only additions are `make_dnn` (packs a Python layer table + numpy weights into a `daris_dnn`),
`trace_read_all` (decodes the 32-byte records) and error-code-to-exception conversion."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DARIS_LIB") or os.path.join(_HERE, "libdaris.so")   # DARIS_LIB: another build of the same sources

OK, EINVAL, ENOMEM, EHIP, ESTATE, ERANGE = 0, -1, -2, -3, -4, -5
VIRTUAL_TIME, NO_DEVICE, NO_LAST, NO_PRIOR, NO_FIXED, HP_ADMISSION, KEEP_ACTIVATIONS, WAVE_PRIORITY, SHARED_QUEUE = 1, 2, 4, 8, 16, 32, 64, 128, 256
NO_PAIR, NO_FUSED_INGEST, NO_STAGED_ROWS, NO_SMALL_TILES, NO_FUSED_DW = 512, 1024, 2048, 4096, 8192
LP, HP = 0, 1
FP32, BF16 = 0, 1
ACCEPTED, MIGRATED, REJECT_ADMISSION, REJECT_OVERRUN, QUEUED = 1, 2, 3, 4, 5
T_RELEASE, T_ACCEPT, T_REJECT, T_MIGRATE, T_DISPATCH, T_STAGE_DONE, T_JOB_DONE, T_QUEUED, T_CMD_MIGRATE = range(1, 10)


class DarisError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"daris error {code}: {text}")
        self.code = code


class daris_layer(C.Structure):
    _fields_ = [("op", C.c_int32), ("c_in", C.c_int32), ("c_out", C.c_int32), ("k", C.c_int32), ("stride", C.c_int32),
                ("pad", C.c_int32), ("groups", C.c_int32), ("act", C.c_int32), ("in_from", C.c_int32),
                ("res_from", C.c_int32), ("w", C.POINTER(C.c_float)), ("b", C.POINTER(C.c_float))]


class daris_dnn(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("dtype", C.c_int32), ("layers", C.POINTER(daris_layer))]


class daris_task_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("released", "accepted", "completed", "missed", "rejected_admission",
                                         "rejected_overrun", "resp_min_ns", "resp_max_ns", "resp_sum_ns",
                                         "first_release_ns", "last_finish_ns")] + [("partition", C.c_int32), ("n_stages", C.c_int32)]


TRACE_DTYPE = np.dtype([("seq", "<u8"), ("t_ns", "<i8"), ("type", "u1"), ("level", "u1"), ("stage", "u1"),
                        ("partition", "u1"), ("task", "<u2"), ("stream", "<u2"), ("job", "<u4"), ("aux", "<u4")])
assert TRACE_DTYPE.itemsize == 32

_lib = None

_SIGS = {
    "daris_init": (C.c_int32, [C.c_int, C.c_uint64, C.c_int]),
    "daris_shutdown": (C.c_int32, []),
    "daris_set_timeout": (C.c_int32, [C.c_int64]),
    "daris_set_plan_cus": (C.c_int32, [C.c_int32]),
    "daris_last_error": (C.c_char_p, []),
    "daris_cu_per_partition": (C.c_int32, [C.c_int32] * 4),
    "daris_create_partition": (C.c_int32, [C.c_int]),
    "daris_partition_set_streams": (C.c_int32, [C.c_int32, C.c_int]),
    "daris_partition_get_mask": (C.c_int32, [C.c_int32, C.POINTER(C.c_uint32)]),
    "daris_register_task": (C.c_int32, [C.POINTER(daris_dnn), C.c_int64, C.c_int64, C.c_int]),
    "daris_split_stages": (C.c_int32, [C.c_int32, C.c_int]),
    "daris_get_stage_cuts": (C.c_int32, [C.c_int32, C.POINTER(C.c_int32), C.c_int32]),
    "daris_set_afet": (C.c_int32, [C.c_int32, C.c_int, C.c_int64]),
    "daris_set_window": (C.c_int32, [C.c_int]),
    "daris_set_virtual_time": (C.c_int32, [C.c_int32, C.c_int, C.c_int32, C.c_int64, C.c_int64, C.POINTER(C.c_int64)]),
    "daris_commit": (C.c_int32, []),
    "daris_get_partition": (C.c_int32, [C.c_int32]),
    "daris_release_job": (C.c_int32, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_int32)]),
    "daris_migrate": (C.c_int32, [C.c_int32, C.c_int32]),
    "daris_run_until_idle": (C.c_int32, []),
    "daris_task_set_io": (C.c_int32, [C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32]),
    "daris_run_periodic": (C.c_int32, [C.POINTER(C.c_int64), C.POINTER(C.c_int32)]),
    "daris_run_closed_loop": (C.c_int32, [C.POINTER(C.c_int32), C.c_int64]),
    "daris_get_stats": (C.c_int32, [C.c_int32, C.POINTER(daris_task_stats)]),
    "daris_trace_read": (C.c_int64, [C.c_void_p, C.c_int64]),
    "daris_get_mret": (C.c_int64, [C.c_int32, C.c_int]),
    "daris_forward": (C.c_int32, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32]),
    "daris_forward_static": (C.c_int32, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32]),
    "daris_read_layer": (C.c_int32, [C.c_int32, C.c_int, C.POINTER(C.c_float), C.c_int64]),
    "daris_profile_layers": (C.c_int32, [C.c_int32, C.c_int32, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "daris_kernel_name": (C.c_char_p, [C.c_int32]),
    "daris_calibrate_afet": (C.c_int32, [C.c_int32, C.c_int32, C.c_int]),
    "daris_calibrate_afet_loaded": (C.c_int32, [C.c_int32, C.c_int32, C.c_int]),
    "daris_kernel_timing_start": (C.c_int32, [C.c_int, C.c_int]),
    "daris_driver_profile": (C.c_int32, [C.c_int, C.POINTER(C.c_int64)]),
    "daris_get_launch_plan": (C.c_int32, [C.c_int32, C.c_int, C.POINTER(C.c_int64), C.c_int32]),
    "daris_kernel_timing_read": (C.c_int32, [C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "daris_probe_cus": (C.c_int32, [C.c_int32, C.c_int, C.c_int, C.POINTER(C.c_uint32)]),
}
EXPORTS = sorted(_SIGS)


def lib():
    """The loaded shared library; raises if libdaris.so has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise DarisError(ESTATE, f"{LIB_PATH} not built: run `python -m paper_2504_08795_amd.build`")
        # PyTorch owns the device memory the caller passes in, so both must use ONE HIP runtime: import torch first,
        # then libdaris.so binds to the libamdhip64.so.7 that torch has already mapped into the process.
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            f = getattr(_lib, name)
            f.restype, f.argtypes = res, args
    return _lib


def _chk(code):
    if code < 0:
        raise DarisError(code, lib().daris_last_error().decode())
    return code


def _ptr(x):
    """Device pointer of a torch tensor / int address / None."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    return C.c_void_p(int(x))


def daris_init(device=0, seed=0, flags=0):
    return _chk(lib().daris_init(device, seed, flags))


def daris_shutdown():
    return _chk(lib().daris_shutdown())


def daris_set_timeout(ns):
    return _chk(lib().daris_set_timeout(int(ns)))


def daris_set_plan_cus(n_cu):
    return _chk(lib().daris_set_plan_cus(int(n_cu)))


def daris_cu_per_partition(os_num, os_den, n_cu_max, n_c):
    return _chk(lib().daris_cu_per_partition(os_num, os_den, n_cu_max, n_c))


def daris_create_partition(n_cu):
    return _chk(lib().daris_create_partition(n_cu))


def daris_partition_set_streams(p, n_s):
    return _chk(lib().daris_partition_set_streams(p, n_s))


def daris_partition_get_mask(p):
    m = (C.c_uint32 * 8)()
    _chk(lib().daris_partition_get_mask(p, m))
    return list(m)


def make_dnn(layers, weights, in_shape, dtype):
    """Build a daris_dnn from records with fields op, c_in, c_out, k, stride, pad, groups, act, in_from, res_from and
    per-layer (w, b) float32 numpy arrays (or (None, None)).  Returns (dnn, keepalive)."""
    arr = (daris_layer * len(layers))()
    keep = [arr]
    fp = C.POINTER(C.c_float)
    for i, L in enumerate(layers):
        w, b = weights[i] if weights is not None else (None, None)
        a = arr[i]
        a.op, a.c_in, a.c_out, a.k, a.stride, a.pad = L.op, L.c_in, L.c_out, L.k, L.stride, L.pad
        a.groups, a.act, a.in_from, a.res_from = L.groups, L.act, L.in_from, L.res_from
        if w is not None:
            w = np.ascontiguousarray(w, np.float32)
            keep.append(w)
            a.w = w.ctypes.data_as(fp)
        if b is not None:
            b = np.ascontiguousarray(b, np.float32)
            keep.append(b)
            a.b = b.ctypes.data_as(fp)
    d = daris_dnn(len(layers), in_shape[0], in_shape[1], in_shape[2], BF16 if dtype in (BF16, "bf16") else FP32, arr)
    return d, keep


def daris_register_task(dnn, period_ns, deadline_ns, priority):
    return _chk(lib().daris_register_task(C.byref(dnn), period_ns, deadline_ns, priority))


def daris_split_stages(t, k):
    return _chk(lib().daris_split_stages(t, k))


def daris_get_stage_cuts(t):
    buf = (C.c_int32 * 256)()
    n = _chk(lib().daris_get_stage_cuts(t, buf, 256))
    return list(buf[:n])


PLAN_FIELDS = ("kernel_id", "dense_conv", "rows", "M", "N", "K", "Kpad", "tn", "nw", "S", "sz", "sw", "splitk", "MT", "NTn", "G", "xmode",
               "grid_x", "grid_y", "grid_z", "threads", "ws_bytes", "pair_with", "pair_lead", "out_slot", "in_slot", "res_slot")


def daris_get_launch_plan(t, layer):
    buf = (C.c_int64 * 27)()
    _chk(lib().daris_get_launch_plan(t, layer, buf, 27))
    return dict(zip(PLAN_FIELDS, (int(v) for v in buf)))


def daris_set_afet(t, stage, ns):
    return _chk(lib().daris_set_afet(t, stage, int(ns)))


def daris_set_window(ws):
    return _chk(lib().daris_set_window(ws))


def daris_set_virtual_time(t, stage, p, job_lo, job_hi, et_ns):
    a = np.ascontiguousarray(et_ns, np.int64)
    assert a.size == job_hi - job_lo
    return _chk(lib().daris_set_virtual_time(t, stage, p, job_lo, job_hi, a.ctypes.data_as(C.POINTER(C.c_int64))))


def daris_commit():
    return _chk(lib().daris_commit())


def daris_get_partition(t):
    return _chk(lib().daris_get_partition(t))


def daris_release_job(t, d_input, d_logits, release_ns=-1):
    dec = C.c_int32(0)
    _chk(lib().daris_release_job(t, _ptr(d_input), _ptr(d_logits), int(release_ns), C.byref(dec)))
    return dec.value


def daris_migrate(t, p):
    return _chk(lib().daris_migrate(t, p))


def daris_run_until_idle():
    return _chk(lib().daris_run_until_idle())


def daris_task_set_io(t, d_inputs, n_inputs, d_logits, n_slots):
    return _chk(lib().daris_task_set_io(t, _ptr(d_inputs), n_inputs, _ptr(d_logits), n_slots))


def daris_run_periodic(phase_ns, n_jobs):
    n = np.ascontiguousarray(n_jobs, np.int32)
    ph = None if phase_ns is None else np.ascontiguousarray(phase_ns, np.int64)
    return _chk(lib().daris_run_periodic(None if ph is None else ph.ctypes.data_as(C.POINTER(C.c_int64)),
                                         n.ctypes.data_as(C.POINTER(C.c_int32))))


def daris_run_closed_loop(n_jobs, total_jobs=0):
    n = np.ascontiguousarray(n_jobs, np.int32)
    return _chk(lib().daris_run_closed_loop(n.ctypes.data_as(C.POINTER(C.c_int32)), int(total_jobs)))


def daris_get_stats(t):
    s = daris_task_stats()
    _chk(lib().daris_get_stats(t, C.byref(s)))
    return {n: getattr(s, n) for n, _ in daris_task_stats._fields_}


def daris_trace_read(max_records=1 << 16):
    buf = np.empty(max_records, TRACE_DTYPE)
    n = _chk(lib().daris_trace_read(buf.ctypes.data_as(C.c_void_p), buf.nbytes))
    return buf[: n // 32]


def trace_read_all():
    """All unread trace records as a list of tuples (seq, t, type, level, stage, partition, task, stream, job, aux)."""
    out = []
    while True:
        chunk = daris_trace_read()
        if len(chunk) == 0:
            return out
        out += [tuple(int(v) for v in r) for r in chunk.tolist()]


def daris_get_mret(t, stage):
    return _chk(lib().daris_get_mret(t, stage))


def daris_forward(t, d_input, d_logits, p=0):
    return _chk(lib().daris_forward(t, _ptr(d_input), _ptr(d_logits), p))


def daris_forward_static(t, d_input, d_logits, p=0):
    return _chk(lib().daris_forward_static(t, _ptr(d_input), _ptr(d_logits), p))


def daris_read_layer(t, layer, n_elems):
    out = np.empty(n_elems, np.float32)
    _chk(lib().daris_read_layer(t, layer, out.ctypes.data_as(C.POINTER(C.c_float)), n_elems))
    return out


def daris_profile_layers(t, p, reps, n_layers):
    ms = np.zeros(n_layers, np.float32)
    kid = np.zeros(n_layers, np.int32)
    fl = np.zeros(n_layers, np.float64)
    _chk(lib().daris_profile_layers(t, p, reps, ms.ctypes.data_as(C.POINTER(C.c_float)), kid.ctypes.data_as(C.POINTER(C.c_int32)),
                                    fl.ctypes.data_as(C.POINTER(C.c_double))))
    return ms, kid, fl


def daris_kernel_name(kernel_id):
    return lib().daris_kernel_name(int(kernel_id)).decode()


def daris_kernel_timing_start(every, max_samples):
    return _chk(lib().daris_kernel_timing_start(every, max_samples))


def daris_kernel_timing_read():
    """({kernel name: (launches, total_ms, total_flops)}, empty_pair_ms) of the sampled launches since daris_kernel_timing_start."""
    n, ms, fl = np.zeros(64, np.int64), np.zeros(64, np.float64), np.zeros(64, np.float64)
    ov = C.c_double(0.0)
    k = _chk(lib().daris_kernel_timing_read(64, n.ctypes.data_as(C.POINTER(C.c_int64)), ms.ctypes.data_as(C.POINTER(C.c_double)),
                                            fl.ctypes.data_as(C.POINTER(C.c_double)), C.byref(ov)))
    return {daris_kernel_name(i): (int(n[i]), float(ms[i]), float(fl[i])) for i in range(k) if n[i] > 0}, ov.value


def daris_driver_profile(enable):
    """Totals since the last call (dict, ns) of where the stages' wall time went; switches the gathering on or off."""
    out = np.zeros(8, np.int64)
    _chk(lib().daris_driver_profile(int(bool(enable)), out.ctypes.data_as(C.POINTER(C.c_int64))))
    keys = ("stages", "enqueue_ns", "wait_ns", "lock_ns", "sched_ns", "gpu_ns", "handover_ns")
    return {k: int(out[i]) for i, k in enumerate(keys)}


def daris_calibrate_afet(t, p, reps=5):
    return _chk(lib().daris_calibrate_afet(t, p, reps))


def daris_calibrate_afet_loaded(t, p, reps=5):
    return _chk(lib().daris_calibrate_afet_loaded(t, p, reps))


def daris_probe_cus(p, n_groups=2048, spin=2000):
    """(xcc_id, hw_id) per workgroup of a probe launch on stream 0 of partition p."""
    out = np.zeros(2 * n_groups, np.uint32)
    _chk(lib().daris_probe_cus(p, n_groups, spin, out.ctypes.data_as(C.POINTER(C.c_uint32))))
    return out.reshape(n_groups, 2)
