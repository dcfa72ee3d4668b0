"""ctypes binding of the scheduler / metrics entry points declared in include/kvsched.h
(same shared library as kvswap; host-only code).  Argument marshalling only."""
import ctypes as C

import numpy as np

from . import kvswap as _kv

_lib = _kv._lib

KVS_OK, KVS_EINVAL, KVS_ENOMEM = 0, -1, -2
KVS_NEW, KVS_RUNNING, KVS_PREEMPTED = 0, 1, 2
KVS_KEEP, KVS_RUN, KVS_PREEMPT = 0, 1, 2
KVS_BY_LOAD, KVS_BY_RECOMPUTE = 0, 1
KVS_MODE_IDLE, KVS_MODE_BUFFER_AWARE, KVS_MODE_FCFS = 0, 1, 2

EXPORTS = ["kv_metric_stream", "kv_metric_token_weight", "kv_metric_weight_sum", "kv_metric_effective_sum",
           "kv_metric_qos", "kv_sched_step"]


class kv_sched_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("mem_blocks", C.c_int64), ("ws_blocks", C.c_int64),
                ("max_running", C.c_int32), ("interval", C.c_double), ("gen_rate", C.c_double),
                ("capacity", C.c_double), ("gamma", C.c_double), ("safety", C.c_double), ("w_adjust", C.c_double),
                ("t_critical", C.c_double), ("tau_schedule", C.c_double), ("weight_tau", C.c_double),
                ("weight_alpha", C.c_double), ("evict_gbps", C.c_double), ("load_gbps", C.c_double),
                ("io_fixed", C.c_double), ("evict_queue", C.c_double), ("load_queue", C.c_double),
                ("block_bytes", C.c_double), ("prefill_per_token", C.c_double)]


class kv_sched_req(C.Structure):
    _fields_ = [("state", C.c_int32), ("arrival", C.c_double), ("rate", C.c_double), ("buffer", C.c_double),
                ("blocks", C.c_int32), ("dirty_blocks", C.c_int32), ("tokens", C.c_int32)]


class kv_sched_out(C.Structure):
    _fields_ = [("decision", C.c_int32), ("how", C.c_int32), ("priority_buffer", C.c_double), ("value", C.c_double),
                ("t_overhead", C.c_double)]


_vp, _i32, _dbl = C.c_void_p, C.c_int32, C.c_double
_lib.kv_metric_stream.restype = C.c_int
_lib.kv_metric_stream.argtypes = [_i32, _vp, _dbl, _dbl, _vp, _vp, _vp, _vp]
_lib.kv_metric_token_weight.restype = _dbl
_lib.kv_metric_token_weight.argtypes = [_dbl, _dbl, _dbl]
_lib.kv_metric_weight_sum.restype = C.c_int
_lib.kv_metric_weight_sum.argtypes = [_i32, _vp, _dbl, _dbl, _vp]
_lib.kv_metric_effective_sum.restype = C.c_int
_lib.kv_metric_effective_sum.argtypes = [_i32, _vp, _vp]
_lib.kv_metric_qos.restype = C.c_int
_lib.kv_metric_qos.argtypes = [_i32, _vp, _vp, _vp, _dbl, _dbl, _dbl, _vp]
_lib.kv_sched_step.restype = C.c_int
_lib.kv_sched_step.argtypes = [C.POINTER(kv_sched_config), _i32, _vp, _vp, _vp]


def _p(a):
    return a.ctypes.data_as(_vp)


def kv_metric_stream(t_gen, t_arrival, rate):
    """-> (rc, dict(buffer int32[L], t_read float64[L], ttft, rebuffer))"""
    t = np.ascontiguousarray(np.asarray(t_gen, dtype=np.float64))
    L = len(t)
    buf, rd = np.zeros(L, np.int32), np.zeros(L, np.float64)
    ttft, reb = _dbl(), _dbl()
    rc = _lib.kv_metric_stream(L, _p(t), float(t_arrival), float(rate), _p(buf), _p(rd), C.byref(ttft), C.byref(reb))
    return rc, dict(buffer=buf, t_read=rd, ttft=ttft.value, rebuffer=reb.value)


def kv_metric_token_weight(B, tau, alpha):
    return _lib.kv_metric_token_weight(float(B), float(tau), float(alpha))


def kv_metric_weight_sum(buffer, tau, alpha):
    b = np.ascontiguousarray(np.asarray(buffer, dtype=np.int32))
    s = _dbl()
    rc = _lib.kv_metric_weight_sum(len(b), _p(b), float(tau), float(alpha), C.byref(s))
    return rc, s.value


def kv_metric_effective_sum(buffer):
    b = np.ascontiguousarray(np.asarray(buffer, dtype=np.int32))
    s = _dbl()
    rc = _lib.kv_metric_effective_sum(len(b), _p(b), C.byref(s))
    return rc, s.value


def kv_metric_qos(weight_sum, ttft, rebuffer, lam, mu, T):
    w, t, r = (np.ascontiguousarray(np.asarray(x, dtype=np.float64)) for x in (weight_sum, ttft, rebuffer))
    if not (len(w) == len(t) == len(r)):
        return KVS_EINVAL, 0.0
    q = _dbl()
    rc = _lib.kv_metric_qos(len(w), _p(w), _p(t), _p(r), float(lam), float(mu), float(T), C.byref(q))
    return rc, q.value


def make_config(**kw):
    cfg = kv_sched_config()
    cfg.struct_size = C.sizeof(kv_sched_config)
    for k, v in kw.items():
        setattr(cfg, k, v)
    return cfg


def kv_sched_step(cfg, reqs):
    """reqs: list of dicts with the kv_sched_req fields -> (rc, mode, list of dicts with the kv_sched_out fields)"""
    n = len(reqs)
    arr = (kv_sched_req * max(n, 1))()
    for i, r in enumerate(reqs):
        for k, _ in kv_sched_req._fields_:
            setattr(arr[i], k, r[k])
    out = (kv_sched_out * max(n, 1))()
    mode = _i32(-1)
    rc = _lib.kv_sched_step(C.byref(cfg), n, C.cast(arr, _vp), C.cast(out, _vp), C.byref(mode))
    res = [{k: getattr(out[i], k) for k, _ in kv_sched_out._fields_} for i in range(n)]
    return rc, mode.value, res
