"""ctypes binding of libkvswap.so, the C-ABI library declared in include/kvswap.h.

Argument marshalling only: every byte is moved by the HIP kernels / HIP copies
inside the library.  The functions carry the names of the C entry points; the
`KVPool` class bundles a handle with the tensors it points into so that they
stay alive.  There is no fallback: importing this module without a built
library raises.
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  -- first, so that the library binds to the HIP runtime torch has loaded:
#                               two runtimes in one process do not see each other's allocations

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvswap.so")

KV_OK, KV_EINVAL, KV_ERANGE, KV_EDUP, KV_ENOENT = 0, -1, -2, -3, -4
KV_EEXIST, KV_ENOSPC, KV_EHIP, KV_ESTATE, KV_ENOMEM, KV_E2BIG = -5, -6, -7, -8, -9, -10
KV_NOALLOC_MAX_BLOCKS = 65536
KV_PATH_AUTO, KV_PATH_DMA, KV_PATH_ZEROCOPY, KV_STAGING_DEVICE, KV_PLAN_ONLY, KV_REQ_EVENTS = 0, 1, 2, 4, 8, 16
KV_DELTA_INCLUDE_TAIL = 1
KV_KEEP_STAGING = 1
KV_TUNE_MAX_WGS_DEVICE, KV_TUNE_MAX_WGS_LINK, KV_TUNE_KERNEL_VARIANT, KV_TUNE_DMA_SLICE_BLOCKS = 1, 2, 3, 4
KV_TUNE_SEGMENT_BYTES = 5
KV_TUNE_SCALE_LDS = 6
KV_TUNE_SEGMENT_MAX_BYTES = 7
KV_TUNE_SCATTER_ORDER = 8
KV_TUNE_PHASE_BYTES, KV_TUNE_PHASE_WGS_OUT, KV_TUNE_PHASE_WGS_IN = 9, 10, 11
KV_TUNE_KERNEL_EVENTS = 12
KV_TUNE_HOST_STORES = 13
KV_TUNE_LINK_IN_WGS, KV_TUNE_LINK_IN_UNROLL = 14, 15
KV_F16, KV_BF16, KV_FP8_E4M3 = 0, 1, 2

EXPORTS = ["kv_pool_create", "kv_pool_destroy", "kv_swap_out", "kv_swap_out_delta", "kv_swap_in", "kv_evict_and_load", "kv_sync",
           "kv_move_blocks", "kv_move_blocks_noalloc", "kv_req_reserve", "kv_req_release", "kv_req_query", "kv_last_stats",
           "kv_slot_bytes", "kv_last_plan", "kv_pool_tune", "kv_last_hip_error", "kv_strerror",
           "kv_io_stats_get", "kv_budget_blocks", "kv_req_poll", "kv_req_wait", "kv_last_timeline",
           "kv_swap_out_delta_timed", "kv_bench_copy", "kv_bench_copy_scrambled", "kv_bench_link", "kv_bench_link_bidir",
           "kv_wq_post", "kv_wq_drain", "kv_wq_remove", "kv_wq_pending"]


class kv_pool_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("num_layers", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("dtype", C.c_int32), ("num_blocks", C.c_int64),
                ("pool_dev", C.c_void_p),
                ("layer_stride", C.c_int64), ("kv_stride", C.c_int64), ("block_stride", C.c_int64),
                ("scale_dev", C.c_void_p),
                ("scale_layer_stride", C.c_int64), ("scale_kv_stride", C.c_int64),
                ("scale_block_stride", C.c_int64),
                ("staging_host", C.c_void_p), ("staging_bytes", C.c_int64),
                ("bounce_dev", C.c_void_p), ("bounce_bytes", C.c_int64),
                ("evict_stream", C.c_void_p), ("load_stream", C.c_void_p),
                ("flags", C.c_uint32)]


class kv_stats(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("op", C.c_int32), ("path", C.c_int32), ("launches", C.c_int32),
                ("copies", C.c_int32), ("grid", C.c_int32), ("blocks", C.c_int64), ("bytes", C.c_int64),
                ("plan_us", C.c_double), ("enqueue_us", C.c_double), ("ms_total", C.c_float),
                ("ms_kernel", C.c_float), ("scatter_order", C.c_int32), ("reserved", C.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_ if k not in ("struct_size", "reserved")}


class kv_io_stats(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("inflight_calls", C.c_int32 * 2), ("inflight_bytes", C.c_int64 * 2),
                ("total_calls", C.c_int64 * 2), ("total_bytes", C.c_int64 * 2), ("ewma_gbps", C.c_double * 2),
                ("ewma_small_us", C.c_double * 2)]

    def as_dict(self):
        return {k: list(getattr(self, k)) for k, _ in self._fields_ if k != "struct_size"}


if not os.path.exists(LIB_PATH):
    raise ImportError("libkvswap.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(hipcc --offload-arch=gfx950) first; there is no fallback path")
_lib = C.CDLL(LIB_PATH)

_vp, _i32, _i64, _u32, _u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64
_sig = {
    "kv_pool_create": (C.c_int, [C.POINTER(kv_pool_config), C.POINTER(_vp)]),
    "kv_pool_destroy": (C.c_int, [_vp]),
    "kv_swap_out": (C.c_int, [_vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "kv_swap_out_delta": (C.c_int, [_vp, _i32, _vp, _vp, _vp, _vp, _i64, _u32, _vp, _vp]),
    "kv_swap_out_delta_timed": (C.c_int, [_vp, _i32, _vp, _vp, _vp, _vp, _vp, C.c_double, _u32, _vp, _vp, _vp]),
    "kv_swap_in": (C.c_int, [_vp, _i32, _vp, _vp, _vp, _u32, _vp]),
    "kv_evict_and_load": (C.c_int, [_vp, _i32, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _u32, _vp]),
    "kv_sync": (C.c_int, [_vp]),
    "kv_move_blocks": (C.c_int, [_vp, _i64, _vp, _vp, _vp]),
    "kv_move_blocks_noalloc": (C.c_int, [_vp, _i64, _vp, _vp, _vp]),
    "kv_req_reserve": (C.c_int, [_vp, _u64, _i32]),
    "kv_req_release": (C.c_int, [_vp, _u64]),
    "kv_req_query": (C.c_int, [_vp, _u64, _vp, _vp, _vp, _vp, _vp]),
    "kv_last_stats": (C.c_int, [_vp, C.POINTER(kv_stats)]),
    "kv_slot_bytes": (_i64, [_vp]),
    "kv_last_plan": (_i64, [_vp, _vp, _vp, _i64]),
    "kv_pool_tune": (C.c_int, [_vp, _i32, _i64]),
    "kv_last_hip_error": (C.c_int, [_vp]),
    "kv_strerror": (C.c_char_p, [C.c_int]),
    "kv_req_poll": (C.c_int, [_vp, _u64]),
    "kv_req_wait": (C.c_int, [_vp, _u64]),
    "kv_last_timeline": (_i64, [_vp, _vp, _vp, _i64]),
    "kv_io_stats_get": (C.c_int, [_vp, C.POINTER(kv_io_stats)]),
    "kv_budget_blocks": (_i64, [_vp, _i32, C.c_double]),
    "kv_bench_copy": (C.c_double, [_vp, _vp, _i64, _i32, _i32, _vp]),
    "kv_bench_copy_scrambled": (C.c_double, [_vp, _vp, _i64, _i64, _i32, _i32, _vp]),
    "kv_bench_link": (C.c_double, [_vp, _vp, _i64, _i32, _i32, _vp]),
    "kv_bench_link_bidir": (C.c_double, [_vp, _vp, _vp, _vp, _i64, _i32]),
    "kv_wq_post": (C.c_int, [_vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "kv_wq_drain": (C.c_int, [_vp, C.c_double, _i64, _u32, _vp, _vp, _vp, _vp]),
    "kv_wq_remove": (C.c_int, [_vp, _u64]),
    "kv_wq_pending": (C.c_int, [_vp, _vp, _vp]),
}
for _name, (_res, _args) in _sig.items():
    _f = getattr(_lib, _name)
    _f.restype, _f.argtypes = _res, _args


def _p(a):
    return None if a is None else a.ctypes.data_as(_vp)


def _i32a(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _u64a(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint64))


def _csr_ok(n, offsets, block_ids, *per_request):
    """The C side trusts the array lengths the CSR implies: check them here, where they are known."""
    if len(offsets) != n + 1 or any(len(a) != n for a in per_request):
        return False
    return n == 0 or int(offsets.max()) <= len(block_ids)


def kv_strerror(code):
    return _lib.kv_strerror(int(code)).decode()


def kv_pool_create(cfg):
    """cfg: kv_pool_config -> (rc, handle)"""
    cfg.struct_size = C.sizeof(kv_pool_config)
    h = _vp()
    rc = _lib.kv_pool_create(C.byref(cfg), C.byref(h))
    return rc, h


def kv_pool_destroy(h):
    return _lib.kv_pool_destroy(h)


def kv_swap_out(h, req_ids, offsets, block_ids, num_tokens, wait_event=None):
    r, o, b, t = _u64a(req_ids), _i32a(offsets), _i32a(block_ids), _i32a(num_tokens)
    if not _csr_ok(len(r), o, b, t):
        return KV_EINVAL
    return _lib.kv_swap_out(h, len(r), _p(r), _p(o), _p(b), _p(t), wait_event)


def kv_swap_out_delta(h, req_ids, offsets, block_ids, num_tokens, block_budget=0, flags=0, wait_event=None):
    """-> (rc, blocks_moved int32[n])"""
    r, o, b, t = _u64a(req_ids), _i32a(offsets), _i32a(block_ids), _i32a(num_tokens)
    moved = np.zeros(len(r), dtype=np.int32)
    if not _csr_ok(len(r), o, b, t):
        return KV_EINVAL, moved
    rc = _lib.kv_swap_out_delta(h, len(r), _p(r), _p(o), _p(b), _p(t), int(block_budget), int(flags),
                                _p(moved), wait_event)
    return rc, moved


def kv_swap_out_delta_timed(h, req_ids, offsets, block_ids, num_tokens, priority, interval_us, flags=0,
                            wait_event=None):
    """-> (rc, blocks_moved int32[n] in the caller's order, budget applied)"""
    r, o, b, t = _u64a(req_ids), _i32a(offsets), _i32a(block_ids), _i32a(num_tokens)
    pr = None if priority is None else np.ascontiguousarray(np.asarray(priority, dtype=np.float32))
    moved = np.zeros(len(r), dtype=np.int32)
    if not _csr_ok(len(r), o, b, t) or (pr is not None and len(pr) != len(r)):
        return KV_EINVAL, moved, 0
    used = _i64(0)
    rc = _lib.kv_swap_out_delta_timed(h, len(r), _p(r), _p(o), _p(b), _p(t), _p(pr), float(interval_us), int(flags),
                                      _p(moved), C.byref(used), wait_event)
    return rc, moved, used.value


def kv_wq_post(h, req_ids, offsets, block_ids, num_tokens, priority=None):
    r, o, b, t = _u64a(req_ids), _i32a(offsets), _i32a(block_ids), _i32a(num_tokens)
    pr = None if priority is None else np.ascontiguousarray(np.asarray(priority, dtype=np.float64))
    if not _csr_ok(len(r), o, b, t) or (pr is not None and len(pr) != len(r)):
        return KV_EINVAL
    return _lib.kv_wq_post(h, len(r), _p(r), _p(o), _p(b), _p(t), _p(pr))


def kv_wq_drain(h, interval_us=0.0, block_budget=0, flags=0, wait_event=None):
    """-> (rc, blocks written, full blocks still pending, budget applied)"""
    w, pend, used = _i64(0), _i64(0), _i64(0)
    rc = _lib.kv_wq_drain(h, float(interval_us), int(block_budget), int(flags), C.byref(w), C.byref(pend),
                          C.byref(used), wait_event)
    return rc, w.value, pend.value, used.value


def kv_wq_remove(h, req_id):
    return _lib.kv_wq_remove(h, int(req_id))


def kv_wq_pending(h):
    """-> (rc, full blocks not yet written through, requests that have some)"""
    nb, nr = _i64(0), _i32(0)
    rc = _lib.kv_wq_pending(h, C.byref(nb), C.byref(nr))
    return rc, nb.value, nr.value


def kv_swap_in(h, req_ids, offsets, new_block_ids, flags=0, wait_event=None):
    r, o, b = _u64a(req_ids), _i32a(offsets), _i32a(new_block_ids)
    if not _csr_ok(len(r), o, b):
        return KV_EINVAL
    return _lib.kv_swap_in(h, len(r), _p(r), _p(o), _p(b), int(flags), wait_event)


def kv_evict_and_load(h, out_ids, out_offsets, out_block_ids, out_tokens, in_ids, in_offsets, in_block_ids, in_flags=0,
                      wait_event=None):
    r, o, b, t = _u64a(out_ids), _i32a(out_offsets), _i32a(out_block_ids), _i32a(out_tokens)
    r2, o2, b2 = _u64a(in_ids), _i32a(in_offsets), _i32a(in_block_ids)
    if not _csr_ok(len(r), o, b, t) or not _csr_ok(len(r2), o2, b2):
        return KV_EINVAL
    return _lib.kv_evict_and_load(h, len(r), _p(r), _p(o), _p(b), _p(t), len(r2), _p(r2), _p(o2), _p(b2), int(in_flags),
                                  wait_event)


def kv_sync(h):
    return _lib.kv_sync(h)


def kv_move_blocks(h, src_ids, dst_ids, wait_event=None):
    s, d = _i32a(src_ids), _i32a(dst_ids)
    if len(s) != len(d):
        return KV_EINVAL
    return _lib.kv_move_blocks(h, len(s), _p(s), _p(d), wait_event)


def kv_move_blocks_noalloc(h, src_ids, dst_ids, wait_event=None):
    s, d = _i32a(src_ids), _i32a(dst_ids)
    if len(s) != len(d):
        return KV_EINVAL
    return _lib.kv_move_blocks_noalloc(h, len(s), _p(s), _p(d), wait_event)


def kv_req_reserve(h, req_id, max_blocks):
    return _lib.kv_req_reserve(h, int(req_id), int(max_blocks))


def kv_req_release(h, req_id):
    return _lib.kv_req_release(h, int(req_id))


def kv_req_query(h, req_id):
    """-> (rc, dict(offset, cap, staged, wm, swapped))"""
    off = _i64()
    cap, st, wm, sw = _i32(), _i32(), _i32(), _i32()
    rc = _lib.kv_req_query(h, int(req_id), C.byref(off), C.byref(cap), C.byref(st), C.byref(wm), C.byref(sw))
    return rc, dict(offset=off.value, cap=cap.value, staged=st.value, wm=wm.value, swapped=sw.value)


def kv_last_stats(h):
    st = kv_stats()
    st.struct_size = C.sizeof(kv_stats)
    rc = _lib.kv_last_stats(h, C.byref(st))
    return rc, st.as_dict()


def kv_slot_bytes(h):
    return _lib.kv_slot_bytes(h)


def kv_last_plan(h):
    """-> (phys int32[n], slot int64[n]) of the most recent swap call"""
    n = _lib.kv_last_plan(h, None, None, 0)
    phys, slot = np.zeros(n, np.int32), np.zeros(n, np.int64)
    if n:
        _lib.kv_last_plan(h, _p(phys), _p(slot), n)
    return phys, slot


def kv_req_poll(h, req_id):
    return _lib.kv_req_poll(h, int(req_id))


def kv_req_wait(h, req_id):
    return _lib.kv_req_wait(h, int(req_id))


def kv_last_timeline(h):
    """-> (req_ids uint64[n], done_ms float32[n]) of the most recent swap call"""
    n = _lib.kv_last_timeline(h, None, None, 0)
    if n < 0:
        raise KVSwapError(n, "kv_last_timeline")
    ids, ms = np.zeros(n, np.uint64), np.zeros(n, np.float32)
    if n:
        _lib.kv_last_timeline(h, _p(ids), _p(ms), n)
    return ids, ms


def kv_io_stats_get(h):
    """-> (rc, dict of 2-element lists: index 0 evict stream, 1 load stream)"""
    st = kv_io_stats()
    rc = _lib.kv_io_stats_get(h, C.byref(st))
    return rc, st.as_dict()


def kv_budget_blocks(h, direction, interval_us):
    return _lib.kv_budget_blocks(h, int(direction), float(interval_us))


def kv_pool_tune(h, what, value):
    return _lib.kv_pool_tune(h, int(what), int(value))


def kv_last_hip_error(h):
    return _lib.kv_last_hip_error(h)


def kv_bench_copy(dst_ptr, src_ptr, nbytes, grid, iters, stream=None):
    return _lib.kv_bench_copy(dst_ptr, src_ptr, int(nbytes), int(grid), int(iters), stream)


def kv_bench_copy_scrambled(dst_ptr, src_ptr, nbytes, chunk_bytes, which, iters, stream=None):
    return _lib.kv_bench_copy_scrambled(dst_ptr, src_ptr, int(nbytes), int(chunk_bytes), int(which), int(iters), stream)


def kv_bench_link(host_ptr, dev_ptr, nbytes, direction, iters, stream=None):
    return _lib.kv_bench_link(host_ptr, dev_ptr, int(nbytes), int(direction), int(iters), stream)


def kv_bench_link_bidir(host_a, dev_a, host_b, dev_b, nbytes, iters):
    return _lib.kv_bench_link_bidir(host_a, dev_a, host_b, dev_b, int(nbytes), int(iters))


class KVSwapError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s: %s (%d)" % (what, kv_strerror(code), code))
        self.code = code


class KVPool:
    """A handle plus references to the memory it points into.

    pool / scale / bounce are torch uint8 device tensors, staging a pinned uint8
    host tensor (or a device tensor with KV_STAGING_DEVICE); under KV_PLAN_ONLY
    all of them may be None.  Strides default to the layer-major layout.
    """

    def __init__(self, geom, pool=None, staging=None, scale=None, bounce=None, strides=None, scale_strides=None,
                 flags=0, evict_stream=None, load_stream=None, staging_bytes=None, dtype_code=None):
        from .workloads import DTYPE_CODE
        self.geom = geom
        self._keep = (pool, staging, scale, bounce, evict_stream, load_stream)
        cfg = kv_pool_config()
        cfg.num_layers, cfg.num_kv_heads, cfg.head_dim, cfg.block_size = geom.L, geom.H, geom.D, geom.B
        cfg.dtype = DTYPE_CODE[geom.dtype] if dtype_code is None else dtype_code
        cfg.num_blocks = geom.N
        cfg.pool_dev = pool.data_ptr() if pool is not None else None
        cfg.layer_stride, cfg.kv_stride, cfg.block_stride = strides or geom.strides
        if geom.scales:
            cfg.scale_dev = scale.data_ptr() if scale is not None else None
            cfg.scale_layer_stride, cfg.scale_kv_stride, cfg.scale_block_stride = scale_strides or geom.scale_strides
        cfg.staging_host = staging.data_ptr() if staging is not None else None
        cfg.staging_bytes = staging.numel() if staging is not None else int(staging_bytes or 0)
        cfg.bounce_dev = bounce.data_ptr() if bounce is not None else None
        cfg.bounce_bytes = bounce.numel() if bounce is not None else 0
        cfg.evict_stream = evict_stream.cuda_stream if evict_stream is not None else None
        cfg.load_stream = load_stream.cuda_stream if load_stream is not None else None
        cfg.flags = flags
        rc, self.h = kv_pool_create(cfg)
        if rc:
            self.h = None
            raise KVSwapError(rc, "kv_pool_create")
        self.slot_bytes = kv_slot_bytes(self.h)

    def close(self):
        if getattr(self, "h", None):
            rc = kv_pool_destroy(self.h)
            self.h = None
            return rc
        return KV_OK

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False

    # thin pass-throughs returning the C status codes
    def swap_out(self, req_ids, offsets, block_ids, num_tokens, wait_event=None):
        return kv_swap_out(self.h, req_ids, offsets, block_ids, num_tokens, wait_event)

    def swap_out_delta(self, req_ids, offsets, block_ids, num_tokens, budget=0, flags=0, wait_event=None):
        return kv_swap_out_delta(self.h, req_ids, offsets, block_ids, num_tokens, budget, flags, wait_event)

    def swap_out_delta_timed(self, req_ids, offsets, block_ids, num_tokens, priority, interval_us, flags=0,
                             wait_event=None):
        return kv_swap_out_delta_timed(self.h, req_ids, offsets, block_ids, num_tokens, priority, interval_us, flags,
                                       wait_event)

    def wq_post(self, req_ids, offsets, block_ids, num_tokens, priority=None):
        return kv_wq_post(self.h, req_ids, offsets, block_ids, num_tokens, priority)

    def wq_drain(self, interval_us=0.0, block_budget=0, flags=0, wait_event=None):
        return kv_wq_drain(self.h, interval_us, block_budget, flags, wait_event)

    def wq_remove(self, req_id):
        return kv_wq_remove(self.h, req_id)

    def wq_pending(self):
        return kv_wq_pending(self.h)

    def swap_in(self, req_ids, offsets, new_block_ids, flags=0, wait_event=None):
        return kv_swap_in(self.h, req_ids, offsets, new_block_ids, flags, wait_event)

    def move_blocks(self, src_ids, dst_ids, wait_event=None):
        return kv_move_blocks(self.h, src_ids, dst_ids, wait_event)

    def move_blocks_noalloc(self, src_ids, dst_ids, wait_event=None):
        return kv_move_blocks_noalloc(self.h, src_ids, dst_ids, wait_event)

    def evict_and_load(self, out_ids, out_offsets, out_block_ids, out_tokens, in_ids, in_offsets, in_block_ids, in_flags=0,
                       wait_event=None):
        return kv_evict_and_load(self.h, out_ids, out_offsets, out_block_ids, out_tokens, in_ids, in_offsets,
                                 in_block_ids, in_flags, wait_event)

    def sync(self):
        return kv_sync(self.h)

    def reserve(self, req_id, max_blocks):
        return kv_req_reserve(self.h, req_id, max_blocks)

    def release(self, req_id):
        return kv_req_release(self.h, req_id)

    def query(self, req_id):
        return kv_req_query(self.h, req_id)

    def stats(self):
        rc, st = kv_last_stats(self.h)
        if rc:
            raise KVSwapError(rc, "kv_last_stats")
        return st

    def last_plan(self):
        return kv_last_plan(self.h)

    def req_poll(self, req_id):
        return kv_req_poll(self.h, req_id)

    def req_wait(self, req_id):
        return kv_req_wait(self.h, req_id)

    def timeline(self):
        return kv_last_timeline(self.h)

    def io_stats(self):
        rc, st = kv_io_stats_get(self.h)
        if rc:
            raise KVSwapError(rc, "kv_io_stats_get")
        return st

    def budget_blocks(self, direction, interval_us):
        return kv_budget_blocks(self.h, direction, interval_us)

    def tune(self, what, value):
        return kv_pool_tune(self.h, what, value)
