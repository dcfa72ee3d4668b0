"""ctypes loader for the CPU oracle (kv_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  It holds no arithmetic of its own: it compiles kv_oracle.c with
gcc when the shared object is missing or older than its source, and marshals
numpy arrays into the C calls.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kv_oracle.c")
_HDR = os.path.join(_HERE, "kv_oracle.h")
_LIB = os.path.join(_HERE, "libkv_oracle.so")

OK, EINVAL, ERANGE, EDUP, ENOENT, EEXIST, ENOSPC, ESTATE = 0, -1, -2, -3, -4, -5, -6, -8
DELTA_INCLUDE_TAIL = 1
KEEP_STAGING = 1


def build(force=False):
    """Compile kv_oracle.c -> libkv_oracle.so with plain gcc -O2."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("L", C.c_int32), ("H", C.c_int32), ("D", C.c_int32), ("B", C.c_int32),
                ("elem_bytes", C.c_int32), ("N", C.c_int64),
                ("pool", C.c_void_p),
                ("layer_stride", C.c_int64), ("kv_stride", C.c_int64), ("block_stride", C.c_int64),
                ("scale", C.c_void_p),
                ("s_layer_stride", C.c_int64), ("s_kv_stride", C.c_int64), ("s_block_stride", C.c_int64),
                ("staging", C.c_void_p), ("staging_bytes", C.c_int64)]


_lib = None


def _load(path=None):
    """Load (and cache) the oracle library; `path` loads another build of it uncached."""
    global _lib
    if path is None and _lib is not None:
        return _lib
    lib = C.CDLL(path or build())
    vp, i32, i64, u32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64
    lib.ora_create.restype = vp
    lib.ora_create.argtypes = [C.POINTER(_Cfg)]
    lib.ora_destroy.restype = None
    lib.ora_destroy.argtypes = [vp]
    lib.ora_slot_bytes.restype = i64
    lib.ora_slot_bytes.argtypes = [vp]
    lib.ora_swap_out.restype = C.c_int
    lib.ora_swap_out.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.ora_swap_out_delta.restype = C.c_int
    lib.ora_swap_out_delta.argtypes = [vp, i32, vp, vp, vp, vp, i64, u32, vp]
    lib.ora_swap_in.restype = C.c_int
    lib.ora_swap_in.argtypes = [vp, i32, vp, vp, vp, u32]
    lib.ora_move_blocks.restype = C.c_int
    lib.ora_move_blocks.argtypes = [vp, i64, vp, vp]
    lib.ora_req_reserve.restype = C.c_int
    lib.ora_req_reserve.argtypes = [vp, u64, i32]
    lib.ora_req_release.restype = C.c_int
    lib.ora_req_release.argtypes = [vp, u64]
    lib.ora_req_query.restype = C.c_int
    lib.ora_req_query.argtypes = [vp, u64, vp, vp, vp, vp, vp]
    if path is None:
        _lib = lib
    return lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _u64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint64))


def _csr_ok(n, offsets, block_ids, *per_request):
    if len(offsets) != n + 1 or any(len(a) != n for a in per_request):
        return False
    return n == 0 or int(offsets.max()) <= len(block_ids)


class Oracle:
    """Host-memory KV pool + staging arena driven by the C oracle.

    pool, scale (or None) and staging are 1-D uint8 numpy arrays owned by the
    caller; the oracle reads and writes them in place.
    """

    def __init__(self, L, H, D, B, elem_bytes, N, pool, strides, staging, scale=None, scale_strides=None,
                 lib=None):
        lib = self._lib = lib or _load()
        for a in (pool, staging) + ((scale,) if scale is not None else ()):
            assert a.dtype == np.uint8 and a.ndim == 1 and a.flags["C_CONTIGUOUS"]
        self.pool, self.staging, self.scale = pool, staging, scale
        cfg = _Cfg()
        cfg.L, cfg.H, cfg.D, cfg.B, cfg.elem_bytes, cfg.N = L, H, D, B, elem_bytes, N
        cfg.pool = pool.ctypes.data
        cfg.layer_stride, cfg.kv_stride, cfg.block_stride = strides
        cfg.scale = scale.ctypes.data if scale is not None else None
        if scale is not None:
            cfg.s_layer_stride, cfg.s_kv_stride, cfg.s_block_stride = scale_strides
        cfg.staging = staging.ctypes.data
        cfg.staging_bytes = staging.nbytes
        self._h = lib.ora_create(C.byref(cfg))
        if not self._h:
            raise ValueError("ora_create rejected the configuration")
        self.slot_bytes = lib.ora_slot_bytes(self._h)

    def close(self):
        if self._h:
            self._lib.ora_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def swap_out(self, req_ids, offsets, block_ids, num_tokens):
        r, o, b, t = _u64(req_ids), _i32(offsets), _i32(block_ids), _i32(num_tokens)
        if not _csr_ok(len(r), o, b, t):
            return EINVAL
        return self._lib.ora_swap_out(self._h, len(r), _ptr(r), _ptr(o), _ptr(b), _ptr(t))

    def swap_out_delta(self, req_ids, offsets, block_ids, num_tokens, budget=0, flags=0):
        r, o, b, t = _u64(req_ids), _i32(offsets), _i32(block_ids), _i32(num_tokens)
        moved = np.zeros(len(r), dtype=np.int32)
        if not _csr_ok(len(r), o, b, t):
            return EINVAL, moved
        rc = self._lib.ora_swap_out_delta(self._h, len(r), _ptr(r), _ptr(o), _ptr(b), _ptr(t),
                                        int(budget), int(flags), _ptr(moved))
        return rc, moved

    def swap_in(self, req_ids, offsets, new_block_ids, flags=0):
        r, o, b = _u64(req_ids), _i32(offsets), _i32(new_block_ids)
        if not _csr_ok(len(r), o, b):
            return EINVAL
        return self._lib.ora_swap_in(self._h, len(r), _ptr(r), _ptr(o), _ptr(b), int(flags))

    def move_blocks(self, src_ids, dst_ids):
        s, d = _i32(src_ids), _i32(dst_ids)
        assert len(s) == len(d)
        return self._lib.ora_move_blocks(self._h, len(s), _ptr(s), _ptr(d))

    def reserve(self, req_id, max_blocks):
        return self._lib.ora_req_reserve(self._h, int(req_id), int(max_blocks))

    def release(self, req_id):
        return self._lib.ora_req_release(self._h, int(req_id))

    def query(self, req_id):
        """-> (rc, dict(offset, cap, staged, wm, swapped))"""
        off = C.c_int64()
        cap, st, wm, sw = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
        rc = self._lib.ora_req_query(self._h, int(req_id), C.byref(off), C.byref(cap), C.byref(st),
                                   C.byref(wm), C.byref(sw))
        return rc, dict(offset=off.value, cap=cap.value, staged=st.value, wm=wm.value, swapped=sw.value)
