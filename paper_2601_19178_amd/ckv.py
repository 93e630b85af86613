"""Thin ctypes binding of libckv.so: same names as include/ckv.h, argument marshalling only.

Device arguments may be torch tensors (their data_ptr() is passed), ints (raw device
addresses) or None.  Host arguments are numpy arrays.  There is no fallback: if the library
is missing, import fails with the build command to run.
"""
import ctypes
import os

import numpy as np
import torch  # noqa: F401  -- must come first: libckv.so has to bind to the HIP runtime torch ships,
#                              or torch's device pointers and streams would belong to another runtime.

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "libckv.so")

CKV_F32, CKV_BF16 = 0, 1
CKV_SOFTMAX, CKV_SILU_OVER_N = 0, 1
CKV_SHARE_KV, CKV_SHARE_K, CKV_SHARE_V = 0, 1, 2
CKV_OK, CKV_ERR_NULL, CKV_ERR_SHAPE, CKV_ERR_INDEX, CKV_ERR_LENGTH, CKV_ERR_UNSUPPORTED, CKV_ERR_HIP = 0, -1, -2, -3, -4, -5, -6

EXPORTS = [
    "ckv_build_cache", "ckv_build_cache_offloaded", "ckv_cache_is_offloaded", "ckv_prefill", "ckv_prefill_into",
    "ckv_cache_prefill_workspace", "ckv_prefill_kernel_name", "ckv_plan", "ckv_remap_hot_rows", "ckv_cache_idx", "ckv_cache_user_k", "ckv_cache_user_v", "ckv_cache_lengths",
    "ckv_cache_positions", "ckv_cache_stored_bytes", "ckv_attend", "ckv_reconstruct", "ckv_free",
    "ckv_last_error", "ckv_set_timing", "ckv_kernel_ms", "ckv_kernel_times", "ckv_variant", "ckv_copy", "ckv_trace_enable",
    "ckv_trace_read", "ckv_set_option", "ckv_attend_static_scratch",
]
CKV_STATIC_SCRATCH_BYTES = 32 << 20


class ckv_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d_g", ctypes.c_int32), ("d_u", ctypes.c_int32),
                ("P", ctypes.c_int32), ("Nq", ctypes.c_int32), ("dtype", ctypes.c_int32), ("mode", ctypes.c_int32),
                ("scale", ctypes.c_float), ("share", ctypes.c_int32), ("pool_ld", ctypes.c_int64)]


class ckv_router(ctypes.Structure):
    _fields_ = [("d_e", ctypes.c_int32), ("reserved", ctypes.c_int32)] + [
        (n, ctypes.c_void_p) for n in ("w_rk", "b_rk", "w_rv", "b_rv", "w_k", "b_k", "w_v", "b_v")]


class CkvError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"ckv error {code}: {message}")
        self.code = code


if not os.path.exists(_LIBPATH):
    raise ImportError(f"{_LIBPATH} is not built; run `python -m paper_2601_19178_amd.build` "
                      "(hipcc, gfx950). There is no CPU fallback.")
_lib = ctypes.CDLL(_LIBPATH)

_vp, _i32, _i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
_lib.ckv_build_cache.restype = ctypes.c_int
_lib.ckv_build_cache.argtypes = [ctypes.POINTER(ckv_shape), _vp, _vp, _vp, _vp, _vp, ctypes.POINTER(_vp), _vp]
_lib.ckv_build_cache_offloaded.restype = ctypes.c_int
_lib.ckv_build_cache_offloaded.argtypes = _lib.ckv_build_cache.argtypes
_lib.ckv_prefill.restype = ctypes.c_int
_lib.ckv_prefill.argtypes = [ctypes.POINTER(ckv_shape), ctypes.POINTER(ckv_router), _vp, _vp, ctypes.POINTER(_vp), _vp]
_lib.ckv_prefill_into.restype = ctypes.c_int
_lib.ckv_cache_prefill_workspace.restype = ctypes.c_int64
_lib.ckv_cache_prefill_workspace.argtypes = [_vp]
_lib.ckv_prefill_into.argtypes = [_vp, ctypes.POINTER(ckv_router), _vp, _vp]
_lib.ckv_prefill_kernel_name.restype = ctypes.c_char_p
_lib.ckv_prefill_kernel_name.argtypes = [ctypes.POINTER(ckv_shape), ctypes.POINTER(ckv_router)]
_lib.ckv_remap_hot_rows.restype = ctypes.c_int
_lib.ckv_remap_hot_rows.argtypes = [_vp] * 7
_lib.ckv_plan.restype = _i64
_lib.ckv_plan.argtypes = [ctypes.POINTER(ckv_shape), _vp, ctypes.c_int, ctypes.c_int, _vp, _i64, ctypes.POINTER(_i32), ctypes.c_char_p,
                          ctypes.c_size_t]
_lib.ckv_cache_is_offloaded.restype = ctypes.c_int
_lib.ckv_cache_is_offloaded.argtypes = [_vp]
for _n in ("ckv_cache_idx", "ckv_cache_user_k", "ckv_cache_user_v", "ckv_cache_lengths"):
    getattr(_lib, _n).restype = _vp
    getattr(_lib, _n).argtypes = [_vp]
_lib.ckv_cache_positions.restype = _i64
_lib.ckv_cache_positions.argtypes = [_vp]
_lib.ckv_cache_stored_bytes.restype = _i64
_lib.ckv_cache_stored_bytes.argtypes = [_vp]
_lib.ckv_attend.restype = ctypes.c_int
_lib.ckv_attend.argtypes = [_vp] * 10
_lib.ckv_attend_static_scratch.restype = ctypes.c_int
_lib.ckv_attend_static_scratch.argtypes = [_vp] * 10
_lib.ckv_set_option.restype = ctypes.c_int
_lib.ckv_set_option.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
_lib.ckv_kernel_times.restype = ctypes.c_int
_lib.ckv_kernel_times.argtypes = [_vp, _vp, _vp, ctypes.c_int]
_lib.ckv_reconstruct.restype = ctypes.c_int
_lib.ckv_reconstruct.argtypes = [_vp] * 6
_lib.ckv_free.restype = None
_lib.ckv_free.argtypes = [_vp]
_lib.ckv_last_error.restype = ctypes.c_char_p
_lib.ckv_last_error.argtypes = []
_lib.ckv_set_timing.restype = ctypes.c_int
_lib.ckv_set_timing.argtypes = [_vp, ctypes.c_int]
_lib.ckv_kernel_ms.restype = ctypes.c_float
_lib.ckv_kernel_ms.argtypes = [_vp]
_lib.ckv_variant.restype = ctypes.c_char_p
_lib.ckv_variant.argtypes = [_vp]
_lib.ckv_trace_enable.restype = ctypes.c_int
_lib.ckv_trace_enable.argtypes = [_vp, ctypes.c_int]
_lib.ckv_trace_read.restype = _i64
_lib.ckv_trace_read.argtypes = [_vp, _vp, _i64]
_lib.ckv_copy.restype = ctypes.c_int
_lib.ckv_copy.argtypes = [_vp, _vp, ctypes.c_size_t, _vp]


def _dev(x):
    """torch tensor | int | None -> c_void_p of a device address."""
    if x is None:
        return _vp(0)
    if isinstance(x, int):
        return _vp(x)
    return _vp(x.data_ptr())


def _host(a, dtype=None):
    if a is None:
        return None, _vp(0)
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a, _vp(a.ctypes.data)


def _check(rc):
    if rc != CKV_OK:
        raise CkvError(rc, ckv_last_error())


def ckv_last_error():
    return _lib.ckv_last_error().decode()


def make_shape(B, H, d_g, d_u, P, Nq, dtype, mode, scale, pool_ld, share=CKV_SHARE_KV):
    return ckv_shape(B, H, d_g, d_u, P, Nq, dtype, mode, scale, share, pool_ld)


def ckv_build_cache(shape, lengths, idx_k, idx_v, user_k, user_v, stream=0):
    """Host arrays in, opaque handle (int address) out."""
    keep = [_host(lengths, np.int32), _host(idx_k, np.int32), _host(idx_v, np.int32), _host(user_k), _host(user_v)]
    out = _vp(0)
    _check(_lib.ckv_build_cache(ctypes.byref(shape), *[p for _, p in keep], ctypes.byref(out), _vp(stream)))
    return out.value


def ckv_build_cache_offloaded(shape, lengths, idx_k, idx_v, user_k, user_v, stream=0):
    """As ckv_build_cache, but the packed cache stays in pinned host memory."""
    keep = [_host(lengths, np.int32), _host(idx_k, np.int32), _host(idx_v, np.int32), _host(user_k), _host(user_v)]
    out = _vp(0)
    _check(_lib.ckv_build_cache_offloaded(ctypes.byref(shape), *[p for _, p in keep], ctypes.byref(out), _vp(stream)))
    return out.value


def make_router(d_e, w_rk, b_rk, w_rv, b_rv, w_k, b_k, w_v, b_v):
    """Device tensors (or addresses, or None) -> ckv_router."""
    return ckv_router(d_e, 0, *[_dev(x).value for x in (w_rk, b_rk, w_rv, b_rv, w_k, b_k, w_v, b_v)])


def ckv_prefill(shape, router, lengths, S, stream=0):
    """Router and projection over the device embedding S; returns a new handle (int address)."""
    keep = _host(lengths, np.int32)
    out = _vp(0)
    _check(_lib.ckv_prefill(ctypes.byref(shape), ctypes.byref(router), keep[1], _dev(S), ctypes.byref(out), _vp(stream)))
    return out.value


def ckv_prefill_into(cache, router, S, stream=0):
    _check(_lib.ckv_prefill_into(cache, ctypes.byref(router), _dev(S), _vp(stream)))


def ckv_cache_prefill_workspace(cache):
    return int(_lib.ckv_cache_prefill_workspace(cache))


def ckv_prefill_kernel_name(shape, router):
    return _lib.ckv_prefill_kernel_name(ctypes.byref(shape), ctypes.byref(router)).decode()


def ckv_plan(shape, lengths, cus=256, wg_per_cu=2):
    """Host only: (records int64 [n][8], number of workgroups, kernel name) of the work lists for this shape."""
    keep = _host(lengths, np.int32)
    nwg = _i32(0)
    name = ctypes.create_string_buffer(96)
    n = _lib.ckv_plan(ctypes.byref(shape), keep[1], cus, wg_per_cu, _vp(0), 0, ctypes.byref(nwg), name, 96)
    if n < 0:
        raise CkvError(int(n), ckv_last_error())
    rec = np.zeros((max(int(n), 1), 8), dtype=np.int64)
    n = _lib.ckv_plan(ctypes.byref(shape), keep[1], cus, wg_per_cu, _vp(rec.ctypes.data), int(n), ctypes.byref(nwg), name, 96)
    if n < 0:
        raise CkvError(int(n), ckv_last_error())
    return rec[:n], int(nwg.value), name.value.decode()


def ckv_remap_hot_rows(cache, pool_k, pool_v, pool_k_out, pool_v_out, new_id=None, stream=0):
    _check(_lib.ckv_remap_hot_rows(cache, _dev(pool_k), _dev(pool_v), _dev(pool_k_out), _dev(pool_v_out), _dev(new_id), _vp(stream)))


def ckv_cache_is_offloaded(cache):
    return bool(_lib.ckv_cache_is_offloaded(cache))


def ckv_cache_idx(cache):
    return _lib.ckv_cache_idx(cache) or 0


def ckv_cache_user_k(cache):
    return _lib.ckv_cache_user_k(cache) or 0


def ckv_cache_user_v(cache):
    return _lib.ckv_cache_user_v(cache) or 0


def ckv_cache_lengths(cache):
    return _lib.ckv_cache_lengths(cache) or 0


def ckv_cache_positions(cache):
    return int(_lib.ckv_cache_positions(cache))


def ckv_cache_stored_bytes(cache):
    return int(_lib.ckv_cache_stored_bytes(cache))


def ckv_attend(cache, pool_k, pool_v, idx, user_k, user_v, q, lengths, out, stream=0):
    _check(_lib.ckv_attend(cache, _dev(pool_k), _dev(pool_v), _dev(idx), _dev(user_k), _dev(user_v), _dev(q),
                           _dev(lengths), _dev(out), _vp(stream)))


def ckv_attend_static_scratch(cache, pool_k, pool_v, idx, user_k, user_v, q, lengths, out, stream=0):
    _check(_lib.ckv_attend_static_scratch(cache, _dev(pool_k), _dev(pool_v), _dev(idx), _dev(user_k), _dev(user_v), _dev(q),
                                          _dev(lengths), _dev(out), _vp(stream)))


def ckv_set_option(key, value=None):
    """Tuning option of the calling thread (see include/ckv.h); key None restores every default."""
    _check(_lib.ckv_set_option(None if key is None else key.encode(), None if value is None else str(value).encode()))


def ckv_reconstruct(cache, pool_k, pool_v, k_full, v_full, stream=0):
    _check(_lib.ckv_reconstruct(cache, _dev(pool_k), _dev(pool_v), _dev(k_full), _dev(v_full), _vp(stream)))


def ckv_free(cache):
    _lib.ckv_free(cache)


def ckv_set_timing(cache, enable):
    _check(_lib.ckv_set_timing(cache, int(enable)))


def ckv_kernel_ms(cache):
    return float(_lib.ckv_kernel_ms(cache))


def ckv_kernel_times(cache, max_launches=4096):
    """(main kernel ms, merge kernel ms) per recorded launch, oldest first, as float32 numpy arrays."""
    k = np.zeros(max_launches, dtype=np.float32)
    m = np.zeros(max_launches, dtype=np.float32)
    n = _lib.ckv_kernel_times(cache, _vp(k.ctypes.data), _vp(m.ctypes.data), max_launches)
    if n < 0:
        raise CkvError(int(n), ckv_last_error())
    return k[:n], m[:n]


def ckv_variant(cache):
    return _lib.ckv_variant(cache).decode()


def ckv_copy(dst, src, nbytes, stream=0):
    _check(_lib.ckv_copy(_dev(dst), _dev(src), nbytes, _vp(stream)))


def ckv_trace_enable(cache, enable):
    _check(_lib.ckv_trace_enable(cache, int(enable)))


def ckv_trace_read(cache, max_items):
    """numpy uint64 [n][8] timeline records (see include/ckv.h)."""
    buf = np.zeros((max_items, 8), dtype=np.uint64)
    n = _lib.ckv_trace_read(cache, _vp(buf.ctypes.data), max_items)
    if n < 0:
        raise CkvError(int(n), ckv_last_error())
    return buf[:n]
