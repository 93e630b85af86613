"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It never imports the GPU package; the GPU package never imports it.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ckv_oracle.c")
_LIB = os.path.join(_HERE, "libckv_oracle.so")

F32, BF16 = 0, 1
SOFTMAX, SILU_OVER_N = 0, 1

_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain -O2, OpenMP over (user, head) only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        lib.ckv_oracle_attend.restype = ctypes.c_int
        lib.ckv_oracle_attend.argtypes = [i32] * 8 + [dbl, i64] + [vp] * 9 + [vp, i32]
        lib.ckv_oracle_reconstruct.restype = ctypes.c_int
        lib.ckv_oracle_reconstruct.argtypes = [i32] * 5 + [i64, i64] + [vp] * 8
        lib.ckv_oracle_cache_size.restype = None
        lib.ckv_oracle_cache_size.argtypes = [i64, i32, i32, i32, i32, i32] + [vp] * 4
        lib.ckv_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _check_store(a, dtype, name):
    want = np.float32 if dtype == F32 else np.uint16
    if a.dtype != want or not a.flags.c_contiguous:
        raise ValueError(f"{name}: expected C-contiguous {want.__name__}, got {a.dtype}")
    return a


def attend(w, users=None):
    """Attention outputs, fp64 [B][H][Nq][d_a].

    `w` is a workload dict as made by the seeded generators: keys B, H, d_g, d_u, P, Nq,
    dtype, mode, scale, pool_ld, lengths, idx_k, idx_v, user_k, user_v, pool_k, pool_v, q.
    Rows of users not listed in `users` are NaN.
    """
    lib = _load()
    dt = w["dtype"]
    d_a = w["d_g"] + w["d_u"]
    out = np.full((w["B"], w["H"], w["Nq"], d_a), np.nan, dtype=np.float64)
    lengths = np.ascontiguousarray(w["lengths"], dtype=np.int32)
    idx_k = np.ascontiguousarray(w["idx_k"], dtype=np.int32)
    idx_v = np.ascontiguousarray(w["idx_v"], dtype=np.int32)
    arrs = [_check_store(w[k], dt, k) for k in ("user_k", "user_v", "pool_k", "pool_v", "q")]
    if users is None:
        uptr, nu = ctypes.c_void_p(0), 0
    else:
        ulist = np.ascontiguousarray(users, dtype=np.int32)
        uptr, nu = _ptr(ulist), len(ulist)
    rc = lib.ckv_oracle_attend(
        w["B"], w["H"], w["d_g"], w["d_u"], w["P"], w["Nq"], dt, w["mode"],
        float(w["scale"]), int(w["pool_ld"]),
        _ptr(lengths), _ptr(idx_k), _ptr(idx_v), *[_ptr(a) for a in arrs], _ptr(out), uptr, nu)
    if rc != 0:
        raise ValueError("ckv_oracle_attend rejected its arguments")
    return out


def reconstruct(w):
    """Final K and V rows in the storage dtype, each [T][H][d_a]."""
    lib = _load()
    dt = w["dtype"]
    d_a = w["d_g"] + w["d_u"]
    T = int(np.sum(w["lengths"]))
    store = np.float32 if dt == F32 else np.uint16
    k_full = np.zeros((T, w["H"], d_a), dtype=store)
    v_full = np.zeros((T, w["H"], d_a), dtype=store)
    idx_k = np.ascontiguousarray(w["idx_k"], dtype=np.int32)
    idx_v = np.ascontiguousarray(w["idx_v"], dtype=np.int32)
    arrs = [_check_store(w[k], dt, k) for k in ("user_k", "user_v", "pool_k", "pool_v")]
    rc = lib.ckv_oracle_reconstruct(
        w["H"], w["d_g"], w["d_u"], w["P"], dt, int(w["pool_ld"]), T,
        _ptr(idx_k), _ptr(idx_v), *[_ptr(a) for a in arrs], _ptr(k_full), _ptr(v_full))
    if rc != 0:
        raise ValueError("ckv_oracle_reconstruct rejected its arguments")
    return k_full, v_full


def cache_size(T, H, d_g, d_u, dtype, index_bytes=4):
    """(stored_elems, full_elems, stored_bytes, full_bytes) of a CollectiveKV cache."""
    lib = _load()
    vals = [ctypes.c_int64(0) for _ in range(4)]
    lib.ckv_oracle_cache_size(int(T), H, d_g, d_u, dtype, index_bytes, *[ctypes.byref(v) for v in vals])
    return tuple(int(v.value) for v in vals)


def threads():
    return int(_load().ckv_oracle_threads())
