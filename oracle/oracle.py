"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It never imports the GPU package; the GPU package never imports it.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "ckv_oracle.c"), os.path.join(_HERE, "ckv_prefill_oracle.c")]
_LIB = os.path.join(_HERE, "libckv_oracle.so")

F32, BF16 = 0, 1
SOFTMAX, SILU_OVER_N = 0, 1

_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain -O2, OpenMP over (user, head) only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(s) for s in _SRCS):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, *_SRCS, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        lib.ckv_oracle_attend.restype = ctypes.c_int
        lib.ckv_oracle_attend.argtypes = [i32] * 9 + [dbl, i64] + [vp] * 9 + [vp, i32]
        lib.ckv_oracle_attend_rss.restype = ctypes.c_int
        lib.ckv_oracle_attend_rss.argtypes = [i32] * 9 + [dbl, i64] + [vp] * 10 + [vp, i32]
        lib.ckv_oracle_attend_scales.restype = ctypes.c_int
        lib.ckv_oracle_attend_scales.argtypes = [i32] * 9 + [dbl, i64] + [vp] * 13 + [vp, i32]
        lib.ckv_oracle_reconstruct.restype = ctypes.c_int
        lib.ckv_oracle_reconstruct.argtypes = [i32] * 6 + [i64, i64] + [vp] * 8
        lib.ckv_oracle_cache_size.restype = None
        lib.ckv_oracle_cache_size.argtypes = [i64, i32, i32, i32, i32, i32, i32] + [vp] * 4
        lib.ckv_oracle_threads.restype = ctypes.c_int
        lib.ckv_oracle_set_threads.restype = None
        lib.ckv_oracle_set_threads.argtypes = [i32]
        lib.ckv_oracle_prefill.restype = ctypes.c_int
        lib.ckv_oracle_prefill.argtypes = [i32] * 7 + [i64] + [vp] * 13
        lib.ckv_oracle_router_gap.restype = ctypes.c_int
        lib.ckv_oracle_router_gap.argtypes = [i32] * 4 + [i64] + [vp] * 6
        _lib = lib
    return _lib


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _check_store(a, dtype, name):
    want = np.float32 if dtype == F32 else np.uint16
    if a.dtype != want or not a.flags.c_contiguous:
        raise ValueError(f"{name}: expected C-contiguous {want.__name__}, got {a.dtype}")
    return a


def attend(w, users=None, with_rss=False, with_scales=False, with_asum=False):
    """Attention outputs, fp64 [B][H][Nq][d_a].

    `w` is a workload dict as made by the seeded generators: keys B, H, d_g, d_u, P, Nq,
    dtype, mode, scale, pool_ld, lengths, idx_k, idx_v, user_k, user_v, pool_k, pool_v, q.
    Rows of users not listed in `users` are NaN.
    with_rss: also return, per output element c, the scale the tests' comparison rule uses (same shape):
    sqrt(sum over groups g of positions with one and the same weight of (sum_{i in g} w_i V_i[c])^2).
    with_scales: return (out, rss, sss, acs), sss being the scale of the scores' rounding errors: with
    A_i = |scale| sum_k |q_k K_ik|, sqrt(sum over the same groups of (sum_{i in g} k_i)^2), where
    k_i = w_i (V_i[c] - out[c]) A_i for softmax and f'(s_i) V_i[c] A_i / n for SiLU/n (first-order effect of an
    error delta_i A_i of score i on the output), and acs the scale of the roundings of out[c]'s own additions when they are
    done in single precision in an unknown order: sqrt(n) * (|out[c]| + sqrt(sum_i (w_i V_i[c])^2)), n the user's length.
    with_asum (with with_scales): return (out, rss, sss, acs, asum), asum[c] = sum_i |w_i V_i[c]|.
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
    head = (w["B"], w["H"], w["d_g"], w["d_u"], w["P"], w["Nq"], dt, w["mode"], int(w.get("share", 0)),
            float(w["scale"]), int(w["pool_ld"]),
            _ptr(lengths), _ptr(idx_k), _ptr(idx_v), *[_ptr(a) for a in arrs])
    if with_scales:
        rss = np.full(out.shape, np.nan, dtype=np.float64)
        sss = np.full(out.shape, np.nan, dtype=np.float64)
        acs = np.full(out.shape, np.nan, dtype=np.float64)
        asum = np.full(out.shape, np.nan, dtype=np.float64) if with_asum else None
        rc = lib.ckv_oracle_attend_scales(*head, _ptr(out), _ptr(rss), _ptr(sss), _ptr(acs),
                                          _ptr(asum) if with_asum else ctypes.c_void_p(0), uptr, nu)
    elif with_rss:
        rss = np.full(out.shape, np.nan, dtype=np.float64)
        rc = lib.ckv_oracle_attend_rss(*head, _ptr(out), _ptr(rss), uptr, nu)
    else:
        rc = lib.ckv_oracle_attend(*head, _ptr(out), uptr, nu)
    if rc != 0:
        raise ValueError("ckv_oracle_attend rejected its arguments")
    if with_scales:
        return (out, rss, sss, acs, asum) if with_asum else (out, rss, sss, acs)
    return (out, rss) if with_rss else out


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
        w["H"], w["d_g"], w["d_u"], w["P"], dt, int(w.get("share", 0)), int(w["pool_ld"]), T,
        _ptr(idx_k), _ptr(idx_v), *[_ptr(a) for a in arrs], _ptr(k_full), _ptr(v_full))
    if rc != 0:
        raise ValueError("ckv_oracle_reconstruct rejected its arguments")
    return k_full, v_full


def cache_size(T, H, d_g, d_u, dtype, index_bytes=4, share=0):
    """(stored_elems, full_elems, stored_bytes, full_bytes) of a CollectiveKV cache (share: 0 both sides
    shared, 1 only K, 2 only V)."""
    lib = _load()
    vals = [ctypes.c_int64(0) for _ in range(4)]
    lib.ckv_oracle_cache_size(int(T), H, d_g, d_u, dtype, index_bytes, share, *[ctypes.byref(v) for v in vals])
    return tuple(int(v.value) for v in vals)


def threads():
    return int(_load().ckv_oracle_threads())


def set_threads(n):
    """Threads the (user, head) loop of the oracle uses from now on."""
    _load().ckv_oracle_set_threads(int(n))


def prefill_side_dims(r):
    """(d_uk, d_uv, P_k, P_v) of a prefill workload: an unshared side projects all d_a columns and has no router."""
    share = r.get("share", 0)
    d_u, P = r["d_u"], r["P"]
    d_uk, P_k = (d_u, P) if share in (0, 1) else (r["d_a"], 0)
    d_uv, P_v = (d_u, P) if share in (0, 2) else (r["d_a"], 0)
    return d_uk, d_uv, P_k, P_v


def _prefill_arrays(r):
    dt = r["dtype"]
    ws = [_check_store(r[k], dt, k) for k in ("S", "w_rk", "w_rv", "w_k", "w_v")]
    bs = [np.ascontiguousarray(r[k], dtype=np.float32) for k in ("b_rk", "b_rv", "b_k", "b_v")]
    return ws, bs


def prefill(r):
    """What the prefill stage caches: (idx_k, idx_v int32 [T][H], user_k, user_v float64 [T][H][d_u]).

    `r` is a prefill workload dict as made by the seeded generators: keys H, d_e, d_u, P, dtype,
    S [T][d_e], w_rk, w_rv [H][P][d_e], b_rk, b_rv [H][P], w_k, w_v [H][d_u][d_e], b_k, b_v [H][d_u].
    With r["share"] = 1 (2) only the key (value) side is shared: the other side has no router and its
    projection has r["d_a"] rows.
    """
    lib = _load()
    (S, w_rk, w_rv, w_k, w_v), (b_rk, b_rv, b_k, b_v) = _prefill_arrays(r)
    T, H = S.shape[0], r["H"]
    d_uk, d_uv, P_k, P_v = prefill_side_dims(r)
    idx_k = np.zeros((T, H), dtype=np.int32)
    idx_v = np.zeros((T, H), dtype=np.int32)
    user_k = np.zeros((T, H, d_uk), dtype=np.float64)
    user_v = np.zeros((T, H, d_uv), dtype=np.float64)
    rc = lib.ckv_oracle_prefill(H, r["d_e"], d_uk, d_uv, P_k, P_v, r["dtype"], T, _ptr(S), _ptr(w_rk), _ptr(b_rk), _ptr(w_rv),
                                _ptr(b_rv), _ptr(w_k), _ptr(b_k), _ptr(w_v), _ptr(b_v), _ptr(idx_k), _ptr(idx_v),
                                _ptr(user_k), _ptr(user_v))
    if rc != 0:
        raise ValueError("ckv_oracle_prefill rejected its arguments")
    return idx_k, idx_v, user_k, user_v


def router_gap(r, side, cand):
    """(gap, mag) float64 [T][H] of the candidate indices `cand` [T][H] for the key (side "k") or value
    (side "v") router: distance of the candidate's routing score from the row maximum, and the size of
    the terms behind the candidate's score."""
    lib = _load()
    dt = r["dtype"]
    S = _check_store(r["S"], dt, "S")
    w = _check_store(r["w_r" + side], dt, "w_r" + side)
    b = np.ascontiguousarray(r["b_r" + side], dtype=np.float32)
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    T, H = S.shape[0], r["H"]
    assert cand.shape == (T, H)
    gap = np.zeros((T, H), dtype=np.float64)
    mag = np.zeros((T, H), dtype=np.float64)
    rc = lib.ckv_oracle_router_gap(H, r["d_e"], r["P"], dt, T, _ptr(S), _ptr(w), _ptr(b), _ptr(cand), _ptr(gap), _ptr(mag))
    if rc != 0:
        raise ValueError("ckv_oracle_router_gap rejected its arguments")
    return gap, mag


def hot_row_order(w):
    """Frequency renumbering of the pool rows (router activations overlap across users, appendix "Analysis of
    Router Activations"): for every side and head, rows sorted by how often the cache refers to them, most
    used first, equal counts by row number.  Returns (new_id_k, new_id_v), each int32 [H][P] mapping an old
    row number to its new one (zeros for a side that is not shared).  Plain numpy: bincount + stable argsort."""
    H, P = w["H"], w["P"]
    share = w.get("share", 0)
    out = []
    for side, idx in ((0, w["idx_k"]), (1, w["idx_v"])):
        shared = w["d_g"] > 0 and (share == 0 or (share == 1 and side == 0) or (share == 2 and side == 1))
        new_id = np.zeros((H, P), dtype=np.int32)
        if shared:
            for h in range(H):
                counts = np.bincount(idx[:, h], minlength=P)
                order = np.argsort(-counts, kind="stable")     # old rows in their new order
                new_id[h, order] = np.arange(P, dtype=np.int32)
        out.append(new_id)
    return out[0], out[1]
