"""Device plumbing around the C-ABI calls: holds the torch buffers of one workload.

torch is used for device memory and the stream only; every step of the path runs inside
libckv.so.  Used by the tests, the smoke check and the benchmark.
"""
import numpy as np
import torch

from . import ckv


def _to_device(a, dtype):
    """numpy storage array (float32, or bf16 bit patterns in uint16) -> torch tensor on cuda:0."""
    if dtype == ckv.CKV_F32:
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).cuda().view(torch.bfloat16)


def _to_host(t, dtype):
    """torch tensor -> numpy storage array."""
    if dtype == ckv.CKV_F32:
        return t.cpu().numpy()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


class Session:
    """Pools and queries on the device, the packed cache handle, an output buffer."""

    def __init__(self, w, offloaded=False, prefill=None):
        """prefill: a prefill workload dict (embedding, router and projection weights); the packed cache is
        then computed on the device by ckv_prefill instead of being packed from w's host arrays."""
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the CollectiveKV hot path needs an MI355X (there is no CPU fallback)")
        self.w = w
        self.dtype = w["dtype"]
        self.d_a = w["d_g"] + w["d_u"]
        self.share = w.get("share", 0)
        self.shape = ckv.make_shape(w["B"], w["H"], w["d_g"], w["d_u"], w["P"], w["Nq"], w["dtype"], w["mode"],
                                    w["scale"], w["pool_ld"], self.share)
        # user columns of each side: d_u, or all d_a columns for a side that is not shared
        self.d_uk = w["d_u"] if self.share in (0, 1) else self.d_a
        self.d_uv = w["d_u"] if self.share in (0, 2) else self.d_a
        self.stream = torch.cuda.current_stream().cuda_stream
        self.pool_k = _to_device(w["pool_k"], self.dtype) if w["d_g"] > 0 else None
        self.pool_v = _to_device(w["pool_v"], self.dtype) if w["d_g"] > 0 else None
        self.q = _to_device(w["q"], self.dtype)
        tdt = torch.float32 if self.dtype == ckv.CKV_F32 else torch.bfloat16
        self.out = torch.full((w["B"], w["H"], w["Nq"], self.d_a), float("nan"), dtype=tdt, device="cuda")
        self.router = None
        if prefill is not None:
            r = prefill
            assert not offloaded and r["H"] == w["H"] and r["d_u"] == w["d_u"] and r["dtype"] == w["dtype"]
            assert r.get("share", 0) == self.share
            assert r["T"] == int(np.sum(w["lengths"])) and (w["d_g"] == 0 or r["P"] == w["P"])
            self.S = _to_device(r["S"], self.dtype)
            self.rw = {k: _to_device(r[k], self.dtype) for k in ("w_rk", "w_rv", "w_k", "w_v")}
            self.rb = {k: torch.from_numpy(np.ascontiguousarray(r[k], dtype=np.float32)).cuda()
                       for k in ("b_rk", "b_rv", "b_k", "b_v")}
            self.router = ckv.make_router(r["d_e"], self.rw["w_rk"], self.rb["b_rk"], self.rw["w_rv"], self.rb["b_rv"],
                                          self.rw["w_k"], self.rb["b_k"], self.rw["w_v"], self.rb["b_v"])
            self.cache = ckv.ckv_prefill(self.shape, self.router, w["lengths"], self.S, self.stream)
        else:
            build = ckv.ckv_build_cache_offloaded if offloaded else ckv.ckv_build_cache
            self.cache = build(self.shape, w["lengths"], w["idx_k"], w["idx_v"], w["user_k"], w["user_v"], self.stream)
        self.T = ckv.ckv_cache_positions(self.cache)

    def attend(self, stream=None, static_scratch=False):
        """static_scratch: go through the entry point that keeps the split workspace in the library's fixed array."""
        c = self.cache
        call = ckv.ckv_attend_static_scratch if static_scratch else ckv.ckv_attend
        call(c, self.pool_k, self.pool_v, ckv.ckv_cache_idx(c), ckv.ckv_cache_user_k(c),
             ckv.ckv_cache_user_v(c), self.q, ckv.ckv_cache_lengths(c), self.out,
             self.stream if stream is None else stream)
        return self.out

    def prefill_again(self, stream=None):
        """Recompute the packed cache in place from the embedding and the router (no allocation)."""
        ckv.ckv_prefill_into(self.cache, self.router, self.S, self.stream if stream is None else stream)

    def remap_hot_rows(self):
        """Renumber the pool rows most used first; returns new_id as numpy int32 [2][H][P]."""
        H, P = self.w["H"], self.w["P"]
        new_id = torch.zeros((2, H, P), dtype=torch.int32, device="cuda")
        pk = torch.empty_like(self.pool_k) if self.pool_k is not None else None
        pv = torch.empty_like(self.pool_v) if self.pool_v is not None else None
        ckv.ckv_remap_hot_rows(self.cache, self.pool_k, self.pool_v, pk, pv, new_id, self.stream)
        d_gk = self.w["d_g"] if self.share in (0, 1) else 0
        d_gv = self.w["d_g"] if self.share in (0, 2) else 0
        if d_gk > 0:
            self.pool_k = pk
        if d_gv > 0:
            self.pool_v = pv
        return new_id.cpu().numpy()

    def output(self):
        """Output of the last attend() as float64 numpy (exact widening of the stored values)."""
        torch.cuda.synchronize()
        a = _to_host(self.out, self.dtype)
        if self.dtype == ckv.CKV_F32:
            return a.astype(np.float64)
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)

    def reconstruct(self):
        """Final K and V rows as numpy storage arrays, each [H][T][d_a]."""
        tdt = torch.float32 if self.dtype == ckv.CKV_F32 else torch.bfloat16
        k = torch.zeros((self.w["H"], self.T, self.d_a), dtype=tdt, device="cuda")
        v = torch.zeros_like(k)
        ckv.ckv_reconstruct(self.cache, self.pool_k, self.pool_v, k, v, self.stream)
        torch.cuda.synchronize()
        return _to_host(k, self.dtype), _to_host(v, self.dtype)

    def packed_views(self):
        """Copies of the packed cache as numpy: idx [2][H][T], user_k/user_v [H][T][d_u] storage arrays."""
        H, T = self.w["H"], self.T
        e = 4 if self.dtype == ckv.CKV_F32 else 2

        def pull(addr, nbytes, npdt):
            if nbytes == 0 or not addr:
                return np.zeros(0, dtype=npdt)
            buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            ckv.ckv_copy(buf, addr, nbytes, self.stream)
            torch.cuda.synchronize()
            return buf.cpu().numpy().view(npdt)

        idx = pull(ckv.ckv_cache_idx(self.cache), 2 * H * T * 4, np.int32).reshape(2, H, T) if self.w["d_g"] > 0 else None
        sdt = np.float32 if self.dtype == ckv.CKV_F32 else np.uint16
        uk = pull(ckv.ckv_cache_user_k(self.cache), H * T * self.d_uk * e, sdt).reshape(H, T, self.d_uk)
        uv = pull(ckv.ckv_cache_user_v(self.cache), H * T * self.d_uv * e, sdt).reshape(H, T, self.d_uv)
        return idx, uk, uv

    def close(self):
        if self.cache:
            torch.cuda.synchronize()
            ckv.ckv_free(self.cache)
            self.cache = 0

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
