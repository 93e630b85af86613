"""Seeded synthetic workloads (inputs only; none of the method's arithmetic lives here).

The five workloads stand in for the recommendation datasets and trained weights the paper
evaluates on, which are not available: same shapes, value distributions and index
distributions, drawn from a counter-based generator (Philox) keyed by `seed`.

A workload is a plain dict:
  B, H, d_g, d_u, P, Nq, pool_ld : ints          dtype : 0 fp32 | 1 bf16     mode : 0 softmax | 1 SiLU/n
  share : 0 keys and values shared | 1 only keys | 2 only values
  scale : float
  lengths [B] int32                               history length n of every user
  idx_k, idx_v   [T][H] int32                     pool row per position and head (user-major, ragged)
  user_k, user_v [T][H][d_u]                      user-specific slices
  pool_k, pool_v [H][P][pool_ld]                  global pools; columns >= d_g are padding (NaN)
  q              [B][H][Nq][d_a]                  candidate queries
Stored values are float32 arrays (dtype 0) or bfloat16 bit patterns in uint16 (dtype 1),
rounded to nearest-even once, here.
"""
import numpy as np

F32, BF16 = 0, 1
SOFTMAX, SILU_OVER_N = 0, 1
SHARE_KV, SHARE_K, SHARE_V = 0, 1, 2   # both sides shared (CollectiveKV), only keys (CollectiveK), only values (CollectiveV)


def side_dims(d_u, d_g, share):
    """((d_u, d_g) of the K side, (d_u, d_g) of the V side): a side that is not shared is the ordinary cache,
    all d_a columns stored per position and no pool."""
    full = (d_u + d_g, 0)
    return ((d_u, d_g) if share in (SHARE_KV, SHARE_K) else full,
            (d_u, d_g) if share in (SHARE_KV, SHARE_V) else full)

# name -> recipe.  L = (lo, hi) inclusive, uniform per user.  sigma_* are standard deviations.
CONFIGS = {
    "cfg1": dict(B=4, L=(50, 50), H=1, d_a=64, d_u=8, P=256, idx="uniform", Nq=1,
                 mode=SOFTMAX, dtype=F32, sigma_pool=1.0 / 8.0, seed=1001),
    "cfg2_f32": dict(B=1024, L=(200, 200), H=2, d_a=64, d_u=8, P=4096, idx="uniform", Nq=1,
                     mode=SOFTMAX, dtype=F32, sigma_pool=1.0 / 8.0, seed=1002),
    "cfg2_bf16": dict(B=1024, L=(200, 200), H=2, d_a=64, d_u=8, P=4096, idx="uniform", Nq=1,
                      mode=SOFTMAX, dtype=BF16, sigma_pool=1.0 / 8.0, seed=1002),
    "cfg3": dict(B=512, L=(1024, 1024), H=4, d_a=64, d_u=4, P=16384, idx=("zipf", 1.1), Nq=64,
                 mode=SILU_OVER_N, dtype=BF16, sigma_pool=1.0 / 8.0, seed=1003),
    "cfg4": dict(B=128, L=(2048, 8192), H=8, d_a=128, d_u=8, P=65536, idx="uniform", Nq=128,
                 mode=SOFTMAX, dtype=BF16, sigma_pool=128.0 ** -0.5, seed=1004),
    # config 3 with only the keys shared (CollectiveK) / only the values shared (CollectiveV): the other side
    # is an ordinary 64-column cache
    "cfg3_ck": dict(B=512, L=(1024, 1024), H=4, d_a=64, d_u=4, P=16384, idx=("zipf", 1.1), Nq=64,
                    mode=SILU_OVER_N, dtype=BF16, sigma_pool=1.0 / 8.0, seed=1003, share=SHARE_K),
    "cfg3_cv": dict(B=512, L=(1024, 1024), H=4, d_a=64, d_u=4, P=16384, idx=("zipf", 1.1), Nq=64,
                    mode=SILU_OVER_N, dtype=BF16, sigma_pool=1.0 / 8.0, seed=1003, share=SHARE_V),
    # configs 3 and 4 with an ordinary K/V cache (d_g = 0: every column is user specific; section 5.3's degenerate
    # case): the same decode without compression, for comparison on the same kernel
    "cfg3_plain": dict(B=512, L=(1024, 1024), H=4, d_a=64, d_u=64, P=1, idx="uniform", Nq=64,
                       mode=SILU_OVER_N, dtype=BF16, sigma_pool=1.0 / 8.0, sigma_user=1.0 / 8.0, seed=1003),
    "cfg4_plain": dict(B=128, L=(2048, 8192), H=8, d_a=128, d_u=128, P=1, idx="uniform", Nq=128,
                       mode=SOFTMAX, dtype=BF16, sigma_pool=128.0 ** -0.5, sigma_user=128.0 ** -0.5, seed=1004),
    "cfg5": dict(B=8192, L=(512, 2048), H=4, d_a=64, d_u=2, P=1048576, idx=("zipf", 1.05), Nq=16,
                 mode=SOFTMAX, dtype=BF16, sigma_pool=1.0 / 8.0, seed=1005),
    # the head width behind the compression ratios of Table 1 (d = 256; CR 0.020 is d_u = 4, CR 0.043 is d_u = 10),
    # on config 4's batch of long ragged histories
    "d256_u4": dict(B=128, L=(2048, 8192), H=4, d_a=256, d_u=4, P=32768, idx="uniform", Nq=128,
                    mode=SOFTMAX, dtype=BF16, sigma_pool=1.0 / 16.0, seed=1006),
    "d256_u10": dict(B=128, L=(2048, 8192), H=4, d_a=256, d_u=10, P=32768, idx="uniform", Nq=128,
                     mode=SOFTMAX, dtype=BF16, sigma_pool=1.0 / 16.0, seed=1006),
    # target attention (one query per user, section 2.1) over 256-column heads with Table 1's smallest and largest user
    # widths (CR 0.008 is d_u = 1, CR 0.043 is d_u = 10), histories of the benchmarks' lengths, a pool of the default size
    "tgt256_u1": dict(B=1024, L=(200, 2000), H=1, d_a=256, d_u=1, P=16384, idx="uniform", Nq=1,
                      mode=SOFTMAX, dtype=BF16, sigma_pool=1.0 / 16.0, seed=1008),
    "tgt256_u10": dict(B=1024, L=(200, 2000), H=1, d_a=256, d_u=10, P=16384, idx="uniform", Nq=1,
                       mode=SOFTMAX, dtype=BF16, sigma_pool=1.0 / 16.0, seed=1008),
    # config 3's batch shape with 256-column heads in fp32 storage (128 users): the fp32 matrix-core kernel's widest instance
    "cfg3_f32_d256": dict(B=128, L=(1024, 1024), H=4, d_a=256, d_u=4, P=16384, idx=("zipf", 1.1), Nq=64,
                          mode=SILU_OVER_N, dtype=F32, sigma_pool=1.0 / 16.0, seed=1007),
}


def f32_to_bf16_bits(x):
    """float32 array -> bfloat16 bit patterns (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a, dtype):
    """Stored array -> float64 (exact)."""
    return (a if dtype == F32 else bf16_bits_to_f32(a)).astype(np.float64)


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def _normal(rng, shape, sigma, dtype):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    x *= np.float32(sigma)
    return x if dtype == F32 else f32_to_bf16_bits(x)


def _draw_idx(rng, kind, P, shape, perm_rng):
    """Pool rows for every (position, head).  'uniform', or ('zipf', s): bounded Zipf over
    ranks 1..P with p(r) ~ r^-s, inverse CDF in fp64, ranks mapped to rows by a seeded
    permutation per head so that hot rows are not neighbours."""
    T, H = shape
    if kind == "uniform":
        return rng.integers(0, P, size=shape, dtype=np.int32)
    _, s = kind
    cdf = np.cumsum(np.arange(1, P + 1, dtype=np.float64) ** (-float(s)))
    cdf /= cdf[-1]
    out = np.empty(shape, dtype=np.int32)
    for h in range(H):
        perm = perm_rng.permutation(P).astype(np.int32)
        step = 1 << 22
        for lo in range(0, T, step):
            u = rng.random(size=min(step, T - lo))
            rank = np.minimum(np.searchsorted(cdf, u, side="left"), P - 1)
            out[lo:lo + len(u), h] = perm[rank]
    return out


def make(B, L, H, d_a, d_u, P, idx, Nq, mode, dtype, sigma_pool, seed,
         sigma_user=0.1, sigma_q=1.0, pool_ld=None, scale=None, lengths=None, pad_nan=True, share=SHARE_KV):
    """Build one workload dict from a recipe (see CONFIGS).  share: SHARE_K / SHARE_V give the ablation
    variants that share only keys / only values; the other side's user array then has d_a columns (drawn
    like pool entries) and its indices are zeros that nothing reads."""
    d_g = d_a - d_u
    (d_uk, d_gk), (d_uv, d_gv) = side_dims(d_u, d_g, share)
    if pool_ld is None:
        pool_ld = d_a if d_g > 0 else 0
    if lengths is None:
        lo, hi = L
        lengths = _rng(seed, 0).integers(lo, hi + 1, size=B, dtype=np.int32)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    assert lengths.shape == (B,)
    T = int(lengths.sum())
    P_eff = max(P, 1)
    perm_rng = _rng(seed, 9)
    idx_k = _draw_idx(_rng(seed, 1), idx, P_eff, (T, H), perm_rng) if d_gk > 0 else np.zeros((T, H), dtype=np.int32)
    idx_v = _draw_idx(_rng(seed, 2), idx, P_eff, (T, H), perm_rng) if d_gv > 0 else np.zeros((T, H), dtype=np.int32)
    user_k = _normal(_rng(seed, 3), (T, H, d_uk), sigma_user if d_gk > 0 or d_g == 0 else sigma_pool, dtype)
    user_v = _normal(_rng(seed, 4), (T, H, d_uv), sigma_user if d_gv > 0 or d_g == 0 else sigma_pool, dtype)
    pool_k = _normal(_rng(seed, 5), (H, P_eff, pool_ld), sigma_pool, dtype)
    pool_v = _normal(_rng(seed, 6), (H, P_eff, pool_ld), sigma_pool, dtype)
    if pad_nan and pool_ld > d_g:
        nan = np.float32(np.nan) if dtype == F32 else np.uint16(0x7FC0)
        pool_k[:, :, d_g:] = nan
        pool_v[:, :, d_g:] = nan
    q = _normal(_rng(seed, 7), (B, H, Nq, d_a), sigma_q, dtype)
    if scale is None:
        scale = d_a ** -0.5 if mode == SOFTMAX else 1.0
    return dict(B=B, H=H, d_g=d_g, d_u=d_u, P=P_eff, Nq=Nq, pool_ld=int(pool_ld), dtype=dtype,
                mode=mode, share=share, scale=float(scale), lengths=lengths, idx_k=idx_k, idx_v=idx_v,
                user_k=user_k, user_v=user_v, pool_k=pool_k, pool_v=pool_v, q=q)


def config(name, **override):
    """One of the named workloads, optionally with recipe fields overridden (smaller B, ...)."""
    recipe = dict(CONFIGS[name])
    recipe.update(override)
    return make(**recipe)


def algorithmic_bytes(w):
    """Bytes the method must move for one pass (latency analysis, section 4.4:
    load of s*d_u + s per K and per V, plus the index operation over s*d_g), plus q in and
    out out.  Returns dict(compressed, gathered, q_out, E, position_heads)."""
    e = 4 if w["dtype"] == F32 else 2
    ph = int(np.sum(w["lengths"], dtype=np.int64)) * w["H"]
    d_a = w["d_g"] + w["d_u"]
    sides = side_dims(w["d_u"], w["d_g"], w.get("share", SHARE_KV))
    compressed = ph * sum((4 if dg > 0 else 0) + du * e for du, dg in sides)
    gathered = ph * sum(dg * e for _, dg in sides)
    q_out = 2 * w["B"] * w["H"] * w["Nq"] * d_a * e
    return dict(position_heads=ph, compressed=compressed, gathered=gathered, q_out=q_out,
                E=compressed + gathered + q_out)


def make_prefill(T, H, d_e, d_u, P, dtype, seed, sigma_s=1.0, sigma_b=0.1, integers=None, share=SHARE_KV, d_a=None):
    """Inputs of the prefill stage (section 4.2 / 4.3): history embedding S [T][d_e] shared by the heads,
    per-head router weights w_rk, w_rv [H][P][d_e] (row j = column j of the paper's W_r) with fp32 bias
    b_rk, b_rv [H][P], per-head projection weights w_k, w_v [H][d_u][d_e] with fp32 bias b_k, b_v [H][d_u].
    Weights are N(0, 1/sqrt(d_e)), S is N(0, sigma_s), biases N(0, sigma_b).  With integers=m every value is
    a uniform integer in [-m, m]: all sums are then exact in fp32, so equal routing scores (ties) are common
    and every implementation must agree bit for bit.  They stand in for trained embeddings and routers.
    share = SHARE_K / SHARE_V (needs d_a): the side that is not shared projects all d_a columns (w_v or w_k has
    d_a rows) and its router is not used."""
    P_eff = max(P, 1)
    if share != SHARE_KV:
        assert d_a is not None and d_a >= d_u
    d_uk = d_u if share in (SHARE_KV, SHARE_K) else d_a
    d_uv = d_u if share in (SHARE_KV, SHARE_V) else d_a

    def draw(stream, shape, sigma, dt):
        rng = _rng(seed, stream)
        if integers is not None:
            x = rng.integers(-integers, integers + 1, size=shape).astype(np.float32)
            return x if dt == F32 else f32_to_bf16_bits(x)
        return _normal(rng, shape, sigma, dt)

    sw = d_e ** -0.5
    return dict(H=H, d_e=d_e, d_u=d_u, P=P_eff, dtype=dtype, T=T, share=share, d_a=d_a,
                S=draw(20, (T, d_e), sigma_s, dtype),
                w_rk=draw(21, (H, P_eff, d_e), sw, dtype), w_rv=draw(22, (H, P_eff, d_e), sw, dtype),
                b_rk=draw(23, (H, P_eff), sigma_b, F32), b_rv=draw(24, (H, P_eff), sigma_b, F32),
                w_k=draw(25, (H, d_uk, d_e), sw, dtype), w_v=draw(26, (H, d_uv, d_e), sw, dtype),
                b_k=draw(27, (H, d_uk), sigma_b, F32), b_v=draw(28, (H, d_uv), sigma_b, F32))


# Prefill workloads: the cache shapes of configs 2 and 3 (T positions, heads, d_u, pool size), an embedding
# width of 128 (the paper does not state d_e for its models).
PREFILL_CONFIGS = {
    "prefill_cfg2": dict(T=1024 * 200, H=2, d_e=128, d_u=8, P=4096, dtype=BF16, seed=1102),
    "prefill_cfg3": dict(T=512 * 1024, H=4, d_e=128, d_u=4, P=16384, dtype=BF16, seed=1103),
    "prefill_cfg2_f32": dict(T=1024 * 200, H=2, d_e=128, d_u=8, P=4096, dtype=F32, seed=1102),
}


def prefill_config(name, **override):
    recipe = dict(PREFILL_CONFIGS[name])
    recipe.update(override)
    return make_prefill(**recipe)


def prefill_flops(r):
    """Multiply-adds of the prefill stage counted as 2 flop: two routers and two projections per head."""
    return 2.0 * r["T"] * r["H"] * 2 * (r["P"] + r["d_u"]) * r["d_e"]
