"""The comparison rule of the GPU parity tests, tried on the CPU: a plain single-precision evaluation of the decode stage
(section 4.2) must pass it, also where all weights are equal and value rows nearly cancel, and planted mistakes must not."""
import numpy as np
import pytest

from oracle import oracle
from paper_2601_19178_amd import workloads as wl
from tests.parity import compare


def one_key_row(n=64, d_a=130, Nq=9, H=2, B=3, seed=5077, mode=wl.SILU_OVER_N):
    """Keys shared with a pool of one row and no user columns, values an ordinary cache: every position of a history has
    the same score, hence the same weight, while the value rows differ and some columns nearly cancel."""
    return wl.make(B=B, L=None, H=H, d_a=d_a, d_u=0, P=1, idx="uniform", Nq=Nq, mode=mode, dtype=wl.F32,
                   sigma_pool=d_a ** -0.5, seed=seed, lengths=np.full(B, n, np.int32), share=wl.SHARE_K, pool_ld=d_a + 2)


def single_precision(w, drop=None):
    """out = sum_i w_i V_i with exact weights rounded to fp32, products and additions in IEEE fp32, history order.
    drop: a position left out of every sum (a planted mistake)."""
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    d_a = w["d_g"] + w["d_u"]
    g = np.zeros((w["B"], w["H"], w["Nq"], d_a))
    for b in range(w["B"]):
        n = int(w["lengths"][b])
        for h in range(w["H"]):
            V = w["user_v"][off[b]:off[b + 1], h, :]
            K = np.repeat(w["pool_k"][h, 0, :d_a][None].astype(np.float64), n, 0)
            for j in range(w["Nq"]):
                s = K @ w["q"][b, h, j].astype(np.float64) * w["scale"]
                if w["mode"] == wl.SOFTMAX:
                    wt = np.exp(s - s.max())
                    wt = (wt / wt.sum()).astype(np.float32)
                else:
                    wt = (s / (1 + np.exp(-s)) / n).astype(np.float32)
                acc = np.zeros(d_a, np.float32)
                for i in range(n):
                    if i != drop:
                        acc = (acc + wt[i] * V[i]).astype(np.float32)
                g[b, h, j] = acc
    return g


@pytest.mark.parametrize("mode,n", [(wl.SILU_OVER_N, 64), (wl.SILU_OVER_N, 63), (wl.SOFTMAX, 64), (wl.SOFTMAX, 100)])
def test_single_precision_additions_pass_with_the_fourth_term(mode, n):
    w = one_key_row(mode=mode, n=n)
    ref, rss, sss, acs = oracle.attend(w, with_scales=True)
    np.testing.assert_allclose(rss, np.abs(ref), rtol=1e-9)      # one group: the weights' scale has collapsed
    g = single_precision(w)
    without = compare(g, ref, rss, wl.F32, sss)
    full = compare(g, ref, rss, wl.F32, sss, acs)
    assert without["norm_err"] < 1e-6                             # a faithful fp32 result ...
    if mode == wl.SILU_OVER_N:
        # ... that the first three terms alone reject on the columns that nearly cancel (with softmax the common weight
        # is 1/64, a power of two, the products are exact and fewer roundings remain)
        assert without["worst_ratio"] > 1.0
    assert full["worst_ratio"] < 0.2


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_planted_mistakes_fail_the_full_rule(mode):
    w = one_key_row(mode=mode)
    ref, rss, sss, acs = oracle.attend(w, with_scales=True)
    assert compare(single_precision(w, drop=17), ref, rss, wl.F32, sss, acs)["worst_ratio"] > 50      # a position left out
    g = single_precision(w)
    assert compare(np.roll(g, 1, axis=-1), ref, rss, wl.F32, sss, acs)["worst_ratio"] > 50             # columns off by one
    assert compare(g * (1 + 3e-4), ref, rss, wl.F32, sss, acs)["worst_ratio"] > 1.0                    # 3e-4 relative: beyond 1e-4


def test_fourth_term_is_small_where_weights_differ():
    # an ordinary workload (no two equal weights): the additions' term adds little to the bound
    w = wl.make(B=2, L=None, H=1, d_a=64, d_u=8, P=500, idx="uniform", Nq=4, mode=wl.SOFTMAX, dtype=wl.F32,
                sigma_pool=0.125, seed=11, lengths=np.array([1024, 200], np.int32))
    ref, rss, sss, acs = oracle.attend(w, with_scales=True)
    base = 1e-4 * np.abs(ref) + 1e-4 * rss
    assert np.max(8 * 2.0 ** -24 * acs / base) < 0.2


# ---------------------------------------------------------------------------------------------
# weights that are nearly equal are rounded to bf16 the same way: the bound u_w * asum of the rule
def two_clusters(n=400):
    """One user, one head, one query, eight columns of which the first two are the user's; a pool of two key rows (scores +1
    and -1 up to 1e-4 from the user's columns, no two alike) and two value rows chosen so that the two clusters of SiLU
    weights nearly cancel in the pool columns.  All stored values are exact in bf16."""
    w = wl.make(B=1, L=None, H=1, d_a=8, d_u=2, P=2, idx="uniform", Nq=1, mode=wl.SILU_OVER_N, dtype=wl.BF16,
                sigma_pool=1.0, seed=3, lengths=np.array([n], np.int32), scale=1.0, pool_ld=8)
    bits = wl.f32_to_bf16_bits
    rng = np.random.default_rng(12)
    w["idx_k"][:, 0] = np.arange(n) % 2
    w["idx_v"][:, 0] = np.arange(n) % 2
    pk = np.zeros((1, 2, 8), np.float32); pk[0, 0, 0] = 1.0; pk[0, 1, 0] = -1.0          # pool column 0 carries the score
    pv = np.zeros((1, 2, 8), np.float32); pv[0, 0, :6] = 1.0; pv[0, 1, :6] = 2.71875      # silu(1) : |silu(-1)| = 2.7183
    qq = np.zeros((1, 1, 1, 8), np.float32); qq[0, 0, 0, :3] = 1.0                        # [user columns | pool columns]
    uk = np.stack([rng.integers(-127, 128, size=(n, 1)) * 2.0 ** -20,                     # the keys differ a little
                   rng.integers(-127, 128, size=(n, 1)) * 2.0 ** -27], axis=2).astype(np.float32)
    uv = np.zeros((n, 1, 2), np.float32)
    for k, a in (("pool_k", pk), ("pool_v", pv), ("q", qq), ("user_k", uk), ("user_v", uv)):
        w[k] = bits(a)
    return w, pk, pv, qq, uk


def test_nearly_equal_weights_round_alike_and_the_rule_knows():
    w, pk, pv, qq, uk = two_clusters()
    n = int(w["lengths"][0])
    ref, rss, sss, acs, asum = oracle.attend(w, with_scales=True, with_asum=True)
    # the decode stage with the weights rounded to bf16 and everything else exact
    s = uk[:, 0, :].astype(np.float64).sum(axis=1) + pk[0, np.arange(n) % 2, 0].astype(np.float64)
    wt = s / (1 + np.exp(-s)) / n
    assert len(np.unique(wt)) > n // 2                                   # not two clusters of *equal* weights: ...
    wt16 = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(wt.astype(np.float32))).astype(np.float64)
    assert len(np.unique(wt16)) <= 4                                     # ... but two or three values after rounding
    V = np.concatenate([np.zeros((n, 2)), pv[0, np.arange(n) % 2, :6].astype(np.float64)], axis=1)   # [user | pool]
    exact = (wt[:, None] * V).sum(axis=0)
    np.testing.assert_allclose(ref[0, 0, 0], exact, rtol=1e-9, atol=1e-15)
    g = (wt16[:, None] * V).sum(axis=0)[None, None, None]
    assert np.abs(ref[0, 0, 0, 2]) < 0.02 * asum[0, 0, 0, 2]             # the pool columns nearly cancel
    without = compare(g, ref, rss, wl.BF16, sss, acs)
    full = compare(g, ref, rss, wl.BF16, sss, acs, asum)
    assert without["worst_ratio"] > 1.0        # independent roundings would stay far below tol * rss: these add up
    assert 0.3 < full["worst_ratio"] < 1.0     # the bound that needs no model holds, and not by a wide margin
    # planted mistakes still fail: positions left out, the weights of one cluster off by two bf16 steps
    gone = [17, 19, 21]                                                  # three positions of one cluster
    drop = (np.delete(wt16, gone)[:, None] * np.delete(V, gone, axis=0)).sum(axis=0)[None, None, None]
    assert compare(drop, ref, rss, wl.BF16, sss, acs, asum)["worst_ratio"] > 2.0
    off = ((wt16 * np.where(np.arange(n) % 2 == 0, 1 + 2.0 ** -7, 1.0))[:, None] * V).sum(axis=0)[None, None, None]
    assert compare(off, ref, rss, wl.BF16, sss, acs, asum)["worst_ratio"] > 1.0


def test_magnitude_bound_is_the_smaller_one_for_short_histories():
    # an ordinary bf16 workload: for a history of a hundred positions tol * rss decides, for thousands u_w * asum does,
    # and that one stays at 2^-9 of what was added up
    w = wl.make(B=2, L=None, H=1, d_a=64, d_u=8, P=500, idx="uniform", Nq=4, mode=wl.SOFTMAX, dtype=wl.BF16,
                sigma_pool=0.125, seed=11, lengths=np.array([4096, 100], np.int32))
    ref, rss, sss, acs, asum = oracle.attend(w, with_scales=True, with_asum=True)
    ratio = 2.0 ** -9 * asum / (2e-2 * rss)
    assert np.median(ratio[1]) < 1.0 < np.median(ratio[0]) < 12.0
