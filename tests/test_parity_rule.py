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
