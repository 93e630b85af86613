"""Pins of the prefill oracle (projection + router argmax) against things other than itself (CPU only).

Section 4.2 (prefill stage: K_u = S W_k + b_k, V_u = S W_v + b_v) and section 4.3 (router:
M = S W_r + b_r, I[i] = argmax_j M[i][j]).  A transposed weight, a swapped key/value router, a
missing bias, a head mix-up or a wrong tie rule fails at least one test here.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2601_19178_amd import workloads as wl


def f64(r, k):
    return wl.to_f64(r[k], r["dtype"]) if k[0] in "Sw" else r[k].astype(np.float64)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_matches_library_linear_and_argmax(dtype):
    """torch's linear layer (weight stored [out][in], as here) and argmax in fp64."""
    r = wl.make_prefill(T=83, H=3, d_e=24, d_u=5, P=61, dtype=dtype, seed=3)
    ik, iv, uk, uv = oracle.prefill(r)
    S = torch.from_numpy(f64(r, "S"))
    for h in range(r["H"]):
        for idx, w, b in ((ik, "w_rk", "b_rk"), (iv, "w_rv", "b_rv")):
            M = torch.nn.functional.linear(S, torch.from_numpy(f64(r, w)[h]), torch.from_numpy(f64(r, b)[h]))
            np.testing.assert_array_equal(idx[:, h], M.argmax(dim=1).numpy())
        for u, w, b in ((uk, "w_k", "b_k"), (uv, "w_v", "b_v")):
            ref = torch.nn.functional.linear(S, torch.from_numpy(f64(r, w)[h]), torch.from_numpy(f64(r, b)[h]))
            np.testing.assert_allclose(u[:, h, :], ref.numpy(), rtol=1e-12, atol=1e-12)


def test_one_hot_embedding_reads_one_weight_column():
    """S[i] = e_c makes M[i][j] = W_r[c][j] + b_r[j]: the index is known by construction, and a
    transposed weight matrix would read the wrong entries."""
    d_e, P, H = 7, 11, 2
    r = wl.make_prefill(T=d_e, H=H, d_e=d_e, d_u=2, P=P, dtype=wl.F32, seed=1)
    r["S"] = np.eye(d_e, dtype=np.float32)
    target_k = (3 * np.arange(d_e)[:, None] + np.arange(H)[None, :] + 1) % P   # [c][h]
    target_v = (5 * np.arange(d_e)[:, None] + 2 * np.arange(H)[None, :]) % P
    for w, tgt in (("w_rk", target_k), ("w_rv", target_v)):
        r[w] = np.full((H, P, d_e), -1.0, dtype=np.float32)
        for c in range(d_e):
            for h in range(H):
                r[w][h, tgt[c, h], c] = 2.0
    r["b_rk"][:] = 0.0
    r["b_rv"][:] = 0.0
    ik, iv, uk, uv = oracle.prefill(r)
    np.testing.assert_array_equal(ik, target_k)
    np.testing.assert_array_equal(iv, target_v)
    # the projection of e_c is column c of the weights plus the bias
    for h in range(H):
        np.testing.assert_allclose(uk[:, h, :], r["w_k"][h].T.astype(np.float64) + r["b_k"][h], rtol=0, atol=1e-15)
        np.testing.assert_allclose(uv[:, h, :], r["w_v"][h].T.astype(np.float64) + r["b_v"][h], rtol=0, atol=1e-15)


def test_zero_embedding_leaves_the_biases():
    r = wl.make_prefill(T=4, H=2, d_e=9, d_u=3, P=20, dtype=wl.BF16, seed=2)
    r["S"][:] = 0
    ik, iv, uk, uv = oracle.prefill(r)
    for h in range(2):
        assert (ik[:, h] == np.argmax(r["b_rk"][h])).all() and (iv[:, h] == np.argmax(r["b_rv"][h])).all()
        np.testing.assert_array_equal(uk[:, h, :], np.broadcast_to(r["b_k"][h].astype(np.float64), (4, 3)))
        np.testing.assert_array_equal(uv[:, h, :], np.broadcast_to(r["b_v"][h].astype(np.float64), (4, 3)))


def test_equal_maxima_give_the_lowest_index():
    r = wl.make_prefill(T=6, H=1, d_e=5, d_u=1, P=9, dtype=wl.F32, seed=4)
    r["w_rk"][:] = 0.0
    r["b_rk"][:] = 1.5            # a constant row of the routing map
    r["w_rv"][0, 7] = r["w_rv"][0, 2]  # two identical pool entries ...
    r["b_rv"][0, :] = -100.0
    r["b_rv"][0, 7] = r["b_rv"][0, 2] = 100.0  # ... that dominate every other
    ik, iv, _, _ = oracle.prefill(r)
    assert (ik == 0).all()
    assert (iv == 2).all()


def test_integer_inputs_have_many_ties_and_agree_with_integer_arithmetic():
    """Small integers: the routing map is exact in int64, so the argmax (first maximum) is fixed."""
    r = wl.make_prefill(T=200, H=2, d_e=8, d_u=2, P=50, dtype=wl.BF16, seed=6, integers=1)
    ik, iv, uk, _ = oracle.prefill(r)
    S = np.rint(f64(r, "S")).astype(np.int64)
    ties = 0
    for h in range(2):
        for idx, w, b in ((ik, "w_rk", "b_rk"), (iv, "w_rv", "b_rv")):
            M = S @ np.rint(f64(r, w)[h]).astype(np.int64).T + np.rint(r[b][h]).astype(np.int64)
            np.testing.assert_array_equal(idx[:, h], M.argmax(axis=1))
            ties += int(((M == M.max(axis=1, keepdims=True)).sum(axis=1) > 1).sum())
    assert ties > 50  # the case really exercises the tie rule
    assert np.array_equal(uk, np.rint(uk))


def test_pool_permutation_equivariance_and_positive_rescaling():
    r = wl.make_prefill(T=40, H=2, d_e=12, d_u=2, P=33, dtype=wl.F32, seed=8)
    ik, iv, _, _ = oracle.prefill(r)
    perm = np.random.default_rng(0).permutation(33)
    r2 = dict(r)
    for k in ("w_rk", "w_rv", "b_rk", "b_rv"):
        r2[k] = np.ascontiguousarray(r[k][:, perm] * np.float32(4.0))  # exact scaling by a power of two
    ik2, iv2, _, _ = oracle.prefill(r2)
    np.testing.assert_array_equal(perm[ik2], ik)
    np.testing.assert_array_equal(perm[iv2], iv)


def test_heads_and_sides_are_independent():
    r = wl.make_prefill(T=30, H=3, d_e=10, d_u=2, P=17, dtype=wl.F32, seed=9)
    base = oracle.prefill(r)
    r2 = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in r.items()}
    r2["w_rv"][1] *= -1.0   # value router of head 1 only
    r2["w_k"][2] += 1.0     # key projection of head 2 only
    new = oracle.prefill(r2)
    np.testing.assert_array_equal(new[0], base[0])                 # I_k untouched everywhere
    np.testing.assert_array_equal(new[1][:, [0, 2]], base[1][:, [0, 2]])
    assert (new[1][:, 1] != base[1][:, 1]).any()
    np.testing.assert_array_equal(new[3], base[3])                 # V_u untouched
    np.testing.assert_array_equal(new[2][:, :2], base[2][:, :2])
    assert (new[2][:, 2] != base[2][:, 2]).all()


def test_router_gap_is_the_distance_to_the_row_maximum():
    r = wl.make_prefill(T=25, H=2, d_e=6, d_u=1, P=13, dtype=wl.BF16, seed=10)
    ik, iv, _, _ = oracle.prefill(r)
    gap, mag = oracle.router_gap(r, "k", ik)
    assert (gap == 0).all() and (mag > 0).all()
    cand = (iv + 3) % 13
    gap, mag = oracle.router_gap(r, "v", cand)
    S = f64(r, "S")
    for h in range(2):
        W, b = f64(r, "w_rv")[h], f64(r, "b_rv")[h]
        M = S @ W.T + b
        np.testing.assert_allclose(gap[:, h], M.max(axis=1) - M[np.arange(25), cand[:, h]], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(mag[:, h], np.abs(S[:, None, :] * W[cand[:, h]][:, None, :]).sum(axis=(1, 2)) +
                                   np.abs(b[cand[:, h]]), rtol=1e-12)


def test_prefill_then_decode_is_dense_attention_over_projected_and_routed_rows():
    """End to end on a tiny case: the cache written by the prefill oracle, read by the decode oracle,
    equals attention over K = [S W_k + b_k | P_k[argmax(S W_rk + b_rk)]] built explicitly."""
    lengths = np.array([4, 0, 7, 1], dtype=np.int32)
    w = wl.make(B=4, L=None, H=2, d_a=12, d_u=3, P=19, idx="uniform", Nq=2, mode=wl.SOFTMAX, dtype=wl.F32,
                sigma_pool=0.5, seed=12, lengths=lengths)
    r = wl.make_prefill(T=int(lengths.sum()), H=2, d_e=10, d_u=3, P=19, dtype=wl.F32, seed=12)
    ik, iv, uk, uv = oracle.prefill(r)
    w["idx_k"], w["idx_v"] = ik, iv
    w["user_k"], w["user_v"] = uk.astype(np.float32), uv.astype(np.float32)
    out = oracle.attend(w)
    S = f64(r, "S")
    off = np.concatenate([[0], np.cumsum(lengths)])
    for b in range(4):
        for h in range(2):
            s = S[off[b]:off[b + 1]]
            if len(s) == 0:
                assert (out[b, h] == 0).all()
                continue
            K = np.concatenate([(s @ f64(r, "w_k")[h].T + r["b_k"][h]).astype(np.float32).astype(np.float64),
                                w["pool_k"][h][(s @ f64(r, "w_rk")[h].T + r["b_rk"][h]).argmax(1)][:, :9].astype(np.float64)], axis=1)
            V = np.concatenate([(s @ f64(r, "w_v")[h].T + r["b_v"][h]).astype(np.float32).astype(np.float64),
                                w["pool_v"][h][(s @ f64(r, "w_rv")[h].T + r["b_rv"][h]).argmax(1)][:, :9].astype(np.float64)], axis=1)
            sc = w["scale"] * w["q"][b, h].astype(np.float64) @ K.T
            p = np.exp(sc - sc.max(axis=1, keepdims=True))
            ref = (p / p.sum(axis=1, keepdims=True)) @ V
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("share", [wl.SHARE_K, wl.SHARE_V])
def test_prefill_with_one_side_shared(share):
    """The side that is not shared has no router; all its d_a columns are the projection."""
    r = wl.make_prefill(T=40, H=2, d_e=12, d_u=3, P=21, dtype=wl.F32, seed=14, share=share, d_a=10)
    ik, iv, uk, uv = oracle.prefill(r)
    S = f64(r, "S")
    shared, plain = (("k", ik, uk), ("v", iv, uv)) if share == wl.SHARE_K else (("v", iv, uv), ("k", ik, uk))
    assert shared[2].shape == (40, 2, 3) and plain[2].shape == (40, 2, 10)
    assert (plain[1] == 0).all()
    for h in range(2):
        M = S @ f64(r, "w_r" + shared[0])[h].T + r["b_r" + shared[0]][h]
        np.testing.assert_array_equal(shared[1][:, h], M.argmax(axis=1))
        for side, _, u in (shared, plain):
            np.testing.assert_allclose(u[:, h, :], S @ f64(r, "w_" + side)[h].T + r["b_" + side][h], rtol=1e-12, atol=1e-12)
