"""Pins of the CPU oracle against things other than itself (CPU only).

Each test fixes the oracle to a library routine, a closed form, an invariant or a value the
paper prints, chosen so that a dropped term, a swapped index plane, a wrong column order or
a wrong scale fails at least one of them.
"""
import os

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2601_19178_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small(dtype=wl.F32, mode=wl.SOFTMAX, d_a=16, d_u=3, H=2, P=37, Nq=3, lengths=(5, 1, 0, 9, 64, 2),
          seed=7, idx="uniform", **kw):
    lengths = np.asarray(lengths, dtype=np.int32)
    return wl.make(B=len(lengths), L=None, H=H, d_a=d_a, d_u=d_u, P=P, idx=idx, Nq=Nq, mode=mode,
                   dtype=dtype, sigma_pool=0.5, seed=seed, sigma_user=0.7, lengths=lengths, **kw)


def dense_kv(w):
    """Explicit final K, V per (user, head) in fp64 torch: cat(user slice, pool[index])."""
    dt = w["dtype"]
    uk, uv = (torch.from_numpy(wl.to_f64(w[k], dt)) for k in ("user_k", "user_v"))
    pk, pv = (torch.from_numpy(wl.to_f64(w[k], dt)) for k in ("pool_k", "pool_v"))
    ik, iv = (torch.from_numpy(w[k].astype(np.int64)) for k in ("idx_k", "idx_v"))
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    d_g = w["d_g"]
    for b in range(w["B"]):
        for h in range(w["H"]):
            s = slice(int(off[b]), int(off[b + 1]))
            K = torch.cat([uk[s, h, :], pk[h][ik[s, h]][:, :d_g]], dim=1)
            V = torch.cat([uv[s, h, :], pv[h][iv[s, h]][:, :d_g]], dim=1)
            yield b, h, K, V


def library_attention(w):
    """softmax form: torch's scaled_dot_product_attention; SiLU form: silu(QK^T) V / n."""
    q = torch.from_numpy(wl.to_f64(w["q"], w["dtype"]))
    ref = torch.zeros_like(q)
    for b, h, K, V in dense_kv(w):
        n = K.shape[0]
        if n == 0:
            continue
        if w["mode"] == wl.SOFTMAX:
            ref[b, h] = torch.nn.functional.scaled_dot_product_attention(
                q[b, h][None], K[None], V[None], scale=w["scale"])[0]
        else:
            ref[b, h] = torch.nn.functional.silu(w["scale"] * q[b, h] @ K.T) @ V / n
    return ref.numpy()


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_matches_library_dense_attention(dtype, mode):
    # ragged lengths incl. n = 1 and n = 0, two heads, independent K and V index planes
    w = small(dtype=dtype, mode=mode)
    out = oracle.attend(w)
    np.testing.assert_allclose(out, library_attention(w), rtol=1e-11, atol=1e-13)


def test_config1_matches_library():
    w = wl.config("cfg1")
    assert w["scale"] == 1.0 / 8.0 and w["d_g"] == 56 and w["pool_ld"] == 64
    np.testing.assert_allclose(oracle.attend(w), library_attention(w), rtol=1e-11, atol=1e-13)


def test_zero_length_user_is_zero():
    w = small()
    out = oracle.attend(w)
    assert np.all(out[2] == 0.0)


def test_user_subset_only_touches_listed_users():
    w = small()
    full = oracle.attend(w)
    part = oracle.attend(w, users=[4, 0])
    np.testing.assert_array_equal(part[[4, 0]], full[[4, 0]])
    assert np.all(np.isnan(part[[1, 2, 3, 5]]))


def test_du_zero_is_pure_pool_attention():
    w = small(d_u=0, d_a=12)
    q = torch.from_numpy(w["q"].astype(np.float64))
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    out = oracle.attend(w)
    for b in range(w["B"]):
        s = slice(int(off[b]), int(off[b + 1]))
        if s.start == s.stop:
            continue
        for h in range(w["H"]):
            K = torch.from_numpy(w["pool_k"][h][w["idx_k"][s, h]][:, :12].astype(np.float64))
            V = torch.from_numpy(w["pool_v"][h][w["idx_v"][s, h]][:, :12].astype(np.float64))
            ref = torch.softmax(q[b, h] @ K.T / np.sqrt(12.0), dim=-1) @ V
            np.testing.assert_allclose(out[b, h], ref.numpy(), rtol=1e-11, atol=1e-13)


def test_dg_zero_is_ordinary_attention_over_user_kv():
    # d_u -> d_a: the method degenerates into the original KV (section 5.3)
    w = small(d_u=16, d_a=16)
    assert w["d_g"] == 0
    q = torch.from_numpy(w["q"].astype(np.float64))
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    out = oracle.attend(w)
    for b in range(w["B"]):
        s = slice(int(off[b]), int(off[b + 1]))
        if s.start == s.stop:
            continue
        for h in range(w["H"]):
            K = torch.from_numpy(w["user_k"][s, h].astype(np.float64))
            V = torch.from_numpy(w["user_v"][s, h].astype(np.float64))
            ref = torch.nn.functional.scaled_dot_product_attention(q[b, h][None], K[None], V[None])[0]
            np.testing.assert_allclose(out[b, h], ref.numpy(), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_history_permutation_invariance(mode):
    w = small(mode=mode, lengths=(33, 7))
    rng = np.random.default_rng(3)
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    perm = np.concatenate([off[b] + rng.permutation(int(w["lengths"][b])) for b in range(w["B"])])
    w2 = dict(w)
    for k in ("idx_k", "idx_v", "user_k", "user_v"):
        w2[k] = np.ascontiguousarray(w[k][perm])
    np.testing.assert_allclose(oracle.attend(w2), oracle.attend(w), rtol=1e-12, atol=1e-14)


def test_zero_query_closed_forms():
    # softmax with q = 0 weights every position 1/n: the user columns are the mean of V_u and
    # the pool columns are the index histogram applied to P_v.  SiLU(0) = 0.
    w = small(lengths=(40, 3), Nq=2)
    w["q"] = np.zeros_like(w["q"])
    out = oracle.attend(w)
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    d_u, d_g, P = w["d_u"], w["d_g"], w["P"]
    for b in range(w["B"]):
        s = slice(int(off[b]), int(off[b + 1]))
        n = s.stop - s.start
        for h in range(w["H"]):
            hist = np.bincount(w["idx_v"][s, h], minlength=P).astype(np.float64)
            ref = np.concatenate([w["user_v"][s, h].astype(np.float64).mean(axis=0),
                                  hist @ w["pool_v"][h][:, :d_g].astype(np.float64) / n])
            for j in range(w["Nq"]):
                np.testing.assert_allclose(out[b, h, j], ref, rtol=1e-12, atol=1e-14)
    w["mode"] = wl.SILU_OVER_N
    assert np.all(oracle.attend(w) == 0.0)


def test_constant_value_rows():
    # every final V row equal to [c | v]: softmax returns it for any q; SiLU returns it times
    # sum_i silu(s_i) / n.
    w = small(lengths=(21,), H=1, Nq=2)
    c = np.linspace(-1, 1, w["d_u"]).astype(np.float32)
    v = np.linspace(2, 3, w["d_g"]).astype(np.float32)
    w["user_v"][:] = c
    w["pool_v"][:, :, :w["d_g"]] = v
    row = np.concatenate([c, v]).astype(np.float64)
    out = oracle.attend(w)
    np.testing.assert_allclose(out[0, 0], np.stack([row, row]), rtol=1e-12)
    w["mode"], w["scale"] = wl.SILU_OVER_N, 1.0
    out = oracle.attend(w)
    (_, _, K, _), = list(dense_kv(w))
    s = torch.from_numpy(w["q"][0, 0].astype(np.float64)) @ K.T
    g = (s * torch.sigmoid(s)).sum(dim=1).numpy() / 21
    np.testing.assert_allclose(out[0, 0], g[:, None] * row[None, :], rtol=1e-11)


def test_single_position():
    w = small(lengths=(1, 1), Nq=2)
    out = oracle.attend(w)
    rows = {(b, h): (K, V) for b, h, K, V in dense_kv(w)}
    for (b, h), (K, V) in rows.items():
        for j in range(2):
            np.testing.assert_allclose(out[b, h, j], V[0].numpy(), rtol=1e-14)
    w["mode"], w["scale"] = wl.SILU_OVER_N, 1.0
    out = oracle.attend(w)
    for (b, h), (K, V) in rows.items():
        for j in range(2):
            s = float(np.dot(w["q"][b, h, j].astype(np.float64), K[0].numpy()))
            np.testing.assert_allclose(out[b, h, j], s / (1 + np.exp(-s)) * V[0].numpy(), rtol=1e-12)


def test_dominant_key_selects_its_value_row_through_both_index_planes():
    # Make position i* the only key aligned with q: softmax puts all weight there, so the
    # output is [V_u[i*] | P_v[I_v[i*]]].  I_k and I_v differ, so using the wrong plane, the
    # wrong pool or the wrong column order fails.
    w = small(lengths=(30,), H=1, Nq=1, P=64, d_a=16, d_u=3)
    istar = 17
    w["idx_k"][:, 0] = np.arange(30) % 64
    w["idx_v"][:, 0] = (np.arange(30) * 7 + 5) % 64
    w["user_k"][:] = 0
    w["pool_k"][0, :, :w["d_g"]] = 0
    w["pool_k"][0, w["idx_k"][istar, 0], :w["d_g"]] = 1.0          # only row of i* is non-zero
    w["q"][:] = 0
    w["q"][0, 0, 0, w["d_u"]:] = 50.0                                # acts on the pool columns only
    w["scale"] = 1.0
    out = oracle.attend(w)[0, 0, 0]
    ref = np.concatenate([w["user_v"][istar, 0], w["pool_v"][0, w["idx_v"][istar, 0], :w["d_g"]]])
    np.testing.assert_allclose(out, ref.astype(np.float64), rtol=1e-12, atol=1e-200)


def test_user_columns_come_first():
    # appendix "Discussion of the sharing mechanism": the first d_u dimensions are the
    # user-specific ones.  A query that is non-zero only there must ignore the key pool.
    w = small(lengths=(12,), H=1, Nq=1)
    w["q"][..., w["d_u"]:] = 0
    a = oracle.attend(w)
    w["pool_k"][:, :, :w["d_g"]] += 3.0
    b = oracle.attend(w)
    np.testing.assert_array_equal(a, b)
    w["user_k"][3] += 1.0                        # one position only: a common shift cancels in softmax
    assert not np.allclose(oracle.attend(w), a)


def test_pool_padding_columns_are_ignored():
    w = small(pool_ld=20)
    assert np.isnan(w["pool_k"][0, 0, w["d_g"]:]).all()
    assert np.isfinite(oracle.attend(w)).all()
    w2 = small(pool_ld=13)                       # unpadded: same draws land elsewhere, so compare via library
    np.testing.assert_allclose(oracle.attend(w2), library_attention(w2), rtol=1e-11, atol=1e-13)


def test_rejects_bad_index_and_length():
    w = small()
    w["idx_v"][3, 1] = w["P"]
    with pytest.raises(ValueError):
        oracle.attend(w)
    w = small()
    w["lengths"] = w["lengths"].copy()
    w["lengths"][0] = -1
    with pytest.raises(ValueError):
        oracle.attend(w)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_reconstruct_is_byte_copy_of_user_slice_then_pool_row(dtype):
    w = small(dtype=dtype)
    k_full, v_full = oracle.reconstruct(w)
    d_g = w["d_g"]
    for h in range(w["H"]):
        np.testing.assert_array_equal(
            k_full[:, h], np.concatenate([w["user_k"][:, h], w["pool_k"][h][w["idx_k"][:, h]][:, :d_g]], axis=1))
        np.testing.assert_array_equal(
            v_full[:, h], np.concatenate([w["user_v"][:, h], w["pool_v"][h][w["idx_v"][:, h]][:, :d_g]], axis=1))


def read_paper_cr():
    vals = []
    with open(os.path.join(GOLDEN, "compression_rates.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            vals += [float(x) for x in line.split()[1:] if x != "-"]
    return vals


def test_compression_rate_matches_paper_table():
    # Every CR the paper prints is (d_u + 1) / d_a for an integer d_u at d_a = 256 (the K/V
    # dimension quoted in section 3.2), with one index counted as one element per K and V
    # (section 4.4).  The smallest is the abstract's 0.8 %.
    printed = read_paper_cr()
    assert len(printed) == 14 and min(printed) == 0.008
    reachable = {}
    for d_u in range(0, 32):
        se, fe, _, _ = oracle.cache_size(T=1000, H=3, d_g=256 - d_u, d_u=d_u, dtype=oracle.F32)
        reachable[round(se / fe, 3)] = d_u
        assert se * 256 == fe * (d_u + 1)
    assert all(cr in reachable for cr in printed), (printed, reachable)
    assert sorted({reachable[cr] for cr in printed}) == [1, 2, 3, 4, 6, 10]


@pytest.mark.parametrize("name,byte_cr,elem_cr", [
    ("cfg1", 0.140625, 9 / 64), ("cfg2_f32", 0.140625, 9 / 64), ("cfg2_bf16", 0.15625, 9 / 64),
    ("cfg3", 0.09375, 5 / 64), ("cfg4", 0.078125, 9 / 128), ("cfg5", 0.0625, 3 / 64)])
def test_compression_rate_of_the_workloads(name, byte_cr, elem_cr):
    r = wl.CONFIGS[name]
    se, fe, sb, fb = oracle.cache_size(T=12345, H=r["H"], d_g=r["d_a"] - r["d_u"], d_u=r["d_u"], dtype=r["dtype"])
    assert se / fe == elem_cr
    assert sb / fb == byte_cr


# ---------------------------------------------------------------------------------------------
# sharing only keys or only values (ablation "sharing keys or values": CollectiveK, CollectiveV)
def dense_kv_shared(w):
    """Explicit final K, V per (user, head): a shared side is cat(user slice, pool[index]); a side that is
    not shared is its own d_a-wide array, untouched."""
    dt = w["dtype"]
    (d_uk, d_gk), (d_uv, d_gv) = wl.side_dims(w["d_u"], w["d_g"], w["share"])
    uk, uv = (torch.from_numpy(wl.to_f64(w[k], dt)) for k in ("user_k", "user_v"))
    pk, pv = (torch.from_numpy(wl.to_f64(w[k], dt)) for k in ("pool_k", "pool_v"))
    ik, iv = (torch.from_numpy(w[k].astype(np.int64)) for k in ("idx_k", "idx_v"))
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    for b in range(w["B"]):
        for h in range(w["H"]):
            s = slice(int(off[b]), int(off[b + 1]))
            K = torch.cat([uk[s, h, :], pk[h][ik[s, h]][:, :d_gk]], dim=1) if d_gk else uk[s, h, :]
            V = torch.cat([uv[s, h, :], pv[h][iv[s, h]][:, :d_gv]], dim=1) if d_gv else uv[s, h, :]
            yield b, h, K, V


@pytest.mark.parametrize("share", [wl.SHARE_K, wl.SHARE_V])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_single_side_sharing_matches_library_attention(share, mode):
    w = small(dtype=wl.BF16, mode=mode, share=share)
    assert w["user_k"].shape[2] == (3 if share == wl.SHARE_K else 16)
    assert w["user_v"].shape[2] == (16 if share == wl.SHARE_K else 3)
    q = torch.from_numpy(wl.to_f64(w["q"], w["dtype"]))
    ref = torch.zeros_like(q)
    for b, h, K, V in dense_kv_shared(w):
        assert K.shape[1] == 16 and V.shape[1] == 16
        if K.shape[0] == 0:
            continue
        if mode == wl.SOFTMAX:
            ref[b, h] = torch.nn.functional.scaled_dot_product_attention(q[b, h][None], K[None], V[None], scale=w["scale"])[0]
        else:
            ref[b, h] = torch.nn.functional.silu(w["scale"] * q[b, h] @ K.T) @ V / K.shape[0]
    np.testing.assert_allclose(oracle.attend(w), ref.numpy(), rtol=1e-11, atol=1e-13)


def test_unshared_side_fed_with_reconstructed_rows_gives_the_shared_result():
    """A cache that shares both sides, and the same cache with its V rows (or K rows) materialised and handed
    over as an ordinary cache, are the same attention problem."""
    w = small(dtype=wl.F32)
    ref = oracle.attend(w)
    k_full, v_full = oracle.reconstruct(w)
    wk = dict(w, share=wl.SHARE_K, user_v=v_full)
    wv = dict(w, share=wl.SHARE_V, user_k=k_full)
    np.testing.assert_array_equal(oracle.attend(wk), ref)
    np.testing.assert_array_equal(oracle.attend(wv), ref)
    for w2 in (wk, wv):
        k2, v2 = oracle.reconstruct(w2)
        np.testing.assert_array_equal(k2, k_full)
        np.testing.assert_array_equal(v2, v_full)


def test_cache_size_with_one_side_shared():
    # the shared side stores d_u + 1 elements per position, the ordinary side d_a
    se, fe, sb, fb = oracle.cache_size(T=100, H=2, d_g=56, d_u=8, dtype=oracle.BF16, share=wl.SHARE_K)
    assert (se, fe) == (100 * 2 * (8 + 1 + 64), 100 * 2 * 128)
    assert (sb, fb) == (100 * 2 * (8 * 2 + 4 + 64 * 2), 100 * 2 * 128 * 2)
    assert oracle.cache_size(T=100, H=2, d_g=56, d_u=8, dtype=oracle.BF16, share=wl.SHARE_V) == (se, fe, sb, fb)
    both = oracle.cache_size(T=100, H=2, d_g=56, d_u=8, dtype=oracle.BF16)
    assert both[0] == 100 * 2 * 2 * 9 and both[0] < se


# ---------------------------------------------------------------------------------------------
# frequency renumbering of pool rows: a relabeling, so attention must not change
def test_hot_row_renumbering_is_a_relabeling():
    w = small(dtype=wl.BF16, idx=("zipf", 1.2), lengths=(40, 3, 0, 77, 64, 9), P=23)
    nk, nv = oracle.hot_row_order(w)
    ref = oracle.attend(w)
    w2 = dict(w)
    w2["pool_k"], w2["pool_v"] = np.empty_like(w["pool_k"]), np.empty_like(w["pool_v"])
    for h in range(w["H"]):
        assert sorted(nk[h]) == list(range(w["P"])) and sorted(nv[h]) == list(range(w["P"]))
        w2["pool_k"][h][nk[h]] = w["pool_k"][h]
        w2["pool_v"][h][nv[h]] = w["pool_v"][h]
        # most used first: counts are non-increasing along the new numbering, ties by old row number
        for new_id, idx in ((nk, w["idx_k"]), (nv, w["idx_v"])):
            counts = np.bincount(idx[:, h], minlength=w["P"])
            by_new = np.empty(w["P"], dtype=np.int64)
            by_new[new_id[h]] = counts
            assert (np.diff(by_new) <= 0).all()
            old_of_new = np.argsort(new_id[h])
            same = np.diff(by_new) == 0
            assert (np.diff(old_of_new)[same] > 0).all()
    w2["idx_k"] = np.stack([nk[h][w["idx_k"][:, h]] for h in range(w["H"])], axis=1).astype(np.int32)
    w2["idx_v"] = np.stack([nv[h][w["idx_v"][:, h]] for h in range(w["H"])], axis=1).astype(np.int32)
    np.testing.assert_array_equal(oracle.attend(w2), ref)   # same rows, same order of summation: bit for bit
    ok, ov = oracle.reconstruct(w)
    ok2, ov2 = oracle.reconstruct(w2)
    np.testing.assert_array_equal(ok, ok2)
    np.testing.assert_array_equal(ov, ov2)


# ---------------------------------------------------------------------------------------------
# split-history merge identity (online softmax): the oracle on chunks of a history, joined by the
# (m, l, acc) rule written out here, equals the oracle on the whole history
def _scores(w, b, h):
    """scale * q K^T of one (user, head), fp64 numpy [Nq][n], from explicitly concatenated K rows."""
    for bb, hh, K, _ in dense_kv(w):
        if (bb, hh) == (b, h):
            return w["scale"] * wl.to_f64(w["q"], w["dtype"])[b, h] @ K.numpy().T
    raise KeyError((b, h))


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("cuts", [(0, 1, 38, 64, 97), (0, 96, 97), (0, 50, 97), (0, 97)])
def test_chunks_merged_by_max_sum_acc_equal_the_whole_history(dtype, mode, cuts):
    n = cuts[-1]
    w = small(dtype=dtype, mode=mode, lengths=(n,), H=2, Nq=3, P=11)
    whole = oracle.attend(w)[0]                                   # [H][Nq][d_a]
    merged = np.zeros_like(whole)
    for h in range(w["H"]):
        s = _scores(w, 0, h)                                      # [Nq][n]
        m_c, l_c, acc_c = [], [], []
        for lo, hi in zip(cuts[:-1], cuts[1:]):                   # the first chunk of the first case has one position
            wc = dict(w)
            wc["lengths"] = np.array([hi - lo], np.int32)
            for k in ("idx_k", "idx_v", "user_k", "user_v"):
                wc[k] = np.ascontiguousarray(w[k][lo:hi])
            part = oracle.attend(wc)[0, h]                        # the chunk's own normalised output
            if mode == wl.SOFTMAX:
                m = s[:, lo:hi].max(axis=1)
                l = np.exp(s[:, lo:hi] - m[:, None]).sum(axis=1)
                m_c.append(m); l_c.append(l); acc_c.append(part * l[:, None])   # acc relative to the chunk maximum
            else:
                acc_c.append(part * (hi - lo))                    # undo the chunk's 1/n
        if mode == wl.SOFTMAX:
            M = np.max(np.stack(m_c), axis=0)
            scale_c = [np.exp(m - M) for m in m_c]
            denom = sum(a * l for a, l in zip(scale_c, l_c))
            merged[h] = sum(a[:, None] * acc for a, acc in zip(scale_c, acc_c)) / denom[:, None]
        else:
            merged[h] = sum(acc_c) / n
    np.testing.assert_allclose(merged, whole, rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------------------------------------
# the per-element scale of the comparison rule: root-sum-square of an element's summands
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("share", [wl.SHARE_KV, wl.SHARE_K, wl.SHARE_V])
def test_summand_scale_matches_explicit_weights(dtype, mode, share):
    w = small(dtype=dtype, mode=mode, share=share)
    out, rss = oracle.attend(w, with_rss=True)
    np.testing.assert_array_equal(out, oracle.attend(w))          # the extra output changes nothing
    q = wl.to_f64(w["q"], dtype)
    for b, h, K, V in dense_kv_shared(w):
        n = K.shape[0]
        if n == 0:
            assert np.all(rss[b, h] == 0)
            continue
        s = torch.from_numpy(w["scale"] * q[b, h]) @ K.T
        wt = torch.softmax(s, dim=-1) if mode == wl.SOFTMAX else torch.nn.functional.silu(s) / n
        terms = wt[:, :, None] * V[None, :, :]                    # [Nq][n][d_a]
        # the random workload has no two equal weights: every position is a group of its own
        np.testing.assert_allclose(rss[b, h], terms.pow(2).sum(dim=1).sqrt().numpy(), rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(out[b, h], terms.sum(dim=1).numpy(), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_summand_scale_groups_positions_of_equal_weight(mode):
    # no user columns and a key pool of three rows: a query sees at most three different weights, however long the
    # history; positions that share a weight form one group whose summands are added before squaring
    w = small(mode=mode, d_u=0, d_a=12, P=3, lengths=(50, 7), H=1, Nq=2)
    out, rss = oracle.attend(w, with_rss=True)
    q = wl.to_f64(w["q"], w["dtype"])
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    for b, h, K, V in dense_kv(w):
        n, V = K.shape[0], V.numpy()
        s = (w["scale"] * q[b, h]) @ K.numpy().T
        wt = torch.softmax(torch.from_numpy(s), dim=-1).numpy() if mode == wl.SOFTMAX else s / (1 + np.exp(-s)) / n
        rows = w["idx_k"][off[b]:off[b + 1], h]                   # the key row decides the weight
        for j in range(w["Nq"]):
            groups = np.stack([(wt[j][rows == r, None] * V[rows == r]).sum(axis=0) for r in np.unique(rows)])
            assert len(np.unique(wt[j])) == len(groups) <= 3
            np.testing.assert_allclose(rss[b, h, j], np.sqrt((groups ** 2).sum(axis=0)), rtol=1e-11, atol=1e-14)


def test_summand_scale_closed_forms():
    # one position: the only summand is the output itself
    w = small(lengths=(1,), Nq=2)
    out, rss = oracle.attend(w, with_rss=True)
    np.testing.assert_allclose(rss, np.abs(out), rtol=1e-14)
    # q = 0, softmax: every weight is 1/n, one group, so the scale is the output itself
    w = small(lengths=(40,), H=1, Nq=1)
    w["q"] = np.zeros_like(w["q"])
    out, rss = oracle.attend(w, with_rss=True)
    np.testing.assert_allclose(rss, np.abs(out), rtol=1e-12)
    # users not listed stay NaN, like out
    w = small()
    _, rss = oracle.attend(w, users=[1], with_rss=True)
    assert np.isnan(rss[0]).all() and np.isfinite(rss[1]).all()


# ---------------------------------------------------------------------------------------------
# the scale of the scores' rounding errors: first-order effect of an error delta_i * A_i of score i on the output
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("share", [wl.SHARE_KV, wl.SHARE_K])
def test_score_scale_matches_autograd_jacobian(dtype, mode, share):
    """d out[c] / d s_i from torch's autograd through torch's own softmax / SiLU, times A_i = |scale| sum_k |q_k K_ik|;
    the random workload has no two equal rows, so every position is a group of its own."""
    w = small(dtype=dtype, mode=mode, share=share)
    out, rss, sss, _ = oracle.attend(w, with_scales=True)
    o2, r2 = oracle.attend(w, with_rss=True)
    np.testing.assert_array_equal(out, o2)                        # the extra outputs change nothing
    np.testing.assert_array_equal(rss, r2)
    q = wl.to_f64(w["q"], dtype)
    for b, h, K, V in dense_kv_shared(w):
        n = K.shape[0]
        if n == 0:
            assert np.all(sss[b, h] == 0)
            continue
        for j in range(w["Nq"]):
            qj = torch.from_numpy(q[b, h, j])
            s0 = (w["scale"] * qj) @ K.T
            A = abs(w["scale"]) * (qj.abs()[None, :] * K.abs()).sum(dim=1)

            def f(s):
                wt = torch.softmax(s, dim=-1) if mode == wl.SOFTMAX else torch.nn.functional.silu(s) / n
                return wt @ V
            J = torch.autograd.functional.jacobian(f, s0)          # [d_a][n]
            want = ((J * A[None, :]) ** 2).sum(dim=1).sqrt().numpy()
            np.testing.assert_allclose(sss[b, h, j], want, rtol=1e-9, atol=1e-14)


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_score_scale_groups_positions_of_equal_score(mode):
    # a key pool of three rows and no user columns: positions with the same key row have the same score and the same
    # error, so their effects are added before squaring
    w = small(mode=mode, d_u=0, d_a=12, P=3, lengths=(50, 7), H=1, Nq=2)
    out, _, sss, _ = oracle.attend(w, with_scales=True)
    q = wl.to_f64(w["q"], w["dtype"])
    off = np.concatenate([[0], np.cumsum(w["lengths"])])
    for b, h, K, V in dense_kv(w):
        n = K.shape[0]
        rows = w["idx_k"][off[b]:off[b + 1], h]
        for j in range(w["Nq"]):
            qj = torch.from_numpy(q[b, h, j])
            s0 = (w["scale"] * qj) @ K.T
            A = abs(w["scale"]) * (qj.abs()[None, :] * K.abs()).sum(dim=1)

            def f(s):
                wt = torch.softmax(s, dim=-1) if mode == wl.SOFTMAX else torch.nn.functional.silu(s) / n
                return wt @ V
            JA = (torch.autograd.functional.jacobian(f, s0) * A[None, :]).numpy()   # [d_a][n]
            groups = np.stack([JA[:, rows == r].sum(axis=1) for r in np.unique(rows)])
            np.testing.assert_allclose(sss[b, h, j], np.sqrt((groups ** 2).sum(axis=0)), rtol=1e-9, atol=1e-14)


def test_score_scale_closed_forms():
    # softmax over one position: the weight is 1 whatever the score, an error of the score changes nothing
    w = small(lengths=(1,), Nq=2, mode=wl.SOFTMAX)
    _, _, sss, _ = oracle.attend(w, with_scales=True)
    assert np.all(sss == 0)
    # SiLU over one position: out = f(s) V, so the scale is |f'(s)| A |V| with f'(s) = sigma (1 + s (1 - sigma))
    w = small(lengths=(1,), Nq=2, mode=wl.SILU_OVER_N, H=1)
    _, _, sss, _ = oracle.attend(w, with_scales=True)
    q = wl.to_f64(w["q"], w["dtype"])
    for b, h, K, V in dense_kv(w):
        K, V = K.numpy()[0], V.numpy()[0]
        for j in range(2):
            s = w["scale"] * q[b, h, j] @ K
            A = abs(w["scale"]) * np.abs(q[b, h, j] * K).sum()
            sg = 1 / (1 + np.exp(-s))
            np.testing.assert_allclose(sss[b, h, j], abs(sg * (1 + s * (1 - sg))) * A * np.abs(V), rtol=1e-12)
    # q = 0: A = 0, no error to propagate
    w = small(lengths=(40,), H=1, Nq=1)
    w["q"] = np.zeros_like(w["q"])
    _, _, sss, _ = oracle.attend(w, with_scales=True)
    assert np.all(sss == 0)


# ---------------------------------------------------------------------------------------------
# the scale of the roundings of the output's own additions: sqrt(n) (|out| + root-sum-square of the summands one by one)
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("share", [wl.SHARE_KV, wl.SHARE_V])
def test_addition_scale_matches_explicit_weights(dtype, mode, share):
    w = small(dtype=dtype, mode=mode, share=share)
    out, rss, _, acs = oracle.attend(w, with_scales=True)
    q = wl.to_f64(w["q"], dtype)
    for b, h, K, V in dense_kv_shared(w):
        n = K.shape[0]
        if n == 0:
            assert np.all(acs[b, h] == 0)
            continue
        s = torch.from_numpy(w["scale"] * q[b, h]) @ K.T
        wt = torch.softmax(s, dim=-1) if mode == wl.SOFTMAX else torch.nn.functional.silu(s) / n
        terms = wt[:, :, None] * V[None, :, :]                    # [Nq][n][d_a]
        want = np.sqrt(n) * (terms.sum(dim=1).abs() + terms.pow(2).sum(dim=1).sqrt()).numpy()
        np.testing.assert_allclose(acs[b, h], want, rtol=1e-11, atol=1e-14)


def test_addition_scale_does_not_group_equal_weights():
    # q = 0, softmax: every weight is 1/n.  The weights' scale collapses to |out| (one group); the additions' scale
    # still sees every summand: sqrt(n) (|mean_i V_i| + sqrt(sum_i V_i^2) / n)
    w = small(lengths=(40,), H=1, Nq=1)
    w["q"] = np.zeros_like(w["q"])
    out, rss, _, acs = oracle.attend(w, with_scales=True)
    for b, h, K, V in dense_kv(w):
        V = V.numpy()
        np.testing.assert_allclose(acs[b, h, 0], np.sqrt(40) * (np.abs(V.mean(axis=0)) + np.sqrt((V ** 2).sum(axis=0)) / 40), rtol=1e-12)
    np.testing.assert_allclose(rss, np.abs(out), rtol=1e-12)
    # one position: the sum has one summand, the scale is twice its size
    w = small(lengths=(1,), Nq=2)
    out, _, _, acs = oracle.attend(w, with_scales=True)
    np.testing.assert_allclose(acs, 2 * np.abs(out), rtol=1e-14)
    # users not listed stay NaN, like out
    w = small()
    _, _, _, acs = oracle.attend(w, users=[1], with_scales=True)
    assert np.isnan(acs[0]).all() and np.isfinite(acs[1]).all()


# ---------------------------------------------------------------------------------------------
# the sum of the magnitudes of an element's summands (the bound on what rounding the weights can do to it)
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("share", [wl.SHARE_KV, wl.SHARE_K])
def test_magnitude_sum_matches_explicit_weights(dtype, mode, share):
    w = small(dtype=dtype, mode=mode, share=share)
    out, rss, _, acs, asum = oracle.attend(w, with_scales=True, with_asum=True)
    q = wl.to_f64(w["q"], dtype)
    for b, h, K, V in dense_kv_shared(w):
        n = K.shape[0]
        if n == 0:
            assert np.all(asum[b, h] == 0)
            continue
        s = torch.from_numpy(w["scale"] * q[b, h]) @ K.T
        wt = torch.softmax(s, dim=-1) if mode == wl.SOFTMAX else torch.nn.functional.silu(s) / n
        want = (wt[:, :, None] * V[None, :, :]).abs().sum(dim=1).numpy()
        np.testing.assert_allclose(asum[b, h], want, rtol=1e-11, atol=1e-14)
    # it bounds the output and the grouped root-sum-square from above, and a planted mistake (signed sum) would not
    assert (asum >= np.abs(out) * (1 - 1e-12)).all() and (asum >= rss * (1 - 1e-12)).all()
    assert (asum > np.abs(out) * 1.01).any()


def test_magnitude_sum_special_cases():
    # one position: the magnitude of the one summand
    w = small(lengths=(1,), Nq=2)
    out, _, _, _, asum = oracle.attend(w, with_scales=True, with_asum=True)
    np.testing.assert_allclose(asum, np.abs(out), rtol=1e-14)
    # q = 0, softmax: every weight is 1/n: the mean of |V_i|
    w = small(lengths=(40,), H=1, Nq=1)
    w["q"] = np.zeros_like(w["q"])
    _, _, _, _, asum = oracle.attend(w, with_scales=True, with_asum=True)
    for b, h, K, V in dense_kv(w):
        np.testing.assert_allclose(asum[b, h, 0], np.abs(V.numpy()).mean(axis=0), rtol=1e-12)
    # users not listed stay NaN, like out; without with_asum the call returns four arrays as before
    w = small()
    r = oracle.attend(w, users=[1], with_scales=True, with_asum=True)
    assert np.isnan(r[4][0]).all() and np.isfinite(r[4][1]).all()
    assert len(oracle.attend(w, with_scales=True)) == 4
