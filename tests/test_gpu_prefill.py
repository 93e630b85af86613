"""GPU parity of the prefill stage (projection + router argmax written into the packed cache) through
the C ABI against the CPU oracle.

Indices are integers decided by floating point: on inputs whose sums are exact in fp32 (small integers)
both sides must agree bit for bit, ties included; on random inputs the GPU forms the routing map in fp32
and the oracle in fp64, so an index may differ where two scores are closer than the fp32 rounding of
their sums: there the GPU's pick must be within that rounding of the row maximum (its validity), and
nearly all indices must still be identical.
"""
import sys

import numpy as np
import pytest

from oracle import oracle
from paper_2601_19178_amd import workloads as wl
from tests.parity import check_against_oracle

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2601_19178_amd import ckv, session
    return ckv, session


def decode_workload(lengths, r, Nq=2, mode=wl.SOFTMAX, d_g=None, seed=31):
    """A decode workload whose cache shape matches the prefill workload r."""
    lengths = np.asarray(lengths, dtype=np.int32)
    if r.get("share", 0) != wl.SHARE_KV:
        d_g = r["d_a"] - r["d_u"]
    d_g = (56 if r["P"] > 1 else 0) if d_g is None else d_g
    d_a = d_g + r["d_u"]
    return wl.make(B=len(lengths), L=None, H=r["H"], d_a=d_a, d_u=r["d_u"], P=r["P"], idx="uniform", Nq=Nq, mode=mode,
                   dtype=r["dtype"], sigma_pool=max(d_a, 1) ** -0.5, seed=seed, lengths=lengths, share=r.get("share", 0))


def user_tolerance(ref, dtype):
    # fp32 accumulation of d_e <= 256 products of magnitude ~0.1 (worst case d_e * 2^-24 of their absolute sum,
    # ~2^-16 of a result of order one), then one rounding to the storage type (2^-9 for bf16)
    eps = 2.0 ** -8 if dtype == wl.BF16 else 2.0 ** -16
    return eps * np.abs(ref) + eps


def run_prefill(gpu, lengths, r, what, expect_kernel, exact, d_g=None):
    ckv, session = gpu
    w = decode_workload(lengths, r, d_g=d_g)
    say(f"[case] {what}: T={r['T']} H={r['H']} d_e={r['d_e']} d_u={r['d_u']} P={r['P']} dtype={r['dtype']} d_g={w['d_g']}")
    with session.Session(w, prefill=r) as s:
        name = ckv.ckv_prefill_kernel_name(s.shape, s.router)
        say(f"  kernel {name}")
        assert name.startswith(expect_kernel), name
        idx, uk, uv = s.packed_views()
        # the handle works like any other: attend over the cache the prefill wrote
        s.attend()
        out = s.output()
    ik, iv, ruk, ruv = oracle.prefill(r)
    T, H = r["T"], r["H"]
    if w["d_g"] > 0:
        shared_sides = {wl.SHARE_KV: "kv", wl.SHARE_K: "k", wl.SHARE_V: "v"}[w["share"]]
        for side, got, ref in (("k", idx[0].T, ik), ("v", idx[1].T, iv)):
            if side not in shared_sides:
                continue
            assert got.size == 0 or (got.min() >= 0 and got.max() < r["P"])
            same = float((got == ref).mean()) if got.size else 1.0
            if exact:
                np.testing.assert_array_equal(got, ref, err_msg=f"{what}: I_{side}")
            else:
                gap, mag = oracle.router_gap(r, side, np.ascontiguousarray(got))
                bound = (r["d_e"] + 2) * 2.0 ** -23 * mag
                assert (gap <= bound).all(), f"{what}: I_{side}: a pick is {float((gap - bound).max()):.3e} beyond fp32 rounding of the maximum"
                assert same > 0.995, f"{what}: I_{side}: only {same:.4f} of the indices equal the fp64 argmax"
            say(f"  I_{side}: {same:.5f} identical to the oracle")
    sdt = np.float32 if r["dtype"] == wl.F32 else np.uint16
    guk = wl.to_f64(uk.astype(sdt), r["dtype"]).transpose(1, 0, 2)
    guv = wl.to_f64(uv.astype(sdt), r["dtype"]).transpose(1, 0, 2)
    for side, got, ref in (("k", guk, ruk), ("v", guv, ruv)):
        if exact:
            want = ref.astype(np.float32)
            want = want.astype(np.float64) if r["dtype"] == wl.F32 else wl.to_f64(wl.f32_to_bf16_bits(want), wl.BF16)
            np.testing.assert_array_equal(got, want, err_msg=f"{what}: {side.upper()}_u")
        else:
            assert (np.abs(got - ref) <= user_tolerance(ref, r["dtype"])).all(), f"{what}: {side.upper()}_u out of tolerance"
    # decode over exactly what the prefill cached
    if T > 0:
        w2 = dict(w)
        if w["d_g"] > 0:
            if w["share"] in (wl.SHARE_KV, wl.SHARE_K):
                w2["idx_k"] = np.ascontiguousarray(idx[0].T)
            if w["share"] in (wl.SHARE_KV, wl.SHARE_V):
                w2["idx_v"] = np.ascontiguousarray(idx[1].T)
        w2["user_k"] = np.ascontiguousarray(uk.astype(sdt).transpose(1, 0, 2))
        w2["user_v"] = np.ascontiguousarray(uv.astype(sdt).transpose(1, 0, 2))
        check_against_oracle(out, w2, what=what + " (decode over the prefilled cache)")
    say("  ok")


LENGTHS = (5, 0, 300, 1, 64, 257, 33)   # T = 660: three position blocks of 256 and a ragged tail


@pytest.mark.parametrize("d_e,d_u,P,H", [(64, 8, 1000, 2), (128, 3, 77, 3), (128, 8, 4096, 1), (256, 32, 333, 2),
                                          (64, 0, 31, 1), (128, 16, 32, 2), (256, 2, 5, 1)])
def test_mfma_exact_on_integer_inputs(gpu, d_e, d_u, P, H):
    r = wl.make_prefill(T=sum(LENGTHS), H=H, d_e=d_e, d_u=d_u, P=P, dtype=wl.BF16, seed=40 + d_u, integers=1)
    run_prefill(gpu, LENGTHS, r, f"prefill mfma exact d_e={d_e} d_u={d_u} P={P}", "prefill_mfma_bf16", exact=True)


@pytest.mark.parametrize("d_e,d_u,P,H", [(64, 8, 1000, 2), (128, 4, 4099, 2), (256, 8, 500, 1)])
def test_mfma_random_inputs(gpu, d_e, d_u, P, H):
    r = wl.make_prefill(T=sum(LENGTHS), H=H, d_e=d_e, d_u=d_u, P=P, dtype=wl.BF16, seed=50 + d_u)
    run_prefill(gpu, LENGTHS, r, f"prefill mfma random d_e={d_e} d_u={d_u} P={P}", "prefill_mfma_bf16", exact=False)


@pytest.mark.parametrize("d_e,d_u,P,H,integers", [(64, 8, 1000, 2, 1), (128, 3, 77, 3, 2), (128, 8, 4096, 1, 1), (256, 32, 333, 2, 1),
                                                   (64, 4, 2049, 2, None), (128, 8, 1000, 2, None), (256, 5, 500, 1, None)])
def test_mfma_fp32_storage(gpu, d_e, d_u, P, H, integers):
    """fp32 embeddings and weights on the fp32 matrix instruction: exact on integer inputs, within the fp32
    rounding bound on random ones."""
    r = wl.make_prefill(T=sum(LENGTHS), H=H, d_e=d_e, d_u=d_u, P=P, dtype=wl.F32, seed=140 + d_u, integers=integers)
    run_prefill(gpu, LENGTHS, r, f"prefill mfma fp32 d_e={d_e} d_u={d_u} P={P} integers={integers}", "prefill_mfma_f32",
                exact=integers is not None)


def expected_kernel(dtype, d_e):
    """Matrix-core kernel for rows of whole 16-byte chunks up to 256 columns, scalar kernel otherwise."""
    es = 4 if dtype == wl.F32 else 2
    if d_e <= 256 and (d_e * es) % 16 == 0:
        return ("prefill_mfma_f32" if dtype == wl.F32 else "prefill_mfma_bf16") + f"_e{64 if d_e <= 64 else (128 if d_e <= 128 else 256)}"
    return "prefill_scalar"


@pytest.mark.parametrize("dtype,d_e,d_u,P,integers", [(wl.F32, 25, 3, 61, 2), (wl.F32, 300, 8, 300, None),
                                                       (wl.BF16, 36, 5, 129, 2), (wl.BF16, 260, 2, 50, None)])
def test_scalar_kernel(gpu, dtype, d_e, d_u, P, integers):
    lengths = (5, 0, 120, 1, 64)
    r = wl.make_prefill(T=sum(lengths), H=2, d_e=d_e, d_u=d_u, P=P, dtype=dtype, seed=60 + d_e, integers=integers)
    run_prefill(gpu, lengths, r, f"prefill scalar dtype={dtype} d_e={d_e}", "prefill_scalar", exact=integers is not None)


@pytest.mark.parametrize("dtype,d_e,d_u,P,integers", [(wl.F32, 24, 3, 61, 2), (wl.F32, 100, 8, 300, None), (wl.F32, 4, 2, 40, 2),
                                                       (wl.BF16, 40, 5, 129, 2), (wl.BF16, 72, 2, 50, None), (wl.BF16, 8, 1, 33, 2),
                                                       (wl.BF16, 200, 8, 1000, None), (wl.F32, 192, 4, 700, 1)])
def test_narrow_rows_run_in_the_next_wider_kernel(gpu, dtype, d_e, d_u, P, integers):
    """An embedding narrower than the width a kernel is built for: its missing columns count as zeros."""
    r = wl.make_prefill(T=sum(LENGTHS), H=2, d_e=d_e, d_u=d_u, P=P, dtype=dtype, seed=160 + d_e, integers=integers)
    run_prefill(gpu, LENGTHS, r, f"prefill narrow rows dtype={dtype} d_e={d_e}", expected_kernel(dtype, d_e), exact=integers is not None)


def test_no_pool_and_no_user_columns(gpu):
    # d_g = 0: "degenerates into the original KV" (only the projection); d_u = 0: only the router
    r = wl.make_prefill(T=sum(LENGTHS), H=2, d_e=64, d_u=16, P=1, dtype=wl.BF16, seed=70, integers=1)
    run_prefill(gpu, LENGTHS, r, "prefill d_g=0", "prefill_mfma_bf16", exact=True, d_g=0)
    r = wl.make_prefill(T=sum(LENGTHS), H=2, d_e=128, d_u=0, P=200, dtype=wl.BF16, seed=71, integers=1)
    run_prefill(gpu, LENGTHS, r, "prefill d_u=0", "prefill_mfma_bf16", exact=True, d_g=64)


@pytest.mark.parametrize("share", [wl.SHARE_K, wl.SHARE_V])
def test_prefill_with_one_side_shared(gpu, share):
    # the side that is not shared has no router; its projection has d_a rows (several 32-column tiles)
    r = wl.make_prefill(T=sum(LENGTHS), H=2, d_e=128, d_u=8, P=1000, dtype=wl.BF16, seed=80, integers=1, share=share, d_a=64)
    run_prefill(gpu, LENGTHS, r, f"prefill mfma exact share={share}", "prefill_mfma_bf16", exact=True)
    r = wl.make_prefill(T=sum(LENGTHS), H=2, d_e=64, d_u=3, P=333, dtype=wl.BF16, seed=81, share=share, d_a=40)
    run_prefill(gpu, LENGTHS, r, f"prefill mfma random share={share}", "prefill_mfma_bf16", exact=False)
    r = wl.make_prefill(T=200, H=2, d_e=24, d_u=3, P=61, dtype=wl.F32, seed=82, integers=2, share=share, d_a=16)
    run_prefill(gpu, (5, 0, 131, 64), r, f"prefill fp32 narrow exact share={share}", "prefill_mfma_f32_e64", exact=True)
    r = wl.make_prefill(T=200, H=2, d_e=25, d_u=3, P=61, dtype=wl.F32, seed=83, integers=2, share=share, d_a=16)
    run_prefill(gpu, (5, 0, 131, 64), r, f"prefill scalar exact share={share}", "prefill_scalar", exact=True)


def test_all_histories_empty(gpu):
    r = wl.make_prefill(T=0, H=2, d_e=64, d_u=8, P=100, dtype=wl.BF16, seed=72)
    run_prefill(gpu, (0, 0, 0), r, "prefill T=0", "prefill_mfma_bf16", exact=True)


def test_prefill_into_recomputes_in_place(gpu):
    ckv, session = gpu
    r = wl.make_prefill(T=sum(LENGTHS), H=2, d_e=128, d_u=8, P=1000, dtype=wl.BF16, seed=73)
    w = decode_workload(LENGTHS, r)
    say("[case] prefill_into")
    with session.Session(w, prefill=r) as s:
        first = [a.copy() for a in s.packed_views()]
        import torch
        # overwrite the packed cache, then recompute it
        n = 2 * r["H"] * r["T"]
        junk = torch.full((n,), 7, dtype=torch.int32, device="cuda")
        ckv.ckv_copy(ckv.ckv_cache_idx(s.cache), junk, n * 4, s.stream)
        torch.cuda.synchronize()
        assert (s.packed_views()[0] == 7).all()
        s.prefill_again()
        again = s.packed_views()
    for a, b in zip(first, again):
        np.testing.assert_array_equal(a, b)


def test_router_rejects_bad_arguments(gpu):
    ckv, session = gpu
    import torch
    r = wl.make_prefill(T=10, H=1, d_e=64, d_u=8, P=10, dtype=wl.BF16, seed=74)
    w = decode_workload((10,), r)
    sh = ckv.make_shape(w["B"], w["H"], w["d_g"], w["d_u"], w["P"], w["Nq"], w["dtype"], w["mode"], w["scale"], w["pool_ld"])
    S = torch.zeros((10, 64), dtype=torch.bfloat16, device="cuda")
    z = torch.zeros(64 * 64, dtype=torch.float32, device="cuda")
    with pytest.raises(ckv.CkvError) as e:
        ckv.ckv_prefill(sh, ckv.make_router(64, None, z, z, z, z, z, z, z), w["lengths"], S)
    assert e.value.code == ckv.CKV_ERR_NULL
    with pytest.raises(ckv.CkvError) as e:
        ckv.ckv_prefill(sh, ckv.make_router(0, z, z, z, z, z, z, z, z), w["lengths"], S)
    assert e.value.code == ckv.CKV_ERR_SHAPE
    with pytest.raises(ckv.CkvError) as e:
        ckv.ckv_prefill(sh, ckv.make_router(64, z, z, z, z, z, z, z, z), w["lengths"], S.data_ptr() + 2)
    assert e.value.code == ckv.CKV_ERR_UNSUPPORTED


def test_full_size_prefill_sampled(gpu):
    """The workload the benchmark times (config 2's cache: B=1024, L=200, H=2, d_u=8, P=4096; d_e=128),
    oracle on sampled positions."""
    ckv, session = gpu
    r = wl.prefill_config("prefill_cfg2")
    w = wl.config("cfg2_bf16")
    say(f"[case] full-size prefill: T={r['T']} P={r['P']} d_e={r['d_e']}")
    with session.Session(w, prefill=r) as s:
        assert ckv.ckv_prefill_kernel_name(s.shape, s.router) == "prefill_mfma_bf16_e128"
        idx, uk, uv = s.packed_views()
    sample = np.sort(np.random.default_rng(5).choice(r["T"], size=3000, replace=False))
    sample = np.unique(np.concatenate([sample, [0, 255, 256, r["T"] - 1]]))
    rs = dict(r)
    rs["S"] = np.ascontiguousarray(r["S"][sample])
    rs["T"] = len(sample)
    ik, iv, ruk, ruv = oracle.prefill(rs)
    for side, got, ref in (("k", idx[0].T[sample], ik), ("v", idx[1].T[sample], iv)):
        gap, mag = oracle.router_gap(rs, side, np.ascontiguousarray(got))
        assert (gap <= (r["d_e"] + 2) * 2.0 ** -23 * mag).all()
        same = float((got == ref).mean())
        say(f"  I_{side}: {same:.5f} identical to the oracle")
        assert same > 0.995
    for got, ref in ((uk, ruk), (uv, ruv)):
        g = wl.to_f64(got.astype(np.uint16), wl.BF16).transpose(1, 0, 2)[sample]
        assert (np.abs(g - ref) <= user_tolerance(ref, wl.BF16)).all()


def test_short_batch_is_cut_along_the_pool(gpu):
    """A batch too short to fill the chip: the workgroups are cut along the pool entries and meet in an atomic
    maximum.  Ties across the cut (integer inputs; scores of +0 and -0) must still go to the lowest entry, a second
    call must find the workspace clean, and a handle without workspace must give the same cache."""
    import torch
    ckv, session = gpu
    lengths = (300, 0, 77, 1)
    r = wl.make_prefill(T=sum(lengths), H=2, d_e=128, d_u=8, P=4096, dtype=wl.BF16, seed=90, integers=1)
    w = decode_workload(lengths, r)
    say("[case] prefill cut along the pool")
    ik, iv, ruk, ruv = oracle.prefill(r)
    with session.Session(w, prefill=r) as s:
        assert ckv.ckv_cache_prefill_workspace(s.cache) > 0, "this shape should have been cut"
        first = [a.copy() for a in s.packed_views()]
        np.testing.assert_array_equal(first[0][0].T, ik)
        np.testing.assert_array_equal(first[0][1].T, iv)
        s.prefill_again()
        s.prefill_again()
        for a, b in zip(first, s.packed_views()):
            np.testing.assert_array_equal(a, b)
        # the same router through a handle that ckv_build_cache made (no workspace: uncut rounds)
        with session.Session(w) as plain:
            assert ckv.ckv_cache_prefill_workspace(plain.cache) == 0
            ckv.ckv_prefill_into(plain.cache, s.router, s.S, plain.stream)
            for a, b in zip(first, plain.packed_views()):
                np.testing.assert_array_equal(a, b)
    # all scores equal, but -0 in the first half of the pool and +0 in the second: entry 0 must win everywhere
    r["S"][:] = 0
    for k in ("w_rk", "w_rv"):
        r[k][:, :2048] = wl.f32_to_bf16_bits(np.full((2, 2048, 128), -1.0, np.float32))
        r[k][:, 2048:] = wl.f32_to_bf16_bits(np.full((2, 2048, 128), 1.0, np.float32))
    r["b_rk"][:] = 0.0
    r["b_rv"][:] = 0.0
    r["b_rk"][:, :2048] = -0.0
    r["b_rv"][:, :2048] = -0.0
    ik, iv, _, _ = oracle.prefill(r)
    assert (ik == 0).all() and (iv == 0).all()
    with session.Session(w, prefill=r) as s:
        assert ckv.ckv_cache_prefill_workspace(s.cache) > 0
        idx = s.packed_views()[0]
    assert (idx == 0).all(), "equal scores across the cut did not go to the lowest pool entry"
    say("  ok")


@pytest.mark.parametrize("block", range(3))
def test_seeded_random_prefill_shapes(gpu, block):
    """Eight seeded random prefill shapes per block (embedding width, pool size, user width, heads, which side is
    shared, batch from one short history to several position blocks: both the cut and the uncut launch), on
    integer inputs where every index and user slice is fixed exactly, and on random inputs to the fp32 bound."""
    for case in range(8):
        rng = np.random.default_rng(500 + 10 * block + case)
        mfma = rng.random() < 0.75
        d_e = int(rng.choice([64, 128, 256])) if mfma else int(rng.choice([8, 24, 72, 100, 200]))
        dtype = wl.BF16 if mfma else int(rng.choice([wl.F32, wl.BF16]))
        P = int(rng.choice([2, 31, 32, 33, 77, 333, 1000, 2049, 5000]))
        d_u = int(rng.choice([0, 1, 3, 4, 8, 16, 33]))
        H = int(rng.integers(1, 4))
        B = int(rng.integers(1, 7))
        lengths = rng.choice([0, 1, 31, 64, 100, 257, 700], size=B).astype(np.int32)
        if lengths.sum() == 0:
            lengths[0] = 5
        share = int(rng.choice([wl.SHARE_KV, wl.SHARE_KV, wl.SHARE_K, wl.SHARE_V]))
        d_a = d_u + int(rng.choice([8, 24, 56]))
        exact = rng.random() < 0.6
        r = wl.make_prefill(T=int(lengths.sum()), H=H, d_e=d_e, d_u=d_u, P=P, dtype=dtype, seed=600 + 10 * block + case,
                            integers=1 if exact else None, share=share, d_a=d_a if share != wl.SHARE_KV else None)
        run_prefill(gpu, lengths, r, f"random prefill {block}.{case}: d_e={d_e} P={P} d_u={d_u} H={H} share={share} lengths={lengths.tolist()}",
                    expected_kernel(dtype, d_e), exact=exact, d_g=d_a - d_u)
