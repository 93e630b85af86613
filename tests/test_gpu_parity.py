"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
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


def make(lengths, dtype, mode, d_a, d_u, H, P, Nq, seed=11, idx="uniform", **kw):
    lengths = np.asarray(lengths, dtype=np.int32)
    return wl.make(B=len(lengths), L=None, H=H, d_a=d_a, d_u=d_u, P=P, idx=idx, Nq=Nq, mode=mode, dtype=dtype,
                   sigma_pool=d_a ** -0.5, seed=seed, lengths=lengths, **kw)


def run_and_check(gpu, w, what, users=None, expect_variant=None, impl=None):
    """impl: None (library's choice) or "staged" (force the register-staged matrix-core kernel)."""
    ckv, session = gpu
    ckv.ckv_set_option("mfma_impl", impl)
    try:
        return _run_and_check(ckv, session, w, what, users, expect_variant)
    finally:
        ckv.ckv_set_option(None)


def _run_and_check(ckv, session, w, what, users, expect_variant):
    say(f"[case] {what}: B={w['B']} H={w['H']} d_g={w['d_g']} d_u={w['d_u']} P={w['P']} Nq={w['Nq']} "
        f"dtype={w['dtype']} mode={w['mode']} T={int(w['lengths'].sum())}")
    with session.Session(w) as s:
        variant = ckv.ckv_variant(s.cache)
        say(f"  variant {variant}")
        if expect_variant:
            assert variant.startswith(expect_variant), variant
        s.attend()
        out = s.output()
    norm = check_against_oracle(out, w, users=users, what=what)
    say(f"  ok, norm-wise error {norm:.3e}")
    return out


RAGGED = (5, 1, 0, 9, 64, 2, 63, 65, 128, 200, 0, 331)


# ---------------------------------------------------------------------------------------------
# packed layout and reconstructed rows: bit exact
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_pack_and_reconstruct_bit_exact(gpu, dtype):
    ckv, session = gpu
    w = make(RAGGED, dtype, wl.SOFTMAX, d_a=24, d_u=3, H=3, P=101, Nq=2, pool_ld=29)
    say(f"[case] reconstruct dtype={dtype}")
    with session.Session(w) as s:
        idx, uk, uv = s.packed_views()
        k_full, v_full = s.reconstruct()
        stored = ckv.ckv_cache_stored_bytes(s.cache)
    np.testing.assert_array_equal(idx[0], w["idx_k"].T)
    np.testing.assert_array_equal(idx[1], w["idx_v"].T)
    np.testing.assert_array_equal(uk, w["user_k"].transpose(1, 0, 2))
    np.testing.assert_array_equal(uv, w["user_v"].transpose(1, 0, 2))
    ok, ov = oracle.reconstruct(w)                       # [T][H][d_a]
    np.testing.assert_array_equal(k_full, ok.transpose(1, 0, 2))
    np.testing.assert_array_equal(v_full, ov.transpose(1, 0, 2))
    T = int(w["lengths"].sum())
    _, _, sb, _ = oracle.cache_size(T, w["H"], w["d_g"], w["d_u"], dtype)
    assert stored == sb


# ---------------------------------------------------------------------------------------------
# streaming kernel (few queries, any shape)
def test_config1(gpu):
    run_and_check(gpu, wl.config("cfg1"), "cfg1", expect_variant="stream_f32_v4")


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_stream_ragged(gpu, dtype, mode):
    w = make(RAGGED, dtype, mode, d_a=64, d_u=8, H=2, P=300, Nq=1)
    run_and_check(gpu, w, f"stream ragged dtype={dtype} mode={mode}", expect_variant="stream")


@pytest.mark.parametrize("dtype,d_a,d_u,pool_ld,Nq", [
    (wl.F32, 16, 3, 13, 3),      # unaligned everything: scalar path
    (wl.BF16, 40, 5, 37, 2),
    (wl.F32, 200, 8, 192, 1),    # several column blocks
    (wl.BF16, 96, 16, 80, 5),    # 8-wide bf16 vectors, Nq not a power of two
    (wl.F32, 12, 0, 12, 2),      # d_u = 0: pure pool attention
    (wl.F32, 12, 12, 0, 2),      # d_g = 0: ordinary attention over the user K/V
    (wl.F32, 255, 7, 250, 2),    # the widest rows at each alignment: single elements, sixteen column blocks
    (wl.BF16, 256, 3, 253, 3),
    (wl.F32, 512, 8, 504, 1),    # 4-wide vectors, eight column blocks
    (wl.BF16, 1024, 8, 1016, 2), # 8-wide bf16 vectors, eight column blocks
])
def test_stream_shapes(gpu, dtype, d_a, d_u, pool_ld, Nq):
    w = make(RAGGED, dtype, wl.SOFTMAX, d_a=d_a, d_u=d_u, H=2, P=77, Nq=Nq, pool_ld=pool_ld)
    run_and_check(gpu, w, f"stream shape d_a={d_a} d_u={d_u} ld={pool_ld}", expect_variant="stream")


def test_stream_split_history(gpu):
    # one long history among few users: cut into pieces and merged
    w = make((5000, 70, 2300), wl.F32, wl.SOFTMAX, d_a=64, d_u=8, H=2, P=500, Nq=2)
    run_and_check(gpu, w, "stream split softmax")
    w = make((5000, 70, 2300), wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=8, H=2, P=500, Nq=2)
    run_and_check(gpu, w, "stream split silu")


# wide-row streaming kernel: rows fetched in 16-byte lanes (8, 16, 32 or 64 lanes per row) whatever the user width,
# user slices element by element
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("dtype,d_a,d_u,pool_ld,Nq,expect", [
    # the widths behind Table 1's compression ratios: d_u of 256 columns, one query (target attention)
    (wl.BF16, 256, 1, 256, 1, "streamw_bf16_g32_q1"), (wl.BF16, 256, 2, 256, 1, "streamw_bf16_g32_q1"),
    (wl.BF16, 256, 3, 256, 1, "streamw_bf16_g32_q1"), (wl.BF16, 256, 4, 256, 1, "streamw_bf16_g32_q1"),
    (wl.BF16, 256, 6, 256, 1, "streamw_bf16_g32_q1"), (wl.BF16, 256, 10, 248, 1, "streamw_bf16_g32_q1"),
    (wl.BF16, 256, 10, 256, 2, "streamw_bf16_g32_q2"), (wl.BF16, 256, 4, 264, 2, "streamw_bf16_g32_q2"),
    (wl.F32, 256, 1, 256, 1, "streamw_f32_g64_q1"), (wl.F32, 256, 6, 252, 2, "streamw_f32_g64_q2"),
    (wl.F32, 256, 10, 256, 5, "streamw_f32_g64_q2"),             # five queries: two passes of two and one of one
    # fewer lanes per row; slices of up to eight columns per lane of the row's octets
    (wl.BF16, 64, 3, 64, 1, "streamw_bf16_g8_q1"), (wl.BF16, 64, 8, 56, 2, "stream_bf16_v8_c1_g8"),
    (wl.BF16, 64, 6, 64, 2, "streamw_bf16_g8_q2"), (wl.BF16, 64, 12, 56, 1, "stream_bf16_v4_c1"), (wl.BF16, 64, 10, 56, 1, "streamw_bf16_g16_q1"),
    (wl.BF16, 128, 5, 128, 1, "streamw_bf16_g16_q1"), (wl.BF16, 128, 14, 120, 2, "streamw_bf16_g16_q2"),
    (wl.BF16, 72, 9, 64, 7, "streamw_bf16_g16_q2"),               # a width no matrix-core kernel takes below eight queries
    (wl.BF16, 200, 30, 176, 1, "streamw_bf16_g32_q1"), (wl.BF16, 512, 64, 448, 1, "streamw_bf16_g64_q1"),
    (wl.F32, 64, 6, 60, 1, "streamw_f32_g16_q1"), (wl.F32, 128, 2, 128, 2, "streamw_f32_g32_q2"),
    (wl.F32, 100, 7, 96, 3, "streamw_f32_g32_q2"), (wl.F32, 24, 24, 0, 1, "stream_f32"),   # (d_g = 0 with rows of 96 bytes: whole 16-byte lanes)
])
def test_wide_row_streaming_kernel(gpu, mode, dtype, d_a, d_u, pool_ld, Nq, expect):
    kw = dict(pool_ld=pool_ld) if d_a > d_u else {}
    w = make(RAGGED + (700,), dtype, mode, d_a=d_a, d_u=d_u, H=2, P=77, Nq=Nq, **kw)
    run_and_check(gpu, w, f"wide-row stream d_a={d_a} d_u={d_u} ld={pool_ld} Nq={Nq}", expect_variant=expect)


@pytest.mark.parametrize("share", [wl.SHARE_K, wl.SHARE_V])
@pytest.mark.parametrize("dtype,d_a,d_u,Nq", [(wl.BF16, 256, 3, 1), (wl.BF16, 128, 10, 2), (wl.F32, 64, 5, 1), (wl.F32, 256, 4, 2)])
def test_wide_row_streaming_kernel_one_side_shared(gpu, share, dtype, d_a, d_u, Nq):
    for mode in (wl.SOFTMAX, wl.SILU_OVER_N):
        w = make(RAGGED, dtype, mode, d_a=d_a, d_u=d_u, H=2, P=50, Nq=Nq, share=share, idx=("zipf", 1.1))
        run_and_check(gpu, w, f"wide-row stream share={share} d_a={d_a} d_u={d_u} mode={mode}", expect_variant="streamw")


def test_wide_row_streaming_kernel_split_history_many_items_and_plain_cache(gpu):
    # one long history among few users: cut into pieces and merged
    w = make((5000, 70, 2300, 0), wl.BF16, wl.SOFTMAX, d_a=256, d_u=6, H=2, P=500, Nq=2)
    run_and_check(gpu, w, "wide-row stream split softmax", expect_variant="streamw_bf16_g32_q2")
    w = make((5000, 70, 2300), wl.F32, wl.SILU_OVER_N, d_a=256, d_u=3, H=1, P=500, Nq=1)
    run_and_check(gpu, w, "wide-row stream split silu", expect_variant="streamw_f32_g64_q1")
    # more short items than resident workgroups: two wavefronts per item
    rng = np.random.default_rng(5)
    w = make(rng.integers(0, 300, size=2500), wl.BF16, wl.SOFTMAX, d_a=256, d_u=10, H=2, P=3000, Nq=1, idx=("zipf", 1.05))
    out = run_and_check(gpu, w, "wide-row stream, many short items", expect_variant="streamw_bf16_g32_q1")
    ckv, session = gpu
    with session.Session(w) as s:
        assert ckv.ckv_variant(s.cache).endswith("_w2")
    # an ordinary cache (d_g = 0): both sides are rows of the user arrays, fetched by position
    w = make(RAGGED, wl.BF16, wl.SOFTMAX, d_a=256, d_u=256, H=2, P=1, Nq=2)
    run_and_check(gpu, w, "wide-row stream, ordinary cache", expect_variant="streamw_bf16_g32_q2")
    # large scores: the reference maximum of a row group moves often
    w = make((900, 33), wl.F32, wl.SOFTMAX, d_a=256, d_u=2, H=1, P=400, Nq=1, scale=6.0)
    run_and_check(gpu, w, "wide-row stream, large scores", expect_variant="streamw_f32_g64_q1")
    # the column-block kernel still serves the shape when asked to
    w = make(RAGGED, wl.BF16, wl.SOFTMAX, d_a=256, d_u=6, H=2, P=77, Nq=1)
    ckv.ckv_set_option("stream_impl", "narrow")
    try:
        with session.Session(w) as s:
            assert ckv.ckv_variant(s.cache).startswith("stream_bf16_v1"), ckv.ckv_variant(s.cache)
            s.attend()
            narrow = s.output()
    finally:
        ckv.ckv_set_option(None)
    check_against_oracle(narrow, w, what="column-block kernel on a wide-row shape")


@pytest.mark.parametrize("name", ["tgt256_u1", "tgt256_u10"])
def test_target_attention_over_256_columns_full(gpu, name):
    # the benchmark's target-attention workloads (one query, Table 1's head width and user widths), every output
    run_and_check(gpu, wl.config(name), name, expect_variant="streamw_bf16_g32_q1")


@pytest.mark.parametrize("name", ["cfg2_f32", "cfg2_bf16"])
def test_config2_full(gpu, name):
    run_and_check(gpu, wl.config(name), name, expect_variant="stream")


# ---------------------------------------------------------------------------------------------
# matrix-core kernel (many queries, bf16)
MFMA_LENGTHS = (1, 31, 32, 33, 64, 65, 0, 127, 200, 1500, 96, 2)


@pytest.mark.parametrize("impl", [None, "staged"])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_a,d_u,Nq", [(64, 4, 64), (64, 2, 16), (64, 8, 32), (128, 8, 128), (128, 8, 40),
                                         (64, 3, 20), (128, 16, 64), (64, 0, 16), (128, 24, 100), (64, 8, 200),
                                         (128, 2, 16), (128, 4, 64), (64, 6, 128), (128, 0, 32), (64, 8, 8)])
def test_mfma_ragged(gpu, impl, mode, d_a, d_u, Nq):
    w = make(MFMA_LENGTHS, wl.BF16, mode, d_a=d_a, d_u=d_u, H=2, P=700, Nq=Nq)
    dma_ok = d_u <= 16 and (d_u % 2 == 0 or d_u <= 7)
    expect = "mfma_dma" if (impl is None and dma_ok) else "mfma_bf16"
    run_and_check(gpu, w, f"mfma ragged d_a={d_a} d_u={d_u} Nq={Nq} mode={mode} impl={impl}", expect_variant=expect, impl=impl)


@pytest.mark.parametrize("impl", [None, "staged"])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_mfma_split_history(gpu, impl, mode):
    w = make((5000, 70, 2300, 1024, 1025), wl.BF16, mode, d_a=128, d_u=8, H=2, P=5000, Nq=128)
    run_and_check(gpu, w, f"mfma split mode={mode} impl={impl}", expect_variant="mfma", impl=impl)


@pytest.mark.parametrize("d_a", [128, 256])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_tile_loop_with_the_scores_one_tile_ahead(gpu, mode, d_a):
    """Four wavefronts at 128 and at 256 columns: the loop that takes the scores of tile t + 1 in the iteration that finishes
    tile t and the loop that does not must agree bit for bit (the same arithmetic in the same order) and with the oracle:
    ragged lengths (one tile, tile boundaries, empty), a split history, one side shared, an ordinary cache; at 256 columns
    also few queries (wavefronts without any) and slices of 10 and 32 columns."""
    ckv, session = gpu
    cases = [dict(lengths=MFMA_LENGTHS + (95, 97, 160), d_u=8, Nq=128), dict(lengths=MFMA_LENGTHS, d_u=0, Nq=100),
             dict(lengths=(5000, 70, 2300), d_u=8, Nq=128), dict(lengths=MFMA_LENGTHS, d_u=4, Nq=65, share=wl.SHARE_K),
             dict(lengths=MFMA_LENGTHS, d_u=4, Nq=128, share=wl.SHARE_V), dict(lengths=(65, 1, 640), d_u=d_a, Nq=128)]
    if d_a == 256:
        cases += [dict(lengths=MFMA_LENGTHS, d_u=10, Nq=40), dict(lengths=(3000, 33, 64), d_u=32, Nq=130),
                  dict(lengths=RAGGED, d_u=2, Nq=3)]
    for c in cases:
        w = make(c["lengths"], wl.BF16, mode, d_a=d_a, d_u=c["d_u"], H=2, P=700 if c["d_u"] < d_a else 1, Nq=c["Nq"],
                 share=c.get("share", wl.SHARE_KV))
        outs = []
        for ahead in ("0", "1"):
            ckv.ckv_set_option("dma_scores_ahead", ahead)
            try:
                outs.append(_run_and_check(ckv, session, w, f"scores ahead = {ahead}, d_a={d_a} d_u={c['d_u']} Nq={c['Nq']} mode={mode}", None,
                                           f"mfma_dma_bf16_d{d_a}_w4_g1"))
            finally:
                ckv.ckv_set_option(None)
        np.testing.assert_array_equal(outs[0], outs[1])


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_sixteen_queries_per_work_item(gpu, mode):
    """64 columns, 3 to 16 queries: the organisation on the 16x16x32 matrix instruction (sixteen queries a work item) against
    the oracle, and the organisation with 32 queries a work item, which it replaces there, as well: ragged lengths (one tile,
    tile boundaries, empty), every even slice width, a split history, one side shared, an ordinary cache, unpadded pool rows."""
    ckv, session = gpu
    cases = [dict(lengths=MFMA_LENGTHS + (95, 97, 160), d_u=8, Nq=16), dict(lengths=MFMA_LENGTHS, d_u=0, Nq=3),
             dict(lengths=MFMA_LENGTHS, d_u=2, Nq=9), dict(lengths=RAGGED, d_u=6, Nq=15),
             dict(lengths=(9000, 70, 2300), d_u=2, Nq=16), dict(lengths=(5000, 1), d_u=8, Nq=5, share=wl.SHARE_V),
             dict(lengths=MFMA_LENGTHS, d_u=4, Nq=12, share=wl.SHARE_K), dict(lengths=MFMA_LENGTHS, d_u=4, Nq=16, share=wl.SHARE_V),
             dict(lengths=(65, 1, 640), d_u=64, Nq=16), dict(lengths=MFMA_LENGTHS, d_u=8, Nq=7, pool_ld=56)]
    for c in cases:
        kw = {k: c[k] for k in ("share", "pool_ld") if k in c}
        w = make(c["lengths"], wl.BF16, mode, d_a=64, d_u=c["d_u"], H=2, P=700 if c["d_u"] < 64 else 1, Nq=c["Nq"], **kw)
        for q16, expect in (("1", "mfma_dma_bf16_d64_w1_q16"), ("0", "mfma_dma_bf16_d64_w1_g1")):
            ckv.ckv_set_option("dma_q16", q16)
            try:
                _run_and_check(ckv, session, w, f"sixteen queries = {q16}, d_u={c['d_u']} Nq={c['Nq']} mode={mode} {kw}", None, expect)
            finally:
                ckv.ckv_set_option(None)


def nearly_equal_weights_shape():
    """The shape on which a run over further seeded random shapes broke the rule that had tol * rss_c alone for the rounding of
    the weights (ratio 1.004), drawn exactly as that run drew it: 128 columns of which one is the user's, a pool of two rows,
    796 users of up to 199 positions, 200 queries, SiLU weights, scale 2.  The keys of a history are two pool rows that differ
    from position to position only in the user's column, so the weights of a query come in two clusters of nearly equal
    values, and a cluster is rounded to bf16 all the same way."""
    rng = np.random.default_rng(990000 + 7215)
    assert not rng.random() < 0.6
    d_a = int(rng.choice([64, 128, 256]))
    d_u = int(rng.choice([0, 1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 16]))
    Nq = int(rng.choice([17, 31, 32, 33, 40, 64, 65, 100, 128, 129, 200]))
    d_g = d_a - d_u
    pool_ld = int(rng.choice([(d_g + 7) // 8 * 8, d_a, d_a + 8]))
    share = int(rng.choice([wl.SHARE_KV, wl.SHARE_KV, wl.SHARE_K, wl.SHARE_V]))
    mode = int(rng.choice([wl.SOFTMAX, wl.SILU_OVER_N]))
    B = int(rng.integers(1, 7))
    rng.choice([0, 1, 7, 31, 32, 33, 63, 64, 65, 95, 96, 97, 100, 255, 256, 257, 513, 900, 2500, 6000, 20000], size=B)
    assert rng.random() < 0.1
    B = int(rng.integers(300, 900))
    lengths = rng.integers(0, 200, size=B).astype(np.int32)
    H, P = int(rng.integers(1, 5)), int(rng.choice([1, 2, 77, 700, 3000, 50000]))
    assert not rng.random() < 0.15
    scale = None if rng.random() < 0.8 else float(rng.choice([0.01, 0.5, 2.0]))
    assert (d_a, d_u, Nq, pool_ld, share, mode, B, H, P, scale) == (128, 1, 200, 136, wl.SHARE_KV, wl.SILU_OVER_N, 796, 4, 2, 2.0)
    return wl.make(B=B, L=None, H=H, d_a=d_a, d_u=d_u, P=P, idx=("zipf", 1.1) if rng.random() < 0.3 else "uniform", Nq=Nq, mode=mode,
                   dtype=wl.BF16, sigma_pool=d_a ** -0.5, seed=7000 + 7215, lengths=lengths, share=share, scale=scale, pool_ld=pool_ld)


def test_nearly_equal_weights_round_alike(gpu):
    """Weights that are nearly equal are rounded to bf16 the same way and their errors add up coherently: the rule's bound
    u_w * asum_c stands for that case (see tests/parity.py)."""
    w = nearly_equal_weights_shape()
    run_and_check(gpu, w, "nearly equal weights (pool of two rows, one user column)", expect_variant="mfma_dma_bf16_d128_w4_g1_silu")


def test_mfma_unpadded_pool_rows(gpu):
    # pool_ld == d_g (a multiple of 8): the chunk that would be padding does not exist in memory
    w = make(MFMA_LENGTHS, wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=2, P=333, Nq=16, pool_ld=56)
    run_and_check(gpu, w, "mfma pool_ld=d_g", expect_variant="mfma_dma")
    w = make(MFMA_LENGTHS, wl.BF16, wl.SOFTMAX, d_a=128, d_u=8, H=1, P=333, Nq=64, pool_ld=120)
    run_and_check(gpu, w, "mfma pool_ld=d_g staged", expect_variant="mfma_bf16", impl="staged")


def test_negative_scale_falls_back_to_streaming(gpu):
    w = make((70, 33), wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=1, P=50, Nq=16, scale=-0.125)
    run_and_check(gpu, w, "negative scale", expect_variant="stream")


@pytest.mark.parametrize("impl", [None, "staged"])
def test_mfma_all_users_is_ordinary_attention_when_dg_zero(gpu, impl):
    """d_g = 0 (section 5.3: the method degenerates into the ordinary K/V cache): no pool, no indices."""
    w = make(MFMA_LENGTHS, wl.BF16, wl.SOFTMAX, d_a=64, d_u=64, H=1, P=1, Nq=16)
    run_and_check(gpu, w, "mfma d_g=0", expect_variant="mfma_dma" if impl is None else "mfma_bf16", impl=impl)
    w = make((5000, 70, 2300, 1025), wl.BF16, wl.SILU_OVER_N, d_a=128, d_u=128, H=2, P=1, Nq=128)
    run_and_check(gpu, w, "mfma d_g=0, 128 columns, split history", expect_variant="mfma_dma" if impl is None else "mfma_bf16", impl=impl)


def test_mfma_large_scores_softmax(gpu):
    # big logits exercise the running-maximum bookkeeping (lazy rescale threshold)
    w = make((700, 129), wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=1, P=300, Nq=32, sigma_q=6.0, scale=1.0)
    run_and_check(gpu, w, "mfma large scores", expect_variant="mfma")


# ---------------------------------------------------------------------------------------------
# full-size workloads, in the launch configuration the benchmark times; every output of every user against the oracle
def test_config3_full(gpu):
    run_and_check(gpu, wl.config("cfg3"), "cfg3", expect_variant="mfma_dma_bf16_d64_w1_g2")


def test_config3_keys_only_full(gpu):
    run_and_check(gpu, wl.config("cfg3_ck"), "cfg3_ck", expect_variant="mfma_dma_bf16_d64_w1_g2")


def test_config4_full(gpu):
    run_and_check(gpu, wl.config("cfg4"), "cfg4", expect_variant="mfma_dma_bf16_d128_w4_g1")


@pytest.mark.parametrize("name,Nq", [("d256_u4", 128), ("d256_u10", 128), ("d256_u4", 40)])
def test_256_column_heads_full(gpu, name, Nq):
    """Table 1's head width at config 4's batch, in the launch configuration the bench times; 40 queries leave
    wavefronts without queries that only gather."""
    run_and_check(gpu, wl.config(name, Nq=Nq), f"{name} Nq={Nq}", expect_variant="mfma_dma_bf16_d256_w4_g1")


def test_fp32_256_column_heads_full(gpu):
    """The fp32 matrix-core kernel's widest instance on the workload the bench reports for it."""
    run_and_check(gpu, wl.config("cfg3_f32_d256"), "cfg3_f32_d256", expect_variant="mfma_f32_d256")


def test_config5_full(gpu):
    run_and_check(gpu, wl.config("cfg5"), "cfg5", expect_variant="mfma_dma_bf16_d64_w1_q16")


# ---------------------------------------------------------------------------------------------
# offloaded cache: packed cache in pinned host memory, read in place by the same kernels
@pytest.mark.parametrize("kind", ["stream", "streamw", "dma", "staged"])
def test_offloaded_cache_matches_resident(gpu, kind):
    ckv, session = gpu
    if kind == "stream":
        w = make(RAGGED, wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=2, P=300, Nq=1)
    elif kind == "streamw":
        w = make(RAGGED, wl.BF16, wl.SOFTMAX, d_a=256, d_u=3, H=2, P=300, Nq=1)
    elif kind == "dma":
        w = make(MFMA_LENGTHS, wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=4, H=2, P=700, Nq=64)
    else:
        w = make(MFMA_LENGTHS, wl.BF16, wl.SOFTMAX, d_a=128, d_u=16, H=2, P=700, Nq=40)
    say(f"[case] offloaded {kind}")
    outs = []
    for off in (False, True):
        with session.Session(w, offloaded=off) as s:
            assert ckv.ckv_cache_is_offloaded(s.cache) == off
            s.attend()
            outs.append(s.output().copy())
            idx, uk, uv = s.packed_views()
            np.testing.assert_array_equal(idx[0], w["idx_k"].T)
            np.testing.assert_array_equal(uv, w["user_v"].transpose(1, 0, 2))
    np.testing.assert_array_equal(outs[0], outs[1])
    check_against_oracle(outs[1], w, what=f"offloaded {kind}")


# ---------------------------------------------------------------------------------------------
# sharing only keys or only values (CollectiveK / CollectiveV): the other side is an ordinary d_a-wide cache
@pytest.mark.parametrize("share", [wl.SHARE_K, wl.SHARE_V])
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_single_side_sharing_pack_and_reconstruct_bit_exact(gpu, share, dtype):
    ckv, session = gpu
    w = make(RAGGED, dtype, wl.SOFTMAX, d_a=24, d_u=3, H=3, P=101, Nq=2, pool_ld=29, share=share)
    say(f"[case] reconstruct share={share} dtype={dtype}")
    with session.Session(w) as s:
        idx, uk, uv = s.packed_views()
        k_full, v_full = s.reconstruct()
        stored = ckv.ckv_cache_stored_bytes(s.cache)
    shared_plane, plain_plane = (0, 1) if share == wl.SHARE_K else (1, 0)
    np.testing.assert_array_equal(idx[shared_plane], w["idx_k" if share == wl.SHARE_K else "idx_v"].T)
    assert (idx[plain_plane] == 0).all()
    np.testing.assert_array_equal(uk, w["user_k"].transpose(1, 0, 2))
    np.testing.assert_array_equal(uv, w["user_v"].transpose(1, 0, 2))
    ok, ov = oracle.reconstruct(w)
    np.testing.assert_array_equal(k_full, ok.transpose(1, 0, 2))
    np.testing.assert_array_equal(v_full, ov.transpose(1, 0, 2))
    _, _, sb, _ = oracle.cache_size(int(w["lengths"].sum()), w["H"], w["d_g"], w["d_u"], dtype, share=share)
    assert stored == sb


@pytest.mark.parametrize("share", [wl.SHARE_K, wl.SHARE_V])
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_single_side_sharing_stream(gpu, share, dtype, mode):
    w = make(RAGGED, dtype, mode, d_a=64, d_u=8, H=2, P=300, Nq=2, share=share)
    run_and_check(gpu, w, f"stream share={share} dtype={dtype} mode={mode}", expect_variant="stream")
    w = make(RAGGED, dtype, mode, d_a=20, d_u=3, H=1, P=77, Nq=1, pool_ld=19, share=share)
    run_and_check(gpu, w, f"stream unaligned share={share} dtype={dtype} mode={mode}", expect_variant="stream")


@pytest.mark.parametrize("impl", [None, "staged"])
@pytest.mark.parametrize("share", [wl.SHARE_K, wl.SHARE_V])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_a,d_u,Nq", [(64, 4, 64), (128, 8, 128), (64, 3, 20), (128, 16, 40), (64, 2, 16), (128, 0, 32)])
def test_single_side_sharing_matrix_core(gpu, impl, share, mode, d_a, d_u, Nq):
    w = make(MFMA_LENGTHS, wl.BF16, mode, d_a=d_a, d_u=d_u, H=2, P=700, Nq=Nq, share=share)
    dma_ok = d_u <= 16 and (d_u % 2 == 0 or d_u <= 7)
    expect = "mfma_dma" if (impl is None and dma_ok) else "mfma_bf16"
    run_and_check(gpu, w, f"mfma share={share} d_a={d_a} d_u={d_u} Nq={Nq} mode={mode} impl={impl}", expect_variant=expect, impl=impl)


@pytest.mark.parametrize("impl", [None, "staged"])
def test_single_side_sharing_split_history(gpu, impl):
    w = make((5000, 70, 2300, 1025), wl.BF16, wl.SOFTMAX, d_a=128, d_u=8, H=2, P=5000, Nq=128, share=wl.SHARE_K)
    run_and_check(gpu, w, f"mfma split share=K impl={impl}", expect_variant="mfma", impl=impl)
    w = make((5000, 70, 2300, 1025), wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=4, H=2, P=5000, Nq=64, share=wl.SHARE_V)
    run_and_check(gpu, w, f"mfma split share=V impl={impl}", expect_variant="mfma", impl=impl)
    w = make((5000, 70, 2300), wl.F32, wl.SOFTMAX, d_a=64, d_u=8, H=2, P=500, Nq=2, share=wl.SHARE_V)
    run_and_check(gpu, w, "stream split share=V", expect_variant="stream")


# ---------------------------------------------------------------------------------------------
# frequency renumbering of the pool rows: a relabeling that must not change any output bit
@pytest.mark.parametrize("share", [wl.SHARE_KV, wl.SHARE_K, wl.SHARE_V])
@pytest.mark.parametrize("kind", ["stream", "dma"])
def test_hot_row_renumbering(gpu, share, kind):
    ckv, session = gpu
    if kind == "stream":
        w = make(RAGGED, wl.F32, wl.SOFTMAX, d_a=24, d_u=3, H=3, P=101, Nq=2, pool_ld=29, idx=("zipf", 1.2), share=share)
    else:
        w = make(MFMA_LENGTHS, wl.BF16, wl.SOFTMAX, d_a=64, d_u=4, H=2, P=700, Nq=64, idx=("zipf", 1.1), share=share)
    say(f"[case] hot-row renumbering {kind} share={share}")
    with session.Session(w) as s:
        s.attend()
        before = s.output().copy()
        old_pk = session._to_host(s.pool_k, w["dtype"]).copy()
        old_pv = session._to_host(s.pool_v, w["dtype"]).copy()
        new_id = s.remap_hot_rows()
        idx, _, _ = s.packed_views()
        new_pk = session._to_host(s.pool_k, w["dtype"])
        new_pv = session._to_host(s.pool_v, w["dtype"])
        s.out.fill_(float("nan"))
        s.attend()
        after = s.output()
        k_full, v_full = s.reconstruct()
    nk, nv = oracle.hot_row_order(w)
    np.testing.assert_array_equal(new_id[0], nk)
    np.testing.assert_array_equal(new_id[1], nv)
    for h in range(w["H"]):
        if share in (wl.SHARE_KV, wl.SHARE_K):
            np.testing.assert_array_equal(idx[0][h], nk[h][w["idx_k"][:, h]])
            np.testing.assert_array_equal(new_pk[h][nk[h]].view(np.uint8), old_pk[h].view(np.uint8))   # bytes, padding included
        if share in (wl.SHARE_KV, wl.SHARE_V):
            np.testing.assert_array_equal(idx[1][h], nv[h][w["idx_v"][:, h]])
            np.testing.assert_array_equal(new_pv[h][nv[h]].view(np.uint8), old_pv[h].view(np.uint8))
    np.testing.assert_array_equal(after, before)
    ok, ov = oracle.reconstruct(w)
    np.testing.assert_array_equal(k_full, ok.transpose(1, 0, 2))
    np.testing.assert_array_equal(v_full, ov.transpose(1, 0, 2))
    check_against_oracle(after, w, what=f"renumbered {kind} share={share}")


@pytest.mark.parametrize("dtype,mode,d_a,d_u,H,P,share,idx,rows", [
    (wl.BF16, wl.SOFTMAX, 256, 4, 2, 300, wl.SHARE_KV, ("zipf", 1.1), 32), (wl.BF16, wl.SILU_OVER_N, 256, 10, 2, 20, wl.SHARE_KV, "uniform", 32),
    (wl.BF16, wl.SOFTMAX, 256, 3, 2, 300, wl.SHARE_K, ("zipf", 1.2), 16), (wl.BF16, wl.SOFTMAX, 256, 3, 2, 300, wl.SHARE_V, ("zipf", 1.2), 8),
    (wl.F32, wl.SOFTMAX, 256, 6, 1, 500, wl.SHARE_KV, ("zipf", 1.1), 32), (wl.F32, wl.SILU_OVER_N, 128, 2, 2, 77, wl.SHARE_KV, "uniform", 21),
    (wl.BF16, wl.SOFTMAX, 128, 5, 3, 1000, wl.SHARE_KV, ("zipf", 1.05), 32), (wl.BF16, wl.SOFTMAX, 512, 16, 1, 200, wl.SHARE_KV, ("zipf", 1.1), 32)])
def test_hot_rows_in_lds_of_the_wide_row_streaming_kernel(gpu, dtype, mode, d_a, d_u, H, P, share, idx, rows):
    """The second half of the frequency renumbering (appendix on router activations): the first rows of the pools copied into
    LDS per work item and served from there.  Results must be bit-identical with and without (the same rows, the same
    arithmetic), before and after the renumbering, and match the oracle; pools smaller than the row count, histories shorter
    than four times the row count (fewer rows are then kept) and sides without pool are among the cases."""
    ckv, session = gpu
    w = make(RAGGED + (700, 31, 33, 97), dtype, mode, d_a=d_a, d_u=d_u, H=H, P=P, Nq=1, share=share, idx=idx)
    outs = []
    for hot in (0, rows):
        ckv.ckv_set_option("stream_hot_rows", str(hot))
        try:
            with session.Session(w) as s:
                assert ckv.ckv_variant(s.cache).startswith("streamw")
                s.attend()
                outs.append(s.output().copy())
                s.remap_hot_rows()
                s.out.fill_(float("nan"))
                s.attend()
                outs.append(s.output().copy())
        finally:
            ckv.ckv_set_option(None)
    for o in outs[1:]:
        np.testing.assert_array_equal(o, outs[0])
    check_against_oracle(outs[3], w, what=f"hot rows in LDS, d_a={d_a} d_u={d_u} share={share}")


def test_hot_row_renumbering_rejects_offloaded_and_aliased(gpu):
    ckv, session = gpu
    w = make((10, 20), wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=1, P=50, Nq=1)
    with session.Session(w, offloaded=True) as s:
        with pytest.raises(ckv.CkvError) as e:
            s.remap_hot_rows()
        assert e.value.code == ckv.CKV_ERR_UNSUPPORTED
    with session.Session(w) as s:
        with pytest.raises(ckv.CkvError) as e:
            ckv.ckv_remap_hot_rows(s.cache, s.pool_k, s.pool_v, s.pool_k, s.pool_v, None, s.stream)
        assert e.value.code == ckv.CKV_ERR_NULL


# ---------------------------------------------------------------------------------------------
# error paths that need the device
def test_out_of_range_index_is_rejected(gpu):
    ckv, session = gpu
    w = make((10, 20), wl.F32, wl.SOFTMAX, d_a=16, d_u=4, H=2, P=50, Nq=1)
    w["idx_v"][13, 1] = 50
    with pytest.raises(ckv.CkvError) as e:
        session.Session(w)
    assert e.value.code == ckv.CKV_ERR_INDEX and "position 13 head 1" in str(e.value)
    w["idx_v"][13, 1] = -1
    with pytest.raises(ckv.CkvError):
        session.Session(w)


def test_attend_rejects_unaligned_and_missing_pointers(gpu):
    ckv, session = gpu
    w = make((10, 20), wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=1, P=50, Nq=16)
    with session.Session(w) as s:
        c = s.cache
        args = [s.pool_k, s.pool_v, ckv.ckv_cache_idx(c), ckv.ckv_cache_user_k(c), ckv.ckv_cache_user_v(c), s.q,
                ckv.ckv_cache_lengths(c), s.out]
        for i, code in ((5, ckv.CKV_ERR_UNSUPPORTED), (7, ckv.CKV_ERR_UNSUPPORTED)):
            bad = list(args)
            bad[i] = bad[i].data_ptr() + 2
            with pytest.raises(ckv.CkvError) as e:
                ckv.ckv_attend(c, *bad, s.stream)
            assert e.value.code == code
        for i in (0, 2, 3, 5, 7):
            bad = list(args)
            bad[i] = None
            with pytest.raises(ckv.CkvError) as e:
                ckv.ckv_attend(c, *bad, s.stream)
            assert e.value.code == ckv.CKV_ERR_NULL
        s.attend()  # the handle is still usable
        check_against_oracle(s.output(), w, what="after rejected calls")


def test_attend_refuses_lengths_that_are_not_the_handles(gpu):
    """The work lists follow the lengths the handle was built with; another lengths array (even an equal copy)
    is refused instead of being ignored."""
    import torch
    ckv, session = gpu
    w = make((10, 20), wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=1, P=50, Nq=16)
    with session.Session(w) as s:
        c = s.cache
        grown = torch.tensor([10, 21], dtype=torch.int32, device="cuda")
        same = torch.tensor([10, 20], dtype=torch.int32, device="cuda")
        for other in (grown, same):
            for call in (ckv.ckv_attend, ckv.ckv_attend_static_scratch):
                with pytest.raises(ckv.CkvError) as e:
                    call(c, s.pool_k, s.pool_v, ckv.ckv_cache_idx(c), ckv.ckv_cache_user_k(c), ckv.ckv_cache_user_v(c), s.q,
                         other, s.out, s.stream)
                assert e.value.code == ckv.CKV_ERR_UNSUPPORTED and "ckv_cache_lengths" in str(e.value)
        s.attend()
        check_against_oracle(s.output(), w, what="after refused lengths")


def test_all_histories_empty(gpu):
    w = make((0, 0, 0), wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=2, P=10, Nq=16)
    out = run_and_check(gpu, w, "all empty")
    assert np.all(out == 0)
    w = make((0, 0), wl.F32, wl.SOFTMAX, d_a=16, d_u=4, H=1, P=10, Nq=1)
    out = run_and_check(gpu, w, "all empty stream")
    assert np.all(out == 0)


def test_repeated_calls_are_deterministic(gpu):
    ckv, session = gpu
    w = make((5000, 70, 2300), wl.BF16, wl.SOFTMAX, d_a=128, d_u=8, H=2, P=5000, Nq=128)
    with session.Session(w) as s:
        s.attend()
        a = s.output().copy()
        s.out.fill_(float("nan"))
        s.attend()
        b = s.output()
    np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("kind", ["stream", "streamw", "dma_split"])
def test_attend_replayed_from_a_captured_graph(gpu, kind):
    """A serving loop records ckv_attend once and replays it; every replay (new queries in the captured
    buffer, eager work and synchronisations in between) must equal the eager call bit for bit."""
    import torch
    ckv, session = gpu
    if kind == "stream":
        w = make((300, 0, 41, 1200), wl.F32, wl.SOFTMAX, d_a=32, d_u=4, H=2, P=700, Nq=1)
    elif kind == "streamw":  # wide-row streaming kernel, two queries, a split history and its merge kernel
        w = make((3000, 0, 41, 1200), wl.BF16, wl.SOFTMAX, d_a=256, d_u=3, H=2, P=700, Nq=2)
    else:  # one long history among short ones: split into pieces, merged by a second kernel
        w = make((9000, 64, 3, 0, 500), wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=4, H=2, P=3000, Nq=64)
    rng = np.random.default_rng(5)
    with session.Session(w) as s:
        say(f"[case] graph replay {kind}: variant {ckv.ckv_variant(s.cache)}")
        if kind == "dma_split":
            assert ckv.ckv_variant(s.cache).startswith("mfma_dma")
        if kind == "streamw":
            assert ckv.ckv_variant(s.cache).startswith("streamw")
        s.attend()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):  # capture runs on `side`; nothing executes yet
            s.attend(stream=torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for rep in range(3):
            qn = torch.randn(s.q.shape, generator=torch.Generator().manual_seed(100 + rep)).to(s.q.dtype).cuda()
            s.q.copy_(qn)
            s.out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            got = s.output().copy()
            s.out.fill_(float("nan"))
            s.attend()
            want = s.output()
            np.testing.assert_array_equal(got, want)
            say(f"  replay {rep} equals the eager call")
        # the last queries against the oracle as well
        w2 = dict(w)
        w2["q"] = session._to_host(s.q, w["dtype"])
    check_against_oracle(want, w2, what=f"graph replay {kind}")


@pytest.mark.parametrize("kind", ["dma", "staged", "stream"])
def test_pool_rows_beyond_four_gib(gpu, kind):
    """A pool of more than 2^24 rows of 256 bytes: byte offsets of the rows pass 2^32, so an address
    computed in 32 bits would wrap onto another row.  The pool repeats a random block whose period
    (a prime) does not divide 2^24, which makes a wrapped row differ from the right one."""
    P_big, period = (1 << 24) + 4099, 65521
    Nq = 1 if kind == "stream" else 128
    w = make((700, 3, 0, 1500), wl.BF16, wl.SOFTMAX, d_a=128, d_u=8, H=1, P=period, Nq=Nq, seed=23)
    rng = np.random.default_rng(23)
    T = int(w["lengths"].sum())
    for side in ("k", "v"):
        block = w["pool_" + side][0]
        big = np.empty((1, P_big, block.shape[1]), dtype=block.dtype)
        for r0 in range(0, P_big, period):
            n = min(period, P_big - r0)
            big[0, r0:r0 + n] = block[:n]
        w["pool_" + side] = big
        idx = rng.integers(0, P_big, size=(T, 1), dtype=np.int64)
        high = rng.random((T, 1)) < 0.5
        idx[high] = rng.integers(1 << 24, P_big, size=int(high.sum()))
        idx[0, 0], idx[1, 0] = P_big - 1, 1 << 24
        w["idx_" + side] = idx.astype(np.int32)
    w["P"] = P_big
    assert w["pool_k"].nbytes > 1 << 32 and int(w["idx_k"].max()) * w["pool_ld"] * 2 >= 1 << 32
    ckv, session = gpu
    ckv.ckv_set_option("mfma_impl", "staged" if kind == "staged" else None)
    try:
        say(f"[case] pool beyond 4 GiB, {kind}: P={P_big}, {w['pool_k'].nbytes / 2**30:.2f} GiB per side")
        with session.Session(w) as s:
            variant = ckv.ckv_variant(s.cache)
            say(f"  variant {variant}")
            assert variant.startswith({"dma": "mfma_dma", "staged": "mfma_bf16", "stream": "stream"}[kind]), variant
            s.attend()
            out = s.output()
            k_full, v_full = s.reconstruct()
    finally:
        ckv.ckv_set_option(None)
    ok, ov = oracle.reconstruct(w)
    assert np.array_equal(k_full, ok.transpose(1, 0, 2)) and np.array_equal(v_full, ov.transpose(1, 0, 2))
    norm = check_against_oracle(out, w, what=f"pool beyond 4 GiB ({kind})")
    say(f"  ok, norm-wise error {norm:.3e}, rows bit-exact")


def random_shape(block, case):
    """Seeded random shape number `case` of block `block`, drawn over everything the dispatcher looks at (storage
    type, head width, user width, pool stride, query count, weighting, which side is shared, ragged lengths with
    empty histories).  Returns (workload, description)."""
    rng = np.random.default_rng(1000 * block + case)
    matrix = rng.random() < 0.6
    if matrix:
        dtype, d_a = wl.BF16, int(rng.choice([64, 128, 256]))
        d_u = int(rng.choice([0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 14, 16, 24]))
        Nq = int(rng.integers(8, 300))
    else:
        dtype = int(rng.choice([wl.F32, wl.BF16]))
        d_a = int(rng.choice([8, 12, 16, 40, 64, 72, 128, 200]))
        d_u = int(rng.integers(0, min(d_a, 16) + 1))
        Nq = int(rng.integers(1, 8))
    d_g = d_a - d_u
    align = 8 if matrix else 1
    pool_ld = 0 if d_g == 0 else int(rng.choice([(d_g + align - 1) // align * align, d_a, d_a + 8]))
    if d_g > 0 and pool_ld < d_g:
        pool_ld = d_a
    share = int(rng.choice([wl.SHARE_KV, wl.SHARE_KV, wl.SHARE_K, wl.SHARE_V])) if d_g > 0 else wl.SHARE_KV
    mode = int(rng.choice([wl.SOFTMAX, wl.SILU_OVER_N]))
    B = int(rng.integers(1, 9))
    lengths = rng.choice([0, 1, 31, 32, 33, 64, 100, 257, 900, 3000], size=B).astype(np.int32)
    H, P = int(rng.integers(1, 4)), int(rng.choice([1, 2, 77, 700, 5000]))
    kw = dict(pool_ld=pool_ld) if d_g > 0 else {}
    w = make(lengths, dtype, mode, d_a=d_a, d_u=d_u, H=H, P=P, Nq=Nq, seed=2000 + 100 * block + case,
             idx=("zipf", 1.1) if rng.random() < 0.3 else "uniform", share=share, **kw)
    return w, f"random shape {block}.{case}: d_a={d_a} d_u={d_u} ld={pool_ld} share={share} lengths={lengths.tolist()}"


@pytest.mark.parametrize("block", range(4))
def test_seeded_random_shapes(gpu, block):
    """Twelve seeded random shapes per block, each against the oracle element by element."""
    for case in range(12):
        w, what = random_shape(block, case)
        run_and_check(gpu, w, what)


# Shapes of further blocks of the same generator (blocks 4 to 109 were run once) on which a comparison rule with a
# floor of tol * rms(output row) failed by 1e-7 to 1e-4 on a few elements: rows whose summands nearly cancel (SiLU
# weights of both signs over a pool of one or two rows, or a handful of positions), so that the output row is far
# smaller than what was added up.  All fourteen are kept; the rule in tests/parity.py scales the floor with the
# summands of each element instead.
NEAR_CANCELLING = [(26, 6), (39, 7), (43, 10), (47, 0), (57, 2), (59, 9), (67, 10), (72, 6), (75, 7), (82, 9), (84, 4),
                   (99, 0), (103, 9), (104, 1)]


@pytest.mark.parametrize("block,case", NEAR_CANCELLING)
def test_random_shapes_with_near_cancelling_rows(gpu, block, case):
    w, what = random_shape(block, case)
    run_and_check(gpu, w, what)


def random_shape_many_queries(case):
    """Seeded random shape number `case` of a second generator, aimed at the fp32 matrix-core kernels and the
    register-staged bf16 kernel: head widths that are not 64, 128 or 256 columns, wide and odd user slices, six queries
    or more, pools of one or two rows among the sizes.  Returns (workload, description)."""
    rng = np.random.default_rng(777000 + case)
    fp32 = rng.random() < 0.5
    dtype = wl.F32 if fp32 else wl.BF16
    if fp32:
        d_a = int(rng.choice([8, 16, 24, 48, 64, 72, 96, 100, 128, 130, 160, 192, 200, 256]))
    else:
        d_a = int(rng.choice([8, 16, 24, 32, 40, 48, 56, 72, 80, 96, 104, 120, 64, 128]))
    d_u = min(int(rng.choice([0, 1, 2, 3, 4, 5, 8, 9, 12, 16, 20, 24, 32])), d_a)
    if not fp32 and d_a in (64, 128):  # user widths that the direct-to-LDS kernel does not take
        d_u = int(rng.choice([9, 11, 20, 24, 32]))
    d_g = d_a - d_u
    al = 4 if fp32 else 8
    pool_ld = 0 if d_g == 0 else int(rng.choice([(d_g + al - 1) // al * al, (d_a + al - 1) // al * al, (d_a + al - 1) // al * al + al]))
    Nq = int(rng.choice([6, 8, 9, 16, 31, 32, 33, 40, 64, 65, 100, 128, 129, 200]))
    share = int(rng.choice([wl.SHARE_KV, wl.SHARE_KV, wl.SHARE_K, wl.SHARE_V])) if d_g > 0 else wl.SHARE_KV
    mode = int(rng.choice([wl.SOFTMAX, wl.SILU_OVER_N]))
    B = int(rng.integers(1, 6))
    lengths = rng.choice([0, 1, 31, 32, 33, 64, 100, 257, 900, 2500], size=B).astype(np.int32)
    H, P = int(rng.integers(1, 3)), int(rng.choice([1, 2, 77, 700, 3000]))
    kw = dict(pool_ld=pool_ld) if d_g > 0 else {}
    w = wl.make(B=B, L=None, H=H, d_a=d_a, d_u=d_u, P=P, idx=("zipf", 1.1) if rng.random() < 0.3 else "uniform", Nq=Nq, mode=mode,
                dtype=dtype, sigma_pool=d_a ** -0.5, seed=5000 + case, lengths=lengths, share=share, **kw)
    return w, (f"random many-query shape {case}: dtype={'f32' if fp32 else 'bf16'} d_a={d_a} d_u={d_u} ld={pool_ld} Nq={Nq} "
               f"share={share} lengths={lengths.tolist()}")


@pytest.mark.parametrize("block", range(4))
def test_seeded_random_shapes_many_queries(gpu, block):
    """Forty seeded shapes of the second generator per block.  Case 77 (fp32, keys from a pool of one row, values an
    ordinary cache, 64 positions: all weights equal, some value columns nearly cancel) is the shape that showed the
    comparison rule needs its term for the rounding of the additions."""
    for case in range(40 * block, 40 * block + 40):
        w, what = random_shape_many_queries(case)
        run_and_check(gpu, w, what)


def random_shape_few_queries(case):
    """Seeded random shape number `case` of a third generator, aimed at the two streaming kernels: one to seven queries,
    head widths from 8 to 512 columns, any user width, pool strides that are and are not whole 16-byte lanes, now and then
    a thousand short histories (two wavefronts per item), a forced number of wavefronts per item, or an unusual scale.
    Returns (workload, description, options)."""
    rng = np.random.default_rng(880000 + case)
    fp32 = rng.random() < 0.4
    dtype = wl.F32 if fp32 else wl.BF16
    e = 4 if fp32 else 2
    d_a = int(rng.choice([8, 16, 24, 32, 40, 48, 64, 72, 96, 100, 128, 130, 160, 192, 200, 255, 256, 320, 512]))
    d_u = min(int(rng.choice([0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 16, 20, 24, 32, 33, 64])), d_a)
    if rng.random() < 0.08:
        d_u = d_a
    d_g = d_a - d_u
    al = 16 // e
    pool_ld = 0 if d_g == 0 else int(rng.choice([(d_g + al - 1) // al * al, (d_a + al - 1) // al * al, (d_a + al - 1) // al * al + al, d_g, d_a + 1]))
    if d_g > 0 and pool_ld < d_g:
        pool_ld = d_g
    Nq = int(rng.choice([1, 1, 1, 2, 2, 3, 4, 5, 7]))
    share = int(rng.choice([wl.SHARE_KV, wl.SHARE_KV, wl.SHARE_K, wl.SHARE_V])) if d_g > 0 else wl.SHARE_KV
    mode = int(rng.choice([wl.SOFTMAX, wl.SILU_OVER_N]))
    B = int(rng.integers(1, 7))
    lengths = rng.choice([0, 1, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 255, 256, 257, 513, 900, 2500, 6000], size=B).astype(np.int32)
    if rng.random() < 0.1:
        B = int(rng.integers(800, 1500))
        lengths = rng.integers(0, 90, size=B).astype(np.int32)
    H, P = int(rng.integers(1, 4)), int(rng.choice([1, 2, 77, 700, 3000]))
    opts = {}
    if rng.random() < 0.25:
        opts["stream_waves"] = str(rng.choice([2, 4]))
    kw = dict(pool_ld=pool_ld) if d_g > 0 else {}
    scale = None if rng.random() < 0.8 else float(rng.choice([-0.3, 2.0, 5.0]))
    zipf = rng.random() < 0.3
    w = wl.make(B=B, L=None, H=H, d_a=d_a, d_u=d_u, P=P, idx=("zipf", 1.1) if zipf else "uniform", Nq=Nq, mode=mode,
                dtype=dtype, sigma_pool=d_a ** -0.5, seed=6000 + case, lengths=lengths, share=share, scale=scale, **kw)
    return w, (f"random few-query shape {case}: dtype={'f32' if fp32 else 'bf16'} d_a={d_a} d_u={d_u} ld={pool_ld} Nq={Nq} share={share} "
               f"scale={scale} options={opts} lengths={lengths.tolist()[:8]}"), opts


@pytest.mark.parametrize("block", range(3))
def test_seeded_random_shapes_few_queries(gpu, block):
    """Forty seeded shapes of the third generator per block (1200 were run once, none failed).  Rows of more than 256
    columns on strides that allow no vector loads are refused when the handle is built (the documented limit of the
    streaming kernels); such a case only checks that."""
    ckv, session = gpu
    for case in range(40 * block, 40 * block + 40):
        w, what, opts = random_shape_few_queries(case)
        try:
            for k, v in opts.items():
                ckv.ckv_set_option(k, v)
            try:
                _run_and_check(ckv, session, w, what, None, None)
            except ckv.CkvError as e:
                assert e.code == ckv.CKV_ERR_UNSUPPORTED and w["d_g"] + w["d_u"] > 256 and "limit" in str(e), what
                say(f"  refused: {e}")
        finally:
            ckv.ckv_set_option(None)


@pytest.mark.parametrize("dtype,d_a,Nq", [(wl.F32, 130, 9), (wl.F32, 64, 1), (wl.BF16, 128, 9), (wl.BF16, 72, 16), (wl.BF16, 64, 2)])
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
def test_equal_weights_over_cancelling_value_rows(gpu, mode, dtype, d_a, Nq):
    # keys from a pool of one row and no user columns: every position has the same weight; the values are an ordinary cache
    w = make([64, 64, 31, 1000, 1], dtype, mode, d_a=d_a, d_u=0, H=2, P=1, Nq=Nq, seed=5077, share=wl.SHARE_K,
             pool_ld=(d_a + 7) // 8 * 8)
    run_and_check(gpu, w, f"equal weights, dtype {dtype}, d_a={d_a}, Nq={Nq}, mode {mode}")


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_a,d_u,pool_ld,Nq", [(96, 8, 88, 64), (32, 4, 32, 16), (40, 5, 40, 20), (120, 16, 104, 130),
                                                 (8, 2, 8, 9), (72, 0, 72, 33), (100, 3, 104, 64), (56, 56, 0, 40)])
def test_narrow_heads_run_in_the_next_wider_matrix_core_kernel(gpu, mode, d_a, d_u, pool_ld, Nq):
    """bf16 heads narrower than 64 or 128 columns, many queries: the register-staged kernel with zero columns."""
    w = make(MFMA_LENGTHS, wl.BF16, mode, d_a=d_a, d_u=d_u, H=2, P=700, Nq=Nq, **({"pool_ld": pool_ld} if pool_ld else {}))
    run_and_check(gpu, w, f"narrow head d_a={d_a} d_u={d_u} ld={pool_ld} Nq={Nq} mode={mode}",
                  expect_variant=f"mfma_bf16_d{64 if d_a <= 64 else 128}")


def test_narrow_head_split_history_and_one_side_shared(gpu):
    w = make((5000, 70, 2300), wl.BF16, wl.SOFTMAX, d_a=96, d_u=8, H=2, P=5000, Nq=64, pool_ld=88)
    run_and_check(gpu, w, "narrow head, split history", expect_variant="mfma_bf16_d128")
    for share in (wl.SHARE_K, wl.SHARE_V):
        w = make(MFMA_LENGTHS, wl.BF16, wl.SILU_OVER_N, d_a=48, d_u=4, H=2, P=300, Nq=32, share=share)
        run_and_check(gpu, w, f"narrow head, share={share}", expect_variant="mfma_bf16_d64")


# ---------------------------------------------------------------------------------------------
# fp32 storage, many queries: the fp32 matrix instruction
@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_a,d_u,pool_ld,Nq", [(64, 8, 64, 64), (128, 8, 128, 128), (64, 4, 60, 16), (128, 0, 128, 40),
                                                 (64, 3, 64, 20), (96, 8, 88, 33), (128, 24, 104, 200), (32, 32, 0, 9),
                                                 (100, 5, 96, 64), (8, 2, 8, 8), (64, 8, 64, 100), (48, 4, 48, 129)])
def test_fp32_many_queries(gpu, mode, d_a, d_u, pool_ld, Nq):
    """64 queries or fewer per user: wavefront pairs split the columns (work items of 64 queries); more: one wavefront per
    32 queries (work items of 128 queries)."""
    w = make(MFMA_LENGTHS, wl.F32, mode, d_a=d_a, d_u=d_u, H=2, P=700, Nq=Nq, **({"pool_ld": pool_ld} if pool_ld else {}))
    run_and_check(gpu, w, f"fp32 many queries d_a={d_a} d_u={d_u} ld={pool_ld} Nq={Nq} mode={mode}",
                  expect_variant=f"mfma_f32_d{64 if d_a <= 64 else 128}")


def test_fp32_many_queries_split_history_sharing_and_large_scores(gpu):
    w = make((5000, 70, 2300, 1024, 1025), wl.F32, wl.SOFTMAX, d_a=128, d_u=8, H=2, P=5000, Nq=128)
    run_and_check(gpu, w, "fp32 many queries, split history", expect_variant="mfma_f32_d128")
    for share in (wl.SHARE_K, wl.SHARE_V):
        w = make(MFMA_LENGTHS, wl.F32, wl.SILU_OVER_N, d_a=64, d_u=4, H=2, P=300, Nq=32, share=share)
        run_and_check(gpu, w, f"fp32 many queries, share={share}", expect_variant="mfma_f32_d64")
    w = make((700, 129), wl.F32, wl.SOFTMAX, d_a=64, d_u=8, H=1, P=300, Nq=32, sigma_q=6.0, scale=1.0)
    run_and_check(gpu, w, "fp32 many queries, large scores", expect_variant="mfma_f32_d64")
    w = make((70, 33), wl.F32, wl.SOFTMAX, d_a=64, d_u=8, H=1, P=50, Nq=16, scale=-0.125)
    run_and_check(gpu, w, "fp32 negative scale", expect_variant="stream")


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_a,d_u,pool_ld,Nq", [(256, 8, 256, 128), (256, 0, 256, 16), (192, 16, 176, 64), (200, 5, 200, 40),
                                                 (136, 8, 128, 200)])
def test_wide_bf16_heads_many_queries(gpu, mode, d_a, d_u, pool_ld, Nq):
    """Heads of 129 to 256 columns: the 256-column register-staged kernel (one workgroup per compute unit)."""
    w = make(MFMA_LENGTHS, wl.BF16, mode, d_a=d_a, d_u=d_u, H=2, P=700, Nq=Nq, pool_ld=pool_ld)
    run_and_check(gpu, w, f"wide head d_a={d_a} d_u={d_u} ld={pool_ld} Nq={Nq} mode={mode}", expect_variant="mfma_bf16_d256",
                  impl="staged")


def test_wide_bf16_head_split_history(gpu):
    w = make((5000, 70, 2300), wl.BF16, wl.SOFTMAX, d_a=256, d_u=8, H=2, P=5000, Nq=64)
    run_and_check(gpu, w, "wide head, split history", expect_variant="mfma_bf16_d256", impl="staged")


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_u,Nq", [(1, 128), (2, 64), (3, 40), (4, 128), (6, 200), (10, 128), (10, 64), (16, 33), (8, 3), (0, 16),
                                    (24, 128), (32, 64), (20, 40), (30, 200)])
def test_256_column_heads_in_the_direct_to_lds_kernel(gpu, mode, d_u, Nq):
    """d_a = 256 with the user widths behind the compression ratios of Table 1 (d_u = 1, 2, 3, 4, 6, 10) and up to the
    widest slice the kernel appends (32): rows of 512 bytes, up to four slice loads per wavefront and tile."""
    w = make(MFMA_LENGTHS, wl.BF16, mode, d_a=256, d_u=d_u, H=3, P=700, Nq=Nq)
    run_and_check(gpu, w, f"256 columns d_u={d_u} Nq={Nq} mode={mode}",
                  expect_variant="mfma_dma_bf16_d256_w4")


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_a,d_u,Nq", [(128, 10, 128), (128, 12, 64), (128, 16, 32), (128, 14, 100), (64, 10, 64), (64, 16, 128),
                                         (64, 12, 16), (128, 16, 3)])
def test_user_slices_of_ten_to_sixteen_columns_in_the_direct_to_lds_kernel(gpu, mode, d_a, d_u, Nq):
    """Even d_u from 10 to 16 at 64 and 128 columns: the instantiation with the larger slice staging area, with one,
    two and four wavefronts (up to eight slice loads per wavefront and tile)."""
    w = make(MFMA_LENGTHS, wl.BF16, mode, d_a=d_a, d_u=d_u, H=3, P=700, Nq=Nq)
    nw = 1 if Nq <= 32 else (2 if Nq <= 64 else 4)
    run_and_check(gpu, w, f"wide slices d_a={d_a} d_u={d_u} Nq={Nq} mode={mode}", expect_variant=f"mfma_dma_bf16_d{d_a}_w{nw}_g1")


def test_wide_user_slices_split_history_and_one_side_shared(gpu):
    w = make((5000, 70, 2300), wl.BF16, wl.SOFTMAX, d_a=128, d_u=12, H=2, P=5000, Nq=64)
    run_and_check(gpu, w, "wide slices, split history", expect_variant="mfma_dma_bf16_d128_w2")
    for share in (wl.SHARE_K, wl.SHARE_V):
        w = make(MFMA_LENGTHS, wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=10, H=2, P=300, Nq=96, share=share)
        run_and_check(gpu, w, f"wide slices, share={share}", expect_variant="mfma_dma_bf16_d64_w4")


def test_256_column_heads_split_history_one_side_shared_and_plain_cache(gpu):
    w = make((5000, 70, 2300), wl.BF16, wl.SOFTMAX, d_a=256, d_u=8, H=2, P=5000, Nq=64)
    run_and_check(gpu, w, "256 columns, split history", expect_variant="mfma_dma_bf16_d256_w4")
    w = make((9000, 31), wl.BF16, wl.SOFTMAX, d_a=256, d_u=10, H=1, P=3000, Nq=128)
    run_and_check(gpu, w, "256 columns, split history, d_u=10", expect_variant="mfma_dma_bf16_d256_w4")
    for share in (wl.SHARE_K, wl.SHARE_V):
        w = make(MFMA_LENGTHS, wl.BF16, wl.SILU_OVER_N, d_a=256, d_u=4, H=2, P=300, Nq=96, share=share)
        run_and_check(gpu, w, f"256 columns, share={share}", expect_variant="mfma_dma_bf16_d256_w4")
    w = make(MFMA_LENGTHS, wl.BF16, wl.SOFTMAX, d_a=256, d_u=256, H=2, P=1, Nq=128)
    run_and_check(gpu, w, "256 columns, ordinary cache", expect_variant="mfma_dma_bf16_d256_w4")


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_a,d_u,pool_ld,Nq", [(256, 8, 256, 128), (192, 16, 176, 40), (130, 3, 128, 9)])
def test_wide_fp32_heads_many_queries(gpu, mode, d_a, d_u, pool_ld, Nq):
    w = make(MFMA_LENGTHS, wl.F32, mode, d_a=d_a, d_u=d_u, H=2, P=700, Nq=Nq, pool_ld=pool_ld)
    run_and_check(gpu, w, f"wide fp32 head d_a={d_a} d_u={d_u} ld={pool_ld} Nq={Nq} mode={mode}", expect_variant="mfma_f32_d256")


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("Nq", [9, 32, 33, 64, 65, 200])
def test_wide_fp32_heads_query_blocks(gpu, mode, Nq):
    """The 256-column fp32 kernel serves 64 queries per work item with wavefront pairs that split the columns:
    a pair without queries (Nq <= 32), exactly one and two full pairs, a second block of one query, several blocks;
    one history long enough to be cut into pieces that meet in the merge kernel."""
    w = make((3000, 70, 1, 257), wl.F32, mode, d_a=256, d_u=12, H=2, P=900, Nq=Nq)
    run_and_check(gpu, w, f"wide fp32 head Nq={Nq} mode={mode}", expect_variant="mfma_f32_d256")


@pytest.mark.parametrize("share", [wl.SHARE_K, wl.SHARE_V])
def test_wide_fp32_heads_one_side_shared_and_plain_cache(gpu, share):
    w = make(MFMA_LENGTHS, wl.F32, wl.SOFTMAX, d_a=200, d_u=8, H=2, P=300, Nq=70, share=share)
    run_and_check(gpu, w, f"wide fp32 head, share={share}", expect_variant="mfma_f32_d256")
    w = make(MFMA_LENGTHS, wl.F32, wl.SILU_OVER_N, d_a=256, d_u=256, H=2, P=1, Nq=64)
    run_and_check(gpu, w, "wide fp32 head, ordinary cache", expect_variant="mfma_f32_d256")


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("dtype,d_a,d_u,Nq,expect", [(wl.BF16, 64, 8, 3, "mfma_dma_bf16_d64_w1"), (wl.BF16, 128, 4, 5, "mfma_dma_bf16_d128_w1"),
                                                      (wl.BF16, 64, 2, 7, "mfma_dma_bf16_d64_w1"), (wl.BF16, 64, 8, 2, "stream"),
                                                      (wl.BF16, 64, 9, 7, "stream"), (wl.BF16, 64, 1, 4, "mfma_dma_bf16_d64_w1"), (wl.F32, 64, 8, 6, "mfma_f32_d64"),
                                                      (wl.F32, 128, 8, 5, "stream"), (wl.F32, 128, 8, 7, "mfma_f32_d128")])
def test_few_queries_cross_over_to_the_matrix_core_kernels(gpu, mode, dtype, d_a, d_u, Nq, expect):
    """The streaming kernel's time grows with the number of queries, the matrix-core kernels' does not: from three
    queries on (six in fp32, eight for the register-staged kernel) the matrix-core kernels are chosen."""
    w = make(MFMA_LENGTHS, dtype, mode, d_a=d_a, d_u=d_u, H=2, P=700, Nq=Nq)
    run_and_check(gpu, w, f"few queries dtype={dtype} d_a={d_a} d_u={d_u} Nq={Nq} mode={mode}", expect_variant=expect)


@pytest.mark.parametrize("mode", [wl.SOFTMAX, wl.SILU_OVER_N])
@pytest.mark.parametrize("d_a,d_u,Nq", [(64, 1, 16), (64, 1, 64), (64, 1, 128), (128, 1, 128), (128, 3, 32), (64, 3, 64), (128, 3, 100), (128, 1, 40),
                                         (128, 5, 128), (64, 7, 64), (128, 7, 20), (64, 5, 100), (256, 5, 64), (256, 7, 128)])
def test_odd_user_width_in_the_direct_to_lds_kernel(gpu, mode, d_a, d_u, Nq):
    """d_u of 1 (the paper's smallest cache, CR = 2 / d_a) and 3: the slices cannot be moved as whole dwords; with an
    odd number of positions before a head (T is odd here) its slices start on odd elements too."""
    assert sum(MFMA_LENGTHS) % 2 == 1
    w = make(MFMA_LENGTHS, wl.BF16, mode, d_a=d_a, d_u=d_u, H=3, P=700, Nq=Nq)
    run_and_check(gpu, w, f"odd d_u: d_a={d_a} d_u={d_u} Nq={Nq} mode={mode}", expect_variant="mfma_dma")


def test_odd_user_width_split_history_and_one_side_shared(gpu):
    w = make((5001, 70, 2300, 1023), wl.BF16, wl.SOFTMAX, d_a=128, d_u=1, H=2, P=5000, Nq=128)
    run_and_check(gpu, w, "odd d_u, split history", expect_variant="mfma_dma")
    for share in (wl.SHARE_K, wl.SHARE_V):
        w = make(MFMA_LENGTHS, wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=3, H=2, P=300, Nq=32, share=share)
        run_and_check(gpu, w, f"odd d_u, share={share}", expect_variant="mfma_dma")


@pytest.mark.parametrize("kind", ["dma", "fp32", "stream", "staged"])
def test_one_very_long_history(gpu, kind):
    """A single user with 150000 positions: the history is cut into hundreds of pieces over the whole chip and merged
    (several chunks of pieces in the merge kernel); accuracy must hold over the long sums."""
    n = 150001
    if kind == "dma":
        w = make((n,), wl.BF16, wl.SOFTMAX, d_a=128, d_u=8, H=2, P=20000, Nq=64, idx=("zipf", 1.05))
        expect = "mfma_dma"
    elif kind == "fp32":
        w = make((n,), wl.F32, wl.SILU_OVER_N, d_a=64, d_u=4, H=1, P=20000, Nq=32)
        expect = "mfma_f32"
    elif kind == "staged":
        w = make((n,), wl.BF16, wl.SOFTMAX, d_a=64, d_u=24, H=1, P=20000, Nq=32)
        expect = "mfma_bf16"
    else:
        w = make((n, 3), wl.F32, wl.SOFTMAX, d_a=64, d_u=8, H=2, P=20000, Nq=2)
        expect = "stream"
    run_and_check(gpu, w, f"one very long history ({kind})", expect_variant=expect)
