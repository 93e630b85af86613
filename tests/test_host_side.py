"""CPU-only checks of the host side: the built library exports what include/ckv.h declares,
argument validation that happens before any device call, and the workload generators."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2601_19178_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "ckv.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ckv_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    from paper_2601_19178_amd import ckv
    names = declared_functions()
    assert "ckv_build_cache" in names and "ckv_attend" in names and len(names) >= 12
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2601_19178_amd", "libckv.so"))
    for n in names:
        assert hasattr(lib, n), f"libckv.so does not export {n}"
    assert sorted(ckv.EXPORTS) == names          # the binding covers the same set, same names
    for n in names:
        assert hasattr(ckv, n)


def test_shape_struct_matches_header_layout():
    from paper_2601_19178_amd import ckv
    assert ctypes.sizeof(ckv.ckv_shape) == 48
    assert ckv.ckv_shape.pool_ld.offset == 40 and ckv.ckv_shape.scale.offset == 32


def test_build_cache_validates_before_touching_the_device():
    from paper_2601_19178_amd import ckv
    good = dict(B=2, H=1, d_g=8, d_u=0, P=4, Nq=1, dtype=0, mode=0, scale=1.0, pool_ld=8)
    lengths = np.array([1, 1], np.int32)
    zeros = np.zeros((2, 1), np.int32)

    def expect(code, lengths=lengths, idx=(zeros, zeros), **over):
        sh = ckv.make_shape(**{**good, **over})
        with pytest.raises(ckv.CkvError) as e:
            ckv.ckv_build_cache(sh, lengths, idx[0], idx[1], None, None)
        assert e.value.code == code, str(e.value)
        assert ckv.ckv_last_error() in str(e.value)

    expect(ckv.CKV_ERR_SHAPE, B=0)
    expect(ckv.CKV_ERR_SHAPE, H=0)
    expect(ckv.CKV_ERR_SHAPE, d_g=0, d_u=0)
    expect(ckv.CKV_ERR_SHAPE, d_u=-1)
    expect(ckv.CKV_ERR_SHAPE, Nq=0)
    expect(ckv.CKV_ERR_SHAPE, pool_ld=7)
    expect(ckv.CKV_ERR_SHAPE, P=0)
    expect(ckv.CKV_ERR_SHAPE, dtype=2)
    expect(ckv.CKV_ERR_SHAPE, mode=5)
    expect(ckv.CKV_ERR_SHAPE, scale=float("nan"))
    expect(ckv.CKV_ERR_SHAPE, share=3)
    # wider than the streaming kernel serves at this alignment (scalar loads: 256 columns), and no matrix-core shape
    expect(ckv.CKV_ERR_UNSUPPORTED, d_g=257, pool_ld=257)
    # sharing only the keys: idx_v may be absent, idx_k may not
    expect(ckv.CKV_ERR_NULL, idx=(None, zeros), share=ckv.CKV_SHARE_K)
    expect(ckv.CKV_ERR_LENGTH, lengths=np.array([3, -2], np.int32))
    expect(ckv.CKV_ERR_NULL, idx=(None, zeros))
    expect(ckv.CKV_ERR_NULL, d_u=2)          # user slices missing
    with pytest.raises(ckv.CkvError) as e:
        ckv._check(ckv._lib.ckv_attend(None, None, None, None, None, None, None, None, None, None))
    assert e.value.code == ckv.CKV_ERR_NULL


def test_options_are_validated_and_steer_the_plan():
    """ckv_set_option: unknown keys and malformed values are refused; "mfma_impl" moves a shape from the
    direct-to-LDS kernel to the register-staged one (seen through ckv_plan, no device); key None restores defaults."""
    from paper_2601_19178_amd import ckv
    for key, value in (("no_such_option", "1"), ("mfma_impl", "fastest"), ("dma_sched", "lazy"), ("dma_shape", "4"),
                       ("dma_shape", "0,1"), ("dma_slow_speed", "fast"), ("dma_slow_speed", "-1"), ("stream_impl", "wide"), ("stream_waves", "3"), ("stream_hot_rows", "33"), ("stream_hot_rows", "many"),
                       ("dma_scores_ahead", "yes"), ("dma_q16", "2")):
        with pytest.raises(ckv.CkvError) as e:
            ckv.ckv_set_option(key, value)
        assert e.value.code == ckv.CKV_ERR_UNSUPPORTED
    sh = ckv.make_shape(B=3, H=2, d_g=56, d_u=8, P=100, Nq=64, dtype=ckv.CKV_BF16, mode=0, scale=0.125, pool_ld=64)
    lengths = np.array([100, 900, 33], np.int32)
    try:
        assert ckv.ckv_plan(sh, lengths)[2].startswith("mfma_dma_bf16_d64")
        ckv.ckv_set_option("mfma_impl", "staged")
        assert ckv.ckv_plan(sh, lengths)[2].startswith("mfma_bf16_d64")
        ckv.ckv_set_option("mfma_impl", "auto")
        assert ckv.ckv_plan(sh, lengths)[2].startswith("mfma_dma_bf16_d64")
        ckv.ckv_set_option("dma_shape", "4,1")
        assert "_w4_g1" in ckv.ckv_plan(sh, lengths)[2]
        ckv.ckv_set_option("dma_shape", "")
        few = ckv.make_shape(B=3, H=2, d_g=56, d_u=8, P=100, Nq=12, dtype=ckv.CKV_BF16, mode=0, scale=0.125, pool_ld=64)
        assert "_w1_q16_" in ckv.ckv_plan(few, lengths)[2]
        ckv.ckv_set_option("dma_q16", "0")
        assert "_w1_g1_" in ckv.ckv_plan(few, lengths)[2]
        ckv.ckv_set_option("dma_q16", None)
        assert "_w1_q16_" in ckv.ckv_plan(few, lengths)[2]
        rec_static, nwg_static, _ = ckv.ckv_plan(sh, lengths)
        ckv.ckv_set_option("dma_sched", "dynamic")
        rec_dyn, nwg_dyn, _ = ckv.ckv_plan(sh, lengths)
        assert nwg_dyn == len(rec_dyn) and nwg_static != nwg_dyn      # one workgroup per item instead of persistent ones
        ckv.ckv_set_option("mfma_impl", "staged")
        ckv.ckv_set_option(None)
        assert ckv.ckv_plan(sh, lengths)[2].startswith("mfma_dma_bf16_d64") and ckv.ckv_plan(sh, lengths)[1] == nwg_static
        # one query over 256 columns with a user width that breaks the 8- and 16-byte alignment: wide-row streaming kernel
        # unless the column-block one is asked for
        st = ckv.make_shape(B=3, H=2, d_g=246, d_u=10, P=100, Nq=1, dtype=ckv.CKV_BF16, mode=0, scale=0.0625, pool_ld=256)
        assert ckv.ckv_plan(st, lengths)[2].startswith("streamw_bf16_g32_q1")
        ckv.ckv_set_option("stream_impl", "narrow")
        assert ckv.ckv_plan(st, lengths)[2].startswith("stream_bf16_v1_c16")
        ckv.ckv_set_option("stream_impl", "auto")
        assert ckv.ckv_plan(st, lengths)[2].startswith("streamw_bf16_g32_q1")
        # many short items: two wavefronts per item
        many = ckv.make_shape(B=3000, H=2, d_g=246, d_u=10, P=100, Nq=1, dtype=ckv.CKV_BF16, mode=0, scale=0.0625, pool_ld=256)
        assert ckv.ckv_plan(many, np.full(3000, 150, np.int32))[2].endswith("_w2")
        assert not ckv.ckv_plan(many, np.full(3000, 1500, np.int32))[2].endswith("_w2")
    finally:
        ckv.ckv_set_option(None)


def test_workloads_are_seeded_and_shaped():
    a, b = wl.config("cfg1"), wl.config("cfg1")
    for k, v in a.items():
        if isinstance(v, np.ndarray):
            np.testing.assert_array_equal(v, b[k])
    assert a["idx_k"].shape == (200, 1) and a["user_k"].shape == (200, 1, 8) and a["pool_k"].shape == (1, 256, 64)
    assert a["q"].shape == (4, 1, 1, 64) and a["idx_k"].min() >= 0 and a["idx_k"].max() < 256
    assert not np.array_equal(a["idx_k"], a["idx_v"])
    c = wl.config("cfg1", seed=5)
    assert not np.array_equal(a["idx_k"], c["idx_k"])
    r = wl.config("cfg4", B=16, P=512)
    assert r["lengths"].min() >= 2048 and r["lengths"].max() <= 8192 and r["user_k"].dtype == np.uint16
    assert abs(wl.to_f64(r["pool_k"][..., :120], wl.BF16).std() - 128 ** -0.5) < 2e-3


def test_zipf_indices_are_skewed_and_in_range():
    w = wl.config("cfg3", B=64, L=(256, 256))
    cnt = np.sort(np.bincount(w["idx_k"][:, 0], minlength=w["P"]))[::-1]
    assert w["idx_k"].max() < w["P"] and w["idx_k"].min() >= 0
    top64 = cnt[:64].sum() / cnt.sum()
    assert 0.5 < top64 < 0.68          # bounded Zipf(1.1) over 16384 ranks puts ~59 % on the top 64
    hot = np.argsort(np.bincount(w["idx_k"][:, 0], minlength=w["P"]))[::-1][:8]
    assert np.ptp(hot) > 64            # hot rows are scattered by the rank permutation


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40], dtype=np.float32)
    b = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625) and back[3] == -2.5
    import torch
    t = torch.from_numpy(np.random.default_rng(0).standard_normal(4096).astype(np.float32))
    ref = t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(wl.f32_to_bf16_bits(t.numpy()), ref)


def test_algorithmic_bytes_of_the_workloads():
    # compressed stream + gathered rows + q + out, per position-head 8 + 2*d_u*e and 2*d_g*e
    w = wl.config("cfg3", B=4)
    ab = wl.algorithmic_bytes(w)
    assert ab["position_heads"] == 4 * 1024 * 4
    assert ab["compressed"] == ab["position_heads"] * 24 and ab["gathered"] == ab["position_heads"] * 240
    assert ab["q_out"] == 2 * 4 * 4 * 64 * 64 * 2
