"""CPU-only checks of the scheduling arithmetic (ckv_plan): whatever the kernel family and however the
histories are cut and distributed, every (user, head, query block) must be covered exactly once."""
import numpy as np
import pytest

from paper_2601_19178_amd import ckv

F32, BF16 = 0, 1


def plan(lengths, H, d_a, d_u, Nq, dtype, mode=0, cus=256, wg_per_cu=2, share=0):
    lengths = np.asarray(lengths, dtype=np.int32)
    sh = ckv.make_shape(len(lengths), H, d_a - d_u, d_u, 1000, Nq, dtype, mode, 0.125, d_a, share)
    rec, nwg, name = ckv.ckv_plan(sh, lengths, cus, wg_per_cu)
    return lengths, rec, nwg, name


def check_cover(lengths, rec, H, Nq, name):
    offs = np.concatenate([[0], np.cumsum(lengths.astype(np.int64))])
    groups = {}
    for b, h, q0, n, t0, part, n_total, wg in rec.tolist():
        assert 0 <= b < len(lengths) and 0 <= h < H and 0 <= q0 < Nq
        assert n_total == lengths[b] and 0 <= n <= n_total
        assert offs[b] <= t0 and t0 + n <= offs[b + 1]
        groups.setdefault((b, h, q0), []).append((t0 - offs[b], n, part))
    q0s = sorted({k[2] for k in groups})
    qb = q0s[1] - q0s[0] if len(q0s) > 1 else Nq
    assert q0s == list(range(0, Nq, qb)) or len(q0s) == 1
    assert len(groups) == len(lengths) * H * len(q0s), f"{name}: some (user, head, query block) is missing"
    seen_parts = set()
    for (b, h, q0), pieces in groups.items():
        pieces.sort()
        pos = 0
        for lo, n, part in pieces:
            assert lo == pos, f"{name}: pieces of user {b} head {h} overlap or leave a gap"
            pos += n
        assert pos == lengths[b]
        if len(pieces) == 1:
            assert pieces[0][2] == -1
        else:
            parts = [p[2] for p in pieces]
            assert parts == list(range(parts[0], parts[0] + len(parts))) and parts[0] >= 0
            assert not (set(parts) & seen_parts)
            seen_parts |= set(parts)
            assert all(n > 0 for _, n, _ in pieces)
    assert seen_parts == set(range(len(seen_parts)))  # the workspace has no holes


CASES = [
    # lengths recipe, H, d_a, d_u, Nq, dtype: one per kernel family and scheduling regime
    ("uniform200", 2, 64, 8, 1, F32),        # streaming, many short items
    ("few_long", 2, 64, 8, 2, BF16),         # streaming, split histories
    ("cfg3", 4, 64, 4, 64, BF16),            # direct-to-LDS, static lists, 4 workgroups per CU
    ("cfg4", 8, 128, 8, 128, BF16),          # direct-to-LDS, two long ragged histories per workgroup
    ("cfg4", 8, 128, 8, 300, BF16),          # several query blocks
    ("few_long", 2, 128, 8, 128, BF16),      # direct-to-LDS, fewer units than workgroups: cuts
    ("few_long", 2, 128, 24, 100, BF16),     # register-staged matrix-core kernel (wide d_u)
    ("with_empty", 3, 64, 2, 16, BF16),
]


def make_lengths(kind, rng):
    if kind == "uniform200":
        return np.full(1024, 200)
    if kind == "few_long":
        return np.array([5000, 70, 2300, 0, 1025, 40000])
    if kind == "cfg3":
        return np.full(512, 1024)
    if kind == "cfg4":
        return rng.integers(2048, 8193, size=128)
    if kind == "with_empty":
        return np.array([0, 0, 31, 32, 33, 0, 700, 1])
    raise KeyError(kind)


@pytest.mark.parametrize("kind,H,d_a,d_u,Nq,dtype", CASES)
@pytest.mark.parametrize("wg_per_cu", [1, 2, 4])
def test_every_position_is_covered_exactly_once(kind, H, d_a, d_u, Nq, dtype, wg_per_cu):
    rng = np.random.default_rng(len(kind) + H + wg_per_cu)
    lengths, rec, nwg, name = plan(make_lengths(kind, rng), H, d_a, d_u, Nq, dtype, wg_per_cu=wg_per_cu)
    check_cover(lengths, rec, H, Nq, name)
    if name.startswith("mfma_dma"):
        wg = rec[:, 7]
        assert (np.diff(wg) >= 0).all() and wg.max() < nwg == 256 * wg_per_cu
        # a workgroup (XCD = index mod 8) keeps to one head class
        ncls = 8 if H % 8 == 0 else (H if 8 % H == 0 else 1)
        assert ((wg % 8) % ncls == rec[:, 1] % ncls).all()


def test_static_lists_are_balanced_by_speed():
    """Long ragged histories, two workgroups per CU: the first dispatch wave (indices below half) is given
    more positions, in the ratio of the speeds the lists assume, and within each half loads are even."""
    rng = np.random.default_rng(4)
    lengths, rec, nwg, name = plan(rng.integers(2048, 8193, size=128), 8, 128, 8, 128, BF16, wg_per_cu=2)
    assert name.startswith("mfma_dma") and nwg == 512
    load = np.bincount(rec[:, 7], weights=rec[:, 3], minlength=nwg)
    fast, slow = load[:256], load[256:]
    assert 0.70 < slow.mean() / fast.mean() < 0.82
    assert fast.std() / fast.mean() < 0.05 and slow.std() / slow.mean() < 0.06
    # one wavefront per SIMD (a single workgroup of four wavefronts per CU): no weighting
    lengths, rec, nwg, name = plan(rng.integers(2048, 8193, size=128), 8, 128, 8, 128, BF16, wg_per_cu=1)
    load = np.bincount(rec[:, 7], weights=rec[:, 3], minlength=nwg)
    assert load.std() / load.mean() < 0.05


def test_sharing_one_side_keeps_the_kernel_family():
    lengths = np.full(64, 512)
    for share in (0, 1, 2):
        _, rec, _, name = plan(lengths, 2, 64, 4, 64, BF16, share=share)
        assert name.startswith("mfma_dma_bf16_d64_w1_g2")
        check_cover(lengths.astype(np.int32), rec, 2, 64, name)


def test_plan_rejects_bad_arguments():
    sh = ckv.make_shape(2, 1, 8, 0, 4, 1, 0, 0, 1.0, 8)
    with pytest.raises(ckv.CkvError) as e:
        ckv.ckv_plan(sh, np.array([1, -1], np.int32))
    assert e.value.code == ckv.CKV_ERR_LENGTH
    with pytest.raises(ckv.CkvError) as e:
        ckv.ckv_plan(sh, np.array([1, 1], np.int32), cus=0)
    assert e.value.code == ckv.CKV_ERR_SHAPE


@pytest.mark.parametrize("d_a,d_u,Nq,dtype,expect", [
    # direct-to-LDS kernel: wavefronts and query groups by width and query count
    (64, 4, 16, BF16, "mfma_dma_bf16_d64_w1_q16"), (64, 4, 17, BF16, "mfma_dma_bf16_d64_w1_g1"), (64, 4, 64, BF16, "mfma_dma_bf16_d64_w1_g2"),
    (64, 4, 100, BF16, "mfma_dma_bf16_d64_w4_g1"), (64, 64, 64, BF16, "mfma_dma_bf16_d64_w2_g1"),  # ordinary cache: two wavefronts
    (128, 8, 32, BF16, "mfma_dma_bf16_d128_w1_g1"), (128, 8, 64, BF16, "mfma_dma_bf16_d128_w2_g1"),
    (128, 8, 128, BF16, "mfma_dma_bf16_d128_w4_g1"), (256, 4, 16, BF16, "mfma_dma_bf16_d256_w4_g1"),
    (256, 10, 128, BF16, "mfma_dma_bf16_d256_w4_g1"), (256, 32, 64, BF16, "mfma_dma_bf16_d256_w4_g1"),
    # user widths it takes: odd up to 7, even up to 16 (one query group per wavefront from 10 on)
    (64, 7, 64, BF16, "mfma_dma_bf16_d64_w2_g1"), (64, 10, 64, BF16, "mfma_dma_bf16_d64_w2_g1"), (128, 16, 20, BF16, "mfma_dma_bf16_d128_w1_g1"),
    (128, 5, 128, BF16, "mfma_dma_bf16_d128_w4_g1"), (64, 1, 3, BF16, "mfma_dma_bf16_d64_w1_g1"),
    # what stays in the register-staged kernel (from 8 queries on), and below that in the streaming kernel
    (128, 9, 64, BF16, "mfma_bf16_d128"), (128, 24, 64, BF16, "mfma_bf16_d128"), (64, 18, 8, BF16, "mfma_bf16_d64"),
    (96, 8, 64, BF16, "mfma_bf16_d128"), (200, 8, 64, BF16, "mfma_bf16_d256"), (256, 34, 64, BF16, "mfma_bf16_d256"),
    (128, 9, 7, BF16, "streamw_bf16_g16_q2"), (64, 8, 2, BF16, "stream_bf16_v8_c1_g8"), (320, 8, 64, BF16, "streamw_bf16_g64_q2"),
    # fp32 storage
    (64, 8, 6, F32, "mfma_f32_d64"), (128, 8, 5, F32, "streamw_f32_g32_q2"), (256, 8, 64, F32, "mfma_f32_d256"),
    # target attention (one query): rows that fit one block of 16-byte lanes stay in the column-block streaming kernel,
    # wider rows and user slices that break the alignment go to the wide-row one (Table 1's widths: d_u of 256 columns)
    (64, 8, 1, BF16, "stream_bf16_v8_c1_g8"), (128, 8, 1, BF16, "stream_bf16_v8_c1"), (64, 8, 1, F32, "stream_f32_v4_c1"),
    (256, 4, 1, BF16, "streamw_bf16_g32_q1"), (256, 10, 1, BF16, "streamw_bf16_g32_q1"), (256, 1, 1, BF16, "streamw_bf16_g32_q1"),
    (256, 3, 2, BF16, "streamw_bf16_g32_q2"), (64, 3, 1, BF16, "streamw_bf16_g8_q1"), (64, 12, 1, BF16, "stream_bf16_v4_c1"),
    (64, 10, 1, BF16, "streamw_bf16_g16_q1"), (256, 8, 1, F32, "stream_f32_v4_c4"), (256, 8, 2, F32, "streamw_f32_g64_q2"),
    (256, 6, 1, F32, "streamw_f32_g64_q1"), (128, 2, 1, F32, "streamw_f32_g32_q1"), (1024, 8, 1, BF16, "stream_bf16_v8_c8"),
])
def test_kernel_choice_by_shape(d_a, d_u, Nq, dtype, expect):
    """Which kernel the dispatcher picks, and that its work lists cover the batch (host arithmetic only)."""
    lengths, rec, _, name = plan(np.array([700, 33, 0, 2048, 5]), 2, d_a, d_u, Nq, dtype)
    assert name.startswith(expect), name
    check_cover(lengths, rec, 2, Nq, name)
