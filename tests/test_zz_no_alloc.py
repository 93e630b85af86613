"""GPU test of ckv_attend_static_scratch, the attention entry point that allocates nothing: its split workspace is
a fixed array inside the library instead of a buffer owned by the handle.  Same kernels as ckv_attend, so outputs
must agree bit for bit, and both must agree with the oracle; two calls in a row, the second on a smaller input,
share the one array."""
import sys

import numpy as np
import pytest

from paper_2601_19178_amd import workloads as wl
from tests.parity import check_against_oracle

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make(lengths, dtype, mode, d_a, d_u, H, P, Nq, seed=31):
    lengths = np.asarray(lengths, dtype=np.int32)
    return wl.make(B=len(lengths), L=None, H=H, d_a=d_a, d_u=d_u, P=P, idx="uniform", Nq=Nq, mode=mode, dtype=dtype,
                   sigma_pool=d_a ** -0.5, seed=seed, lengths=lengths)


def split_workspace_bytes(ckv, s, w):
    """Bytes of split workspace the handle's kernels use, from the plan of the same shape (host arithmetic)."""
    import re
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    variant = ckv.ckv_variant(s.cache)
    m = re.search(r"_w(\d)_g(\d)", variant)
    qb = 16 if "_q16_" in variant else 32 * int(m.group(1)) * int(m.group(2)) if variant.startswith("mfma_dma") else (
        32 * int(re.search(r"_w(\d)", variant).group(1)) if variant.startswith("mfma_bf16") else (128 if variant.startswith("mfma_f32") else w["Nq"]))
    least = None
    for wg in (1, 2, 3, 4, 8):   # the resident workgroups per compute unit are the kernel's; take the smallest plan
        rec, _, _ = ckv.ckv_plan(s.shape, w["lengths"], cus, wg)
        parts = int((rec[:, 5] >= 0).sum())
        least = parts if least is None else min(least, parts)
    return least * qb * (w["d_g"] + w["d_u"] + 2) * 4


@pytest.mark.parametrize("kind", ["dma", "dma16", "staged", "fp32", "stream", "streamw"])
def test_static_scratch_entry_point_matches_ckv_attend(kind):
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2601_19178_amd import ckv, session
    if kind == "dma":       # direct-to-LDS matrix-core kernel: long histories among short ones are cut and merged
        first = make((5000, 70, 2300, 1024, 1025), wl.BF16, wl.SOFTMAX, d_a=128, d_u=8, H=2, P=5000, Nq=128)
        second = make((3000, 31), wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=4, H=1, P=700, Nq=64)
    elif kind == "dma16":   # the same kernel's organisation with sixteen queries per work item (pieces of sixteen query rows)
        first = make((9000, 70, 2300, 1025), wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=2, P=5000, Nq=16)
        second = make((3000, 31), wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=2, H=1, P=700, Nq=5)
    elif kind == "staged":  # register-staged matrix-core kernel
        first = make((5000, 70, 2300), wl.BF16, wl.SOFTMAX, d_a=128, d_u=24, H=2, P=5000, Nq=64)
        second = make((2000, 1), wl.BF16, wl.SOFTMAX, d_a=64, d_u=24, H=1, P=300, Nq=16)
    elif kind == "fp32":    # fp32 matrix-core kernel
        first = make((5000, 70, 2300), wl.F32, wl.SOFTMAX, d_a=128, d_u=8, H=2, P=5000, Nq=64)
        second = make((1500,), wl.F32, wl.SILU_OVER_N, d_a=64, d_u=4, H=1, P=300, Nq=8)
    elif kind == "streamw":  # wide-row streaming kernel (user widths that break the alignment of the final row)
        first = make((5000, 70, 2300), wl.BF16, wl.SOFTMAX, d_a=256, d_u=10, H=2, P=500, Nq=2)
        second = make((3000, 5), wl.F32, wl.SILU_OVER_N, d_a=128, d_u=3, H=1, P=500, Nq=1)
    else:                   # streaming kernel
        first = make((5000, 70, 2300), wl.F32, wl.SOFTMAX, d_a=64, d_u=8, H=2, P=500, Nq=2)
        second = make((3000, 5), wl.BF16, wl.SILU_OVER_N, d_a=64, d_u=8, H=1, P=500, Nq=1)
    for which, w in (("first", first), ("second (smaller)", second)):
        say(f"[case] static scratch, {kind}, {which} call: B={w['B']} H={w['H']} d_a={w['d_g'] + w['d_u']} Nq={w['Nq']} "
            f"dtype={w['dtype']} mode={w['mode']} lengths={w['lengths'].tolist()}")
        with session.Session(w) as s:
            say(f"  variant {ckv.ckv_variant(s.cache)}, split workspace {split_workspace_bytes(ckv, s, w)} bytes")
            assert split_workspace_bytes(ckv, s, w) > 0, "the case must exercise the scratch"
            s.attend()
            want = s.output().copy()
            s.out.fill_(float("nan"))
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info()[0]
            s.attend(static_scratch=True)
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the amount of free device memory"
            got = s.output().copy()
            np.testing.assert_array_equal(got, want)
            norm = check_against_oracle(got, w, what=f"static scratch {kind} {which}")
            # and once more on the same handle: the array keeps the last call's contents, results must not depend on them
            s.out.fill_(float("nan"))
            s.attend(static_scratch=True)
            np.testing.assert_array_equal(s.output(), want)
        say(f"  ok, bit-identical to ckv_attend, norm-wise error against the oracle {norm:.3e}")


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2601_19178_amd import ckv, session
    # one history of 150001 positions and 384 queries: hundreds of pieces, more partial outputs than the array holds
    w = make((150001,), wl.BF16, wl.SOFTMAX, d_a=128, d_u=8, H=2, P=20000, Nq=384)
    with session.Session(w) as s:
        need = split_workspace_bytes(ckv, s, w)
        say(f"[case] static scratch refusal: variant {ckv.ckv_variant(s.cache)}, split workspace {need} bytes")
        assert need > ckv.CKV_STATIC_SCRATCH_BYTES
        with pytest.raises(ckv.CkvError) as e:
            s.attend(static_scratch=True)
        assert e.value.code == ckv.CKV_ERR_UNSUPPORTED and "static scratch" in str(e.value)
        s.attend()      # the ordinary entry point still serves the handle
        # (a sample of the queries, one from every block of 16: the oracle works through 150001 positions per query on two threads)
        check_against_oracle(s.output(), w, what="after the refused call", queries=np.arange(5, 384, 16))
    # a handle without split histories uses no scratch at all and is served
    w = make((100, 33, 0), wl.BF16, wl.SOFTMAX, d_a=64, d_u=8, H=1, P=50, Nq=16)
    with session.Session(w) as s:
        s.attend(static_scratch=True)
        check_against_oracle(s.output(), w, what="static scratch, nothing split")
