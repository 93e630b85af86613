"""CPU checks of the direct-to-LDS attention kernel's memory accesses through the host model in tests/dma_model.py:
every instantiation the library ships, over the shapes that select it, must keep every global access inside its buffer,
every LDS access inside its area, at most 63 loads outstanding with every wait covering what is read next, and must
assemble exactly the final rows [pool | user] in LDS.  Planted mistakes show that the model notices each kind."""
import numpy as np
import pytest

from tests import dma_model as dm

# (d_a, wavefronts, query groups) of the instantiations with even user slices of up to 8 columns (16 at 256)
SHAPES = [(64, 1, 1), (64, 1, 2), (64, 2, 1), (64, 2, 2), (64, 4, 1), (128, 1, 1), (128, 1, 2), (128, 2, 1), (128, 2, 2),
          (128, 4, 1), (256, 4, 1)]
# (d_a, wavefronts) of the one-query-group instantiations that exist for odd and for wide user slices
NARROW = [(64, 1), (64, 2), (64, 4), (128, 1), (128, 2), (128, 4)]


def buffers_for(rng, DA, d_u, share, H, P, pool_ld, T, B, Nq, parts=0, QB=32):
    d_g = DA - d_u
    ksh, vsh = d_g > 0 and share in (0, 1), d_g > 0 and share in (0, 2)
    d_uk, d_uv = (d_u if ksh else DA), (d_u if vsh else DA)

    def user(cols):
        nbytes = (H * T * cols * 2 + 15) // 16 * 16          # the library rounds its allocations up to 16 bytes
        a = rng.integers(0, 65536, size=nbytes // 2, dtype=np.uint16)
        return a if cols > 0 else None

    buf = dict(
        pool_k=rng.integers(0, 65536, size=(H, P, pool_ld), dtype=np.uint16) if d_g > 0 else None,
        pool_v=rng.integers(0, 65536, size=(H, P, pool_ld), dtype=np.uint16) if d_g > 0 else None,
        idx=rng.integers(0, P, size=(2, H, T), dtype=np.int32) if d_g > 0 else None,
        user_k=user(d_uk), user_v=user(d_uv),
        q=rng.integers(0, 65536, size=(B, H, Nq, DA), dtype=np.uint16),
        out=np.zeros((B, H, Nq, DA), dtype=np.uint16),
        partial=np.zeros((max(parts, 1), QB, DA + 2), dtype=np.float32) if parts else None)
    shape = dict(d_g=d_g, d_u=d_u, share_k=ksh, share_v=vsh, pool_ld=pool_ld, P=P, H=H, T=T, Nq=Nq)
    return shape, buf


def run_case(DA, NW, QG, d_u, share=0, lengths=(33, 1, 100), pool_ld=None, Nq=None, seed=0, split=False, d_a=None, scores_ahead=False,
             q16=False):
    """d_a: the head's own width when it is narrower than the kernel's rows (DA).  scores_ahead: the tile loop that takes the
    scores of a tile one iteration early.  q16: the organisation with sixteen queries per work item."""
    rng = np.random.default_rng(seed)
    d_a = DA if d_a is None else d_a
    d_g = d_a - d_u
    H, P, B = 2, 37, len(lengths)
    pool_ld = pool_ld if pool_ld is not None else ((d_g + 7) // 8 * 8 if d_g > 0 else 0)
    T = int(sum(lengths))
    QB = 16 if q16 else 32 * NW * QG
    Nq = Nq if Nq is not None else QB - 5            # the last wavefront has fewer than 32 query rows
    shape, buf = buffers_for(rng, d_a, d_u, share, H, P, pool_ld, T, B, Nq, parts=4 if split else 0, QB=QB)
    stats = None
    t0 = 0
    for b, n in enumerate(lengths):
        for h in range(H):
            if split and n > 64:                      # two pieces of a split history, the cut on a tile boundary
                pieces = [(0, 64, 0 + 2 * h), (64, n - 64, 1 + 2 * h)]
            else:
                pieces = [(0, n, -1)]
            for lo, nn, part in pieces:
                item = dict(b=b, h=h, q0=0, n=nn, t0=t0 + lo, part=part, QB=QB)
                stats = dm.run_item(DA, NW, QG, shape, item, buf, scores_ahead=scores_ahead, q16=q16)
        t0 += n
    if not split:       # every byte of every output row was written (the model marks what it writes), nothing beyond
        assert (buf["out"].view(np.uint8) == 1).all()
    return stats


@pytest.mark.parametrize("DA,NW,QG", SHAPES)
@pytest.mark.parametrize("d_u", [0, 2, 4, 8])
def test_even_slices_every_shipped_shape(DA, NW, QG, d_u):
    st = run_case(DA, NW, QG, d_u)
    assert st["UK"] == 0 and st["peak_outstanding"] <= 63
    run_case(DA, NW, QG, d_u, lengths=(31, 32, 257), seed=1, split=True)


@pytest.mark.parametrize("DA,NW,QG", SHAPES)
@pytest.mark.parametrize("share", [1, 2])
def test_one_side_shared_and_ordinary_cache(DA, NW, QG, share):
    run_case(DA, NW, QG, 4, share=share, lengths=(65, 3), seed=2)
    run_case(DA, NW, QG, DA, lengths=(65, 3), seed=3)            # d_g = 0: rows by position, no index buffer at all


@pytest.mark.parametrize("DA,NW", NARROW + [(256, 4)])
@pytest.mark.parametrize("d_u", [1, 3])
def test_odd_slices_of_one_and_three_columns(DA, NW, d_u):
    st = run_case(DA, NW, 1, d_u, lengths=(33, 1, 100, 7), seed=4)     # T is odd: slices of the second head start on odd elements
    assert st["UK"] == 1
    run_case(DA, NW, 1, d_u, share=1, lengths=(33, 2), seed=5)
    run_case(DA, NW, 1, d_u, share=2, lengths=(33, 2), seed=6, split=False)


@pytest.mark.parametrize("DA,NW", NARROW)
@pytest.mark.parametrize("d_u,kind", [(10, 2), (12, 2), (16, 2), (5, 3), (7, 3)])
def test_wide_and_odd_wide_slices(DA, NW, d_u, kind):
    st = run_case(DA, NW, 1, d_u, lengths=(33, 1, 101), seed=7)
    assert st["UK"] == kind
    run_case(DA, NW, 1, d_u, share=2, lengths=(64, 31), seed=8, split=True)


@pytest.mark.parametrize("d_u", [5, 7, 10, 16, 24, 32])
def test_256_columns_take_slices_of_up_to_32_columns(d_u):
    st = run_case(256, 4, 1, d_u, lengths=(33, 100), seed=9)
    assert st["peak_outstanding"] <= 63 and st["lds_bytes"] <= 163840


@pytest.mark.parametrize("DA,NW,QG", [(64, 1, 1), (128, 4, 1), (256, 4, 1)])
def test_unpadded_and_overpadded_pool_rows(DA, NW, QG):
    run_case(DA, NW, QG, 8, pool_ld=DA - 8, seed=10)             # pool_ld == d_g: the padding chunk does not exist in memory
    run_case(DA, NW, QG, 8, pool_ld=DA + 8, seed=11)
    run_case(DA, NW, QG, 4, pool_ld=DA, Nq=3, seed=12)           # three queries: most staging rows are zeros


@pytest.mark.parametrize("DA", [128, 256])
@pytest.mark.parametrize("d_u", [0, 2, 4, 8])
def test_tile_loop_with_the_scores_one_tile_ahead(DA, d_u):
    """The loop of the four-wavefront 128- and 256-column instances that publishes a tile one iteration earlier (K operands of
    tile t + 1 are read in the iteration that finishes tile t): histories of one tile, of a few, ragged ends, split pieces,
    one side shared, ordinary cache, unpadded pool rows."""
    st = run_case(DA, 4, 1, d_u, lengths=(33, 1, 100, 32, 64, 65, 0, 257), seed=20, scores_ahead=True)
    ni = 32 // (64 // (DA // 8)) // 4
    assert st["UK"] == 0 and st["peak_outstanding"] <= 2 * (2 * ni + 1 + 1)     # two iterations of loads at most
    run_case(DA, 4, 1, d_u, lengths=(31, 32, 257), seed=21, split=True, scores_ahead=True)
    if d_u == 4:
        run_case(DA, 4, 1, 4, share=1, lengths=(65, 3), seed=22, scores_ahead=True)
        run_case(DA, 4, 1, 4, share=2, lengths=(65, 3), seed=23, scores_ahead=True)
        run_case(DA, 4, 1, DA, lengths=(65, 3), seed=24, scores_ahead=True)
        run_case(DA, 4, 1, 8, pool_ld=DA - 8, seed=25, scores_ahead=True)
        run_case(DA, 4, 1, 4, pool_ld=DA, Nq=3, seed=26, scores_ahead=True)
    if DA == 256:
        for wide in (10, 16, 24, 32):          # slices of up to 32 columns: up to four slice loads per wavefront and tile
            st = run_case(256, 4, 1, wide, lengths=(33, 100, 257), seed=27, scores_ahead=True)
            assert st["peak_outstanding"] <= 2 * (2 * ni + 1 + 4)
    with pytest.raises(dm.ModelError, match="no tile loop with the scores ahead"):
        run_case(128, 2, 1, d_u, scores_ahead=True)


@pytest.mark.parametrize("d_u", [0, 2, 4, 6, 8])
def test_sixteen_queries_per_work_item(d_u):
    """The 64-column one-wavefront instance on the 16x16x32 matrix instruction: the same ring, other operand addresses (every
    K operand must be its position's columns, every transposed V read its four positions by sixteen columns) and an epilogue
    of sixteen rows; ragged ends, split pieces, one side shared, ordinary cache, unpadded pool rows, 1 to 16 queries."""
    st = run_case(64, 1, 1, d_u, lengths=(33, 1, 100, 32, 64, 65, 0, 257), seed=30, q16=True)
    assert st["UK"] == 0 and st["NS"] == 2
    run_case(64, 1, 1, d_u, lengths=(31, 32, 257), seed=31, split=True, q16=True, Nq=16)
    for Nq in (1, 7, 16):
        run_case(64, 1, 1, d_u, lengths=(40,), seed=32 + Nq, q16=True, Nq=Nq)
    if d_u == 4:
        run_case(64, 1, 1, 4, share=1, lengths=(65, 3), seed=33, q16=True)
        run_case(64, 1, 1, 4, share=2, lengths=(65, 3), seed=34, q16=True, split=True)
        run_case(64, 1, 1, 64, lengths=(65, 3), seed=35, q16=True)
        run_case(64, 1, 1, 8, pool_ld=56, seed=36, q16=True)
        run_case(64, 1, 1, 4, pool_ld=72, Nq=3, seed=37, q16=True)
    with pytest.raises(dm.ModelError, match="no sixteen-query organisation"):
        run_case(64, 2, 1, d_u, q16=True)
    with pytest.raises(dm.ModelError, match="no sixteen-query organisation"):
        run_case(128, 1, 1, d_u, q16=True)


def test_model_notices_a_wrong_operand_row_of_the_sixteen_query_organisation(monkeypatch):
    # a swizzle that differs from the one the gathers wrote with: operands come from another chunk of the row
    real = dm.fk
    calls = {"n": 0}

    def other(DA, p):
        calls["n"] += 1
        return real(DA, p) ^ (1 if calls["n"] % 7 == 0 else 0)
    monkeypatch.setattr(dm, "fk", other)
    with pytest.raises(dm.ModelError, match="differ from the final rows|not its position's columns"):
        run_case(64, 1, 1, 4, lengths=(40,), q16=True)


def test_outstanding_loads_of_every_geometry_fit_the_wait_counter():
    """(NS - 1) iterations of loads are in flight at most: 2 NI gathers, one index load and the slice loads each."""
    for DA, NW, QG in SHAPES:
        for wide in (False, True):
            if wide and DA == 256:
                continue
            g = dm.Geo(DA, NW, wide)
            assert g.max_outstanding <= 63, (DA, NW, wide, g.max_outstanding)
    # the two-wavefront 256-column instance that was dropped: 3 x (16 + 1 + NUI) loads in flight, at the counter's limit
    # already with four slice loads and beyond it with the eight that slices of 32 columns would take
    g = dm.Geo(256, 2, False)
    assert 3 * (2 * g.NI + 1 + 4) == 63 and g.max_outstanding > 63


# ---------------------------------------------------------------------------------------------
# planted mistakes: each must be noticed
def test_model_notices_a_pool_that_is_too_short(monkeypatch):
    real = dm.Memory.__init__

    def short(self, name, data, readable=None):
        real(self, name, data, readable)
        if name.startswith("pool_k"):
            self.readable -= 16                       # as if the last row's last chunk were not mapped
    monkeypatch.setattr(dm.Memory, "__init__", short)
    with pytest.raises(dm.ModelError, match="outside pool_k"):
        rng = np.random.default_rng(0)
        shape, buf = buffers_for(rng, 64, 4, 0, 1, 4, 64, 40, 1, 16)    # d_g = 60: the last chunk of a row holds pool columns
        buf["idx"][:] = 3                             # every position gathers the last row
        dm.run_item(64, 1, 1, shape, dict(b=0, h=0, q0=0, n=40, t0=0, part=-1, QB=32), buf)


def test_model_notices_user_columns_that_are_not_appended(monkeypatch):
    real = dm.dma_nui
    monkeypatch.setattr(dm, "dma_nui", lambda d_a, nw, d_u: max(real(d_a, nw, d_u) // 2, 0))   # one slice load too few
    with pytest.raises(dm.ModelError, match="differ from the final rows"):
        run_case(128, 1, 1, 8)


def test_model_notices_a_wait_that_is_too_lax(monkeypatch):
    real = dm.Wave.wait
    monkeypatch.setattr(dm.Wave, "wait", lambda self, n: real(self, n + 3 if n > 0 else n))
    with pytest.raises(dm.ModelError, match="landed|in flight"):
        run_case(128, 4, 1, 8)


def test_model_notices_a_lax_wait_in_the_loop_with_the_scores_ahead(monkeypatch):
    # the wait of the other loop (two iterations of loads may stay outstanding) would publish a tile whose gathers are in flight
    real = dm.Wave.wait
    monkeypatch.setattr(dm.Wave, "wait", lambda self, n: real(self, 2 * n))
    with pytest.raises(dm.ModelError, match="landed|in flight"):
        run_case(128, 4, 1, 8, lengths=(200,), scores_ahead=True)


def test_model_notices_too_many_loads_in_flight():
    # slices of 32 columns on two wavefronts of 256 columns: eight slice loads per tile, 75 loads outstanding
    with pytest.raises(dm.ModelError, match="outstanding|fit|nui"):
        run_case(256, 2, 1, 32, lengths=(200,))


def test_model_notices_an_index_past_the_pool():
    rng = np.random.default_rng(0)
    shape, buf = buffers_for(rng, 128, 8, 0, 2, 16, 128, 70, 1, 128)
    buf["idx"][1, 1, 50] = 16                         # what ckv_build_cache refuses
    with pytest.raises(dm.ModelError, match="outside pool_v"):
        dm.run_item(128, 4, 1, shape, dict(b=0, h=1, q0=0, n=70, t0=0, part=-1, QB=128), buf)
