"""Host model of the memory accesses of the direct-to-LDS attention kernel (csrc/ckv_dma.hip).

The kernel assembles the final K and V rows of a tile in LDS with asynchronous global -> LDS loads whose
addresses are computed per lane; a wrong address there is a GPU memory fault, and a wrong wait count is a
silent race.  This module restates, per geometry (row width DA, wavefronts NW, query groups QG, kind of user
slice UK), the address arithmetic of every access the kernel issues for one work item, and carries it out on
numpy arrays standing for global memory and LDS, lanes vectorised:

  * every global read lies inside the buffer it belongs to (pool of the item's head, index planes, user
    arrays with their allocation rounding, queries) and every global write inside out / the split workspace;
  * every LDS access lies inside the kernel's dynamic LDS size and inside the area it is meant for;
  * per wavefront the asynchronous loads are issued in the kernel's order, every s_waitcnt vmcnt(N) of the
    kernel is applied (loads retire in order), no more than 63 are ever outstanding, and whatever is read
    from LDS (index slots, slice staging, tile rows) has landed and is not overwritten before its last read;
  * the bytes a wavefront finds in a published stage are the final rows [pool | user] of the right
    positions, chunk c of row p at slot c ^ f(p): the gather, the concat and the swizzle, end to end.

It is test infrastructure: it shares no code with the library and exists to be run on the CPU before a new
geometry ever reaches the GPU.  The matrix arithmetic is not modelled (the GPU parity tests cover values).
"""
import numpy as np

TP = 32


class ModelError(AssertionError):
    pass


def need(cond, msg):
    if not cond:
        raise ModelError(msg)


class Geo:
    """Mirror of the kernel's Geo<DA, NW, WIDEU> (sizes in bytes)."""

    def __init__(self, DA, NW, wide_u):
        self.DA, self.NW = DA, NW
        self.NT = NW * 64
        self.NS = 2 if (DA <= 128 and NW == 1) else 4
        self.CH = DA // 8
        self.ROWB = DA * 2
        self.RPI = 64 // self.CH
        self.NI = TP // self.RPI // NW
        self.NUI_MAX = (16 if DA == 256 else (8 if wide_u else 4)) // NW
        self.KV = TP * self.ROWB
        self.USER = NW * 64 * 4 * self.NUI_MAX
        self.STAGE = 2 * self.KV + self.USER
        self.IDX = 256
        self.NIS = 4
        self.LDS = self.NS * self.STAGE + NW * self.NIS * self.IDX
        need(self.NI >= 1, "tile too small for this many wavefronts")
        need(self.LDS <= 163840, f"LDS of one compute unit exceeded: {self.LDS}")
        self.max_outstanding = (self.NS - 1) * (2 * self.NI + 1 + self.NUI_MAX)


def fk(DA, p):
    return (p & 15) if DA >= 128 else ((p >> 1) & 7)


def fv(DA, p):
    return ((p & 3) << 2) if DA >= 128 else (((p >> 1) & 1) << 2)


def dma_nui(d_a, nw, d_u):
    """Mirror of ckv_dma_nui: slice load instructions per wavefront and tile, or -1."""
    if d_a not in (64, 128, 256) or nw not in (1, 2, 4):
        return -1
    if d_a == 256 and nw != 4:
        return -1
    if d_u < 0 or d_u > (32 if d_a == 256 else 16) or ((d_u & 1) and d_u > 7):
        return -1
    n = ((64 if d_u & 1 else 32) * d_u + nw * 64 - 1) // (nw * 64)
    return n if n <= 1 else (2 if n <= 2 else (4 if n <= 4 else 8))


def slice_kind(d_a, d_u, d_g):
    """Mirror of the launcher's choice of UK."""
    wide = d_a != 256 and ((d_u > 3) if (d_u & 1) else (d_u > 8))
    if (d_u & 1) and wide:
        return 3
    if d_u & 1:
        return 1
    if d_g > 0 and wide:
        return 2
    return 0


class Memory:
    """A named byte buffer with bounds-checked, lane-vectorised reads and writes."""

    def __init__(self, name, data, readable=None):
        self.name = name
        self.data = np.ascontiguousarray(data).view(np.uint8).reshape(-1)
        self.readable = len(self.data) if readable is None else readable

    def read(self, off, nbytes, what):
        off = np.asarray(off, dtype=np.int64)
        need(off.min() >= 0 and off.max() + nbytes <= self.readable,
             f"{what}: read of {nbytes} bytes at offset {int(off.min())}..{int(off.max())} outside {self.name} ({self.readable} bytes)")
        return self.data[off[:, None] + np.arange(nbytes)]

    def write(self, off, values, what):
        off = np.asarray(off, dtype=np.int64)
        nbytes = values.shape[1]
        need(off.min() >= 0 and off.max() + nbytes <= len(self.data),
             f"{what}: write of {nbytes} bytes at offset {int(off.min())}..{int(off.max())} outside {self.name} ({len(self.data)} bytes)")
        self.data[off[:, None] + np.arange(nbytes)] = values


class Wave:
    """Asynchronous loads of one wavefront: issued in order, retired in order by wait(N)."""

    def __init__(self, lds, limit=63):
        self.lds, self.limit = lds, limit
        self.pending = []          # (lds offsets per lane, bytes per lane, tag)
        self.peak = 0

    def issue(self, lds_off, values, tag):
        self.pending.append((np.asarray(lds_off, dtype=np.int64), values, tag))
        self.peak = max(self.peak, len(self.pending))
        need(len(self.pending) <= self.limit, f"{len(self.pending)} loads outstanding, the wait counter holds {self.limit} ({tag})")

    def wait(self, n):
        while len(self.pending) > n:
            off, values, tag = self.pending.pop(0)
            self.lds.write(off, values, f"landing of {tag}")

    def landed(self, tag_prefix):
        return not any(t.startswith(tag_prefix) for _, _, t in self.pending)


def scores_ahead_supported(DA, NW, QG, UK):
    """The instantiations whose tile loop exists with the scores one tile ahead."""
    return (DA == 128 and NW == 4 and QG == 1 and UK == 0) or (DA == 256 and UK == 0)


def q16_supported(DA, NW, QG, UK, d_u, d_g):
    """The instantiation with sixteen queries per work item on the 16x16x32 matrix instruction, and the slices it takes."""
    return DA == 64 and NW == 1 and QG == 1 and UK == 0 and (d_g == 0 or (d_u % 2 == 0 and d_u <= 8))


def run_item(DA, NW, QG, shape, item, buffers, check_rows=True, scores_ahead=False, q16=False):
    """One work item through the kernel's access pattern.
    q16: sixteen queries per work item (lane = query lane % 16, group of eight positions lane / 16): other operand
    addresses and another epilogue, the same ring.
    scores_ahead: the tile loop that takes the scores of tile t + 1 in the iteration that finishes tile t (tiles are
    published one iteration earlier, two tiles of gathers in flight instead of three).

    shape: dict(d_g, d_u, share_k, share_v (does the side gather from a pool), pool_ld, P, H, T, Nq)
    item:  dict(b, h, q0, n, t0, part (slot or -1), QB)
    buffers: dict of numpy arrays: pool_k, pool_v [H][P][pool_ld] u16, idx [2][H][T] i32, user_k, user_v (packed layout,
             allocation rounded up to 16 bytes), q, out [B][H][Nq][DA] u16, partial f32 or None
    Returns statistics (peak loads outstanding, LDS bytes).
    """
    d_g, d_u = shape["d_g"], shape["d_u"]
    da = d_g + d_u                        # row width in memory
    need(da == DA, "the kernel serves rows of exactly DA columns")
    chq = da >> 3
    ksh, vsh = shape["share_k"], shape["share_v"]
    UK = slice_kind(DA, d_u, d_g)
    need(not (UK != 0 and QG != 1), "odd and wide user slices exist with one query group per wavefront only")
    G = Geo(DA, NW, UK >= 2)
    nui = 0 if d_g == 0 else dma_nui(DA, NW, d_u)
    need(nui >= 0 and nui <= G.NUI_MAX, f"nui = {nui} does not fit NUI_MAX = {G.NUI_MAX}")
    need(nui in (0, 1) or (G.NUI_MAX >= 2 and nui == 2) or (G.NUI_MAX >= 4 and nui == 4) or (G.NUI_MAX >= 8 and nui == 8),
         "the kernel has no tile loop for this number of slice loads")
    H, T, P, pool_ld, Nq = shape["H"], shape["T"], shape["P"], shape["pool_ld"], shape["Nq"]
    uodd = UK in (1, 3)
    n, h, t0 = item["n"], item["h"], item["t0"]
    hT = h * T + t0
    dgk, dgv = (d_g if ksh else da), (d_g if vsh else da)
    duk, duv = da - dgk, da - dgv

    lds = Memory("LDS", np.zeros(G.LDS, np.uint8))
    g_idx = Memory("idx", buffers["idx"]) if buffers.get("idx") is not None else None
    g_items = Memory("items", np.zeros(64, np.uint8))
    g_uk = Memory("user_k", buffers["user_k"]) if buffers.get("user_k") is not None else None
    g_uv = Memory("user_v", buffers["user_v"]) if buffers.get("user_v") is not None else None
    g_q = Memory("q", buffers["q"])
    g_out = Memory("out", buffers["out"])
    # the rows a side gathers from: the pool of the item's head (a read that strays into another head's pool is an error
    # too), or (side not shared) the user array of the item's positions
    if ksh:
        g_pk, pk_base, krow_bytes = Memory("pool_k of the head", buffers["pool_k"].reshape(H, P, pool_ld)[h]), 0, pool_ld * 2
    else:
        g_pk, pk_base, krow_bytes = g_uk, hT * da * 2, da * 2
    if vsh:
        g_pv, pv_base, vrow_bytes = Memory("pool_v of the head", buffers["pool_v"].reshape(H, P, pool_ld)[h]), 0, pool_ld * 2
    else:
        g_pv, pv_base, vrow_bytes = g_uv, hT * da * 2, da * 2

    lane = np.arange(64)
    qn, hh = lane & 31, lane >> 5
    l16, g4 = lane & 15, lane >> 4
    need(not q16 or q16_supported(DA, NW, QG, UK, d_u, d_g), "this instantiation or slice width has no sixteen-query organisation")
    need(not (q16 and scores_ahead), "one tile loop at a time")
    waves = [Wave(lds) for _ in range(NW)]
    any_pool = ksh or vsh
    ilast = n - 1 if any_pool else 7
    idx_lds = [G.NS * G.STAGE + w * G.NIS * G.IDX for w in range(NW)]
    idx_slot_tile = [[None] * G.NIS for _ in range(NW)]     # which tile's indices a slot holds (issued)
    idx_last_read = [[-10 ** 9] * G.NIS for _ in range(NW)]  # program step of the last read of a slot
    looked_up = [-1] * NW                                    # last tile whose rows a wavefront has looked up
    step = [0]

    def issue_idx(w, tile):
        pos = np.minimum(tile * TP + qn, ilast)
        slot = tile & (G.NIS - 1)
        if any_pool:
            elem = np.where(hh == 1, H * T, 0) + hT + pos         # plane 1 (I_v) for the upper half
            vals = g_idx.read(elem * 4, 4, f"index load of tile {tile}")
        else:
            vals = g_items.read(pos * 4, 4, "placeholder index load")
        dst = idx_lds[w] + slot * G.IDX + 4 * lane
        need(dst.max() + 4 <= G.LDS and dst.min() >= G.NS * G.STAGE, "index slot outside its area")
        waves[w].issue(dst, vals, f"idx:{tile}")
        idx_slot_tile[w][slot] = tile

    QS = DA * 2 + 16
    need(NW * QG * 32 * QS <= G.NS * G.STAGE, "query staging does not fit under the stages")
    qfirst = [item["q0"] + w * QG * 32 for w in range(NW)]
    qrows = [min(max(Nq - qf, 0), 16 if q16 else QG * 32) for qf in qfirst]
    qbyte0 = [((item["b"] * H + h) * Nq + qf) * da * 2 for qf in qfirst]

    ntiles = (n + TP - 1) // TP
    if n > 0:
        for w in range(NW):
            for tile in (0, 1, 2):
                issue_idx(w, tile)

    # ---- queries: coalesced rows into the staging area, then every lane picks its operands
    for w in range(NW):
        qlds = w * QG * 32 * QS
        for i in range(QG * 32 * G.CH // 64):
            e = i * 64 + lane
            row, c = e // G.CH, e % G.CH
            vals = np.zeros((64, 16), np.uint8)
            ok = (row < qrows[w]) & (c < chq)
            if ok.any():
                vals[ok] = g_q.read(qbyte0[w] + row[ok] * da * 2 + c[ok] * 16, 16, "query rows")
            lds.write(qlds + row * QS + c * 16, vals, "query staging")
        for ks in (range(2) if q16 else ()):
            for j in range(4):
                ci = 32 * ks + 8 * g4 + 2 * j
                pc = np.where(ci < dgk, ci + duk, ci - dgk)
                got = lds.read(qlds + l16 * QS + pc * 2, 4, "query operand")
                if check_rows:
                    rows_ok = l16 < qrows[w]
                    want = g_q.data[(qbyte0[w] + l16 * da * 2 + pc * 2)[rows_ok, None] + np.arange(4)]
                    need(np.array_equal(got[rows_ok], want), "a query operand is not the query's own columns")
                    need(not got[~rows_ok].any(), "the operand of a query past the last is not zero")
        for g in (() if q16 else range(QG)):
            for kk in range(DA // 16):
                for j in range(4):
                    ci = 16 * kk + 8 * hh + 2 * j
                    pc = np.where(ci < dgk, ci + duk, np.where(ci < da, ci - dgk, ci))
                    got = lds.read(qlds + (g * 32 + qn) * QS + pc * 2, 2 if uodd else 4, "query operand")
                    pad = ci >= da
                    need(not got[pad].any(), "a padding column of the queries is not zero")
                    if check_rows and not uodd:                # the operand is the query's columns pc, pc + 1 as stored
                        rows_ok = (g * 32 + qn < qrows[w]) & ~pad
                        want = g_q.data[(qbyte0[w] + (g * 32 + qn) * da * 2 + pc * 2)[rows_ok, None] + np.arange(4)]
                        need(np.array_equal(got[rows_ok], want), "a query operand is not the query's own columns")
                    if uodd:
                        pc1 = np.where(ci + 1 < dgk, ci + 1 + duk, ci + 1 - dgk)
                        lds.read(qlds + (g * 32 + qn) * QS + pc1 * 2, 2, "query operand (second half)")
    # (lds_barrier: the staging area is free from here on)

    if ntiles > 0:
        per = []   # per-wave lane constants
        for w in range(NW):
            gslot = lane % G.CH
            gp, gko, gvo = [], [], []
            for i in range(G.NI):
                p = (i * NW + w) * G.RPI + lane // G.CH
                ck = gslot ^ fk(DA, p)
                cv = gslot ^ fv(DA, p)
                ck = np.where(ck * 8 >= dgk, 0, ck)
                cv = np.where(cv * 8 >= dgv, 0, cv)
                gp.append(p); gko.append(ck * 16); gvo.append(cv * 16)
            ROWS_W = TP // NW
            hd = (d_u if uodd else d_u >> 1) if d_u > 0 else 1
            up, uoff, uisv, uok, cdst = [], [], [], [], []
            for u in range(G.NUI_MAX):
                jj = u * 64 + lane
                ok = (u < nui) & (jj < 2 * ROWS_W * hd)
                jj = np.where(ok, jj, 0)
                sl = jj // hd
                off = jj - sl * hd
                isv = sl >= ROWS_W
                ok = ok & np.where(isv, vsh, ksh)
                o = np.where(isv, sl - ROWS_W, sl)
                p = ((o // G.RPI) * NW + w) * G.RPI + (o % G.RPI)
                col = d_g + (off if uodd else 2 * off)
                slot = (col >> 3) ^ np.where(isv, fv(DA, p), fk(DA, p))
                up.append(p); uoff.append(off); uisv.append(isv); uok.append(ok)
                cdst.append(np.where(isv, G.KV, 0) + p * G.ROWB + slot * 16 + (col & 7) * 2)
            per.append(dict(gp=gp, gko=gko, gvo=gvo, up=up, uoff=uoff, uisv=uisv, uok=uok, cdst=cdst, hd=hd))

        def gather_rows(w, tile):
            slot = tile & (G.NIS - 1)
            need(idx_slot_tile[w][slot] == tile, f"row lookup of tile {tile} finds the indices of tile {idx_slot_tile[w][slot]} in its slot")
            need(waves[w].landed(f"idx:{tile}"), f"row lookup of tile {tile} before its indices have landed")
            idx_last_read[w][slot] = step[0]
            looked_up[w] = max(looked_up[w], tile)
            rk, rv = [], []
            for i in range(G.NI):
                gp = per[w]["gp"][i]
                jk = lds.read(idx_lds[w] + slot * G.IDX + 4 * gp, 4, "index slot (K plane)").view(np.int32)[:, 0]
                jv = lds.read(idx_lds[w] + slot * G.IDX + 4 * (32 + gp), 4, "index slot (V plane)").view(np.int32)[:, 0]
                pos = np.minimum(tile * TP + gp, n - 1)
                rk.append(jk if ksh else pos)
                rv.append(jv if vsh else pos)
            return rk, rv

        stage_tile = [None] * G.NS            # which tile a stage holds / is being filled with
        stage_free_at = [-1] * G.NS           # program step from which a stage may be written again

        def tile_dma(w, tile, rk, rv):
            st = (tile & (G.NS - 1)) * G.STAGE
            s_i = tile & (G.NS - 1)
            need(step[0] >= stage_free_at[s_i], f"stage {s_i} is refilled for tile {tile} before its last reader passed the barrier")
            for i in range(G.NI):
                dst = st + (i * NW + w) * G.RPI * G.ROWB + 16 * lane
                need(dst.max() + 16 <= st + G.KV, "K gather leaves the K area of its stage")
                rows = rk[i].astype(np.int64) & 0xFFFFFFFF
                waves[w].issue(dst, g_pk.read(pk_base + rows * krow_bytes + per[w]["gko"][i], 16, f"K gather of tile {tile}"), f"k:{tile}")
                rows = rv[i].astype(np.int64) & 0xFFFFFFFF
                waves[w].issue(dst + G.KV, g_pv.read(pv_base + rows * vrow_bytes + per[w]["gvo"][i], 16, f"V gather of tile {tile}"), f"v:{tile}")
            for u in range(nui):
                c = per[w]
                pos = np.minimum(tile * TP + c["up"][u], n - 1)
                dst = st + 2 * G.KV + (w * G.NUI_MAX + u) * 256 + 4 * lane
                need(dst.max() + 4 <= st + G.STAGE, "slice staging leaves its stage")
                vals = np.zeros((64, 4), np.uint8)
                for isv, mem in ((False, g_uk), (True, g_uv)):
                    sel = c["uisv"][u] == isv
                    if not sel.any():
                        continue
                    need(mem is not None, "a slice load reads a user array that does not exist")
                    if uodd:
                        dword = ((hT + pos[sel]) * d_u + c["uoff"][u][sel]) >> 1
                    else:
                        dword = (hT * d_u >> 1) + pos[sel] * c["hd"] + c["uoff"][u][sel]
                        need((hT * d_u) % 2 == 0, "even slices start on dword boundaries")
                    vals[sel] = mem.read(dword * 4, 4, f"user slice of tile {tile}")
                waves[w].issue(dst, vals, f"u:{tile}")

        def concat(w, tile):
            st = (tile & (G.NS - 1)) * G.STAGE
            c = per[w]
            need(waves[w].landed(f"u:{tile}") and waves[w].landed(f"k:{tile}") and waves[w].landed(f"v:{tile}"),
                 f"concat of tile {tile} before the wavefront's loads of that tile have landed")
            for u in range(nui):
                ok = c["uok"][u]
                if not ok.any():
                    continue
                x = lds.read(st + 2 * G.KV + (w * G.NUI_MAX + u) * 256 + lane * 4, 4, "slice staging")
                dst = st + c["cdst"][u]
                need((dst[ok] + (2 if uodd else 4)).max() <= st + 2 * G.KV, "concat writes past the tile rows")
                if uodd:
                    pos = np.minimum(tile * TP + c["up"][u], n - 1)
                    upper = (((hT + pos) * d_u + c["uoff"][u]) & 1).astype(bool)
                    half = np.where(upper[:, None], x[:, 2:4], x[:, 0:2])
                    lds.write(dst[ok], half[ok], "concat")
                else:
                    lds.write(dst[ok], x[ok], "concat")

        def expected_rows(tile):
            """Final K and V rows of the tile's positions as the kernel lays them out: [pool | user] columns, u16."""
            pos = np.minimum(tile * TP + np.arange(TP), n - 1)
            rows = []
            for side, sh in ((0, ksh), (1, vsh)):
                user = buffers["user_k" if side == 0 else "user_v"]
                if sh:
                    pool = buffers["pool_k" if side == 0 else "pool_v"].reshape(H, P, pool_ld)
                    ix = buffers["idx"].reshape(2, H, T)[side, h, t0 + pos]
                    r = pool[h, ix, :d_g]
                    if d_u > 0:
                        uflat = user.view(np.uint16).reshape(-1)
                        start = (hT + pos) * d_u
                        r = np.concatenate([r, uflat[start[:, None] + np.arange(d_u)]], axis=1)
                else:
                    uflat = user.view(np.uint16).reshape(-1)
                    start = (hT + pos) * da
                    r = uflat[start[:, None] + np.arange(da)]
                rows.append(np.ascontiguousarray(r, dtype=np.uint16))
            return rows

        published = [-1]   # the last tile a barrier has published

        def compute(tile, sides=(0, 1)):
            """Operand reads of every wavefront on a published tile (K rows, V rows or both); contents of the stage against
            the definition."""
            st = (tile & (G.NS - 1)) * G.STAGE
            need(stage_tile[tile & (G.NS - 1)] == tile, f"tile {tile} is computed from a stage that holds tile {stage_tile[tile & (G.NS - 1)]}")
            need(tile <= published[0], f"tile {tile} is read before a barrier has published it")
            kx = fk(DA, qn)
            g16, s16 = lane >> 4, lane & 15
            vrow = G.KV + (4 * hh + (s16 >> 2)) * G.ROWB + (s16 & 1) * 8
            vc, vx = 2 * (g16 & 1) + ((s16 & 3) >> 1), fv(DA, s16 >> 2)
            if q16:
                # A operand of score block b: row m = lane % 16 is tile position 16 b + m, columns 32 ks + 8 (lane / 16) .. + 8;
                # the lane's four results of block b are then positions 16 b + 4 (lane / 16) + r.
                # A operand of the output blocks: a group of sixteen lanes fetches positions 16 hl + 4 (lane / 16) .. + 4 by
                # columns 16 dt .. + 16, four columns a lane, and the transposing read hands lane m column 16 dt + m.
                ek, ev = expected_rows(tile)
                for b in range(2):
                    pk_ = 16 * b + l16
                    for ks in range(2):
                        kaddr = st + pk_ * G.ROWB + (((4 * ks + g4) ^ fk(DA, pk_)) << 4)
                        for grp in range(4):        # sixteen lanes are served together: sixteen different 16-byte slots modulo 16
                            need(len(set(((kaddr[16 * grp:16 * grp + 16] >> 4) & 15).tolist())) == 16, "K operand reads of a lane group share LDS banks")
                        got = lds.read(kaddr, 16, "K operand").view(np.uint16)
                        if check_rows:
                            cols = 32 * ks + 8 * g4[:, None] + np.arange(8)
                            okp = pk_ < min(n - tile * TP, TP)
                            need(np.array_equal(got[okp], ek[pk_[:, None], cols][okp]), f"tile {tile}: a K operand is not its position's columns")
                for hl in range(2):
                    pv_ = 4 * g4 + (l16 >> 2) + 16 * hl
                    for dt in range(4):
                        col = 16 * dt + 4 * (l16 & 3)
                        ad = st + G.KV + pv_ * G.ROWB + (((col >> 3) ^ fv(DA, pv_)) << 4) + (col & 7) * 2
                        need(ad.min() >= st + G.KV and (ad + 8).max() <= st + 2 * G.KV, "V operand outside the V rows of its stage")
                        got = lds.read(ad, 8, "V operand").view(np.uint16)
                        if check_rows:
                            cols = col[:, None] + np.arange(4)
                            okp = pv_ < min(n - tile * TP, TP)
                            need(np.array_equal(got[okp], ev[pv_[:, None], cols][okp]), f"tile {tile}: a V operand is not its position's columns")
                            # within a group of sixteen lanes: four positions (lane / 4 within the group) by sixteen columns
                            need(np.array_equal(np.unique(pv_.reshape(4, 16), axis=1).shape, (4, 4)), "a transposed read does not cover four positions")
                sides = ()   # (the reads of the 32-query organisation below are not issued)
            if 0 in sides:
                for kk in range(DA // 16):
                    lds.read(st + qn * G.ROWB + (((2 * kk + hh) ^ kx) << 4), 16, "K operand")
            if 1 in sides:
                for ks in range(2):
                    for dt in range(DA // 32):
                        ad = st + vrow + 16 * ks * G.ROWB + (((4 * dt + vc) ^ vx) << 4)
                        need(ad.min() >= st + G.KV and (ad + 8 * G.ROWB + 8).max() <= st + 2 * G.KV, "V operand outside the V rows of its stage")
                        lds.read(ad, 8, "V operand")
                        lds.read(ad + 8 * G.ROWB, 8, "V operand")
            if check_rows:
                ek, ev = expected_rows(tile)
                nt = min(n - tile * TP, TP)       # rows past the end of the history hold a clamped copy: not checked
                pp, cc = np.meshgrid(np.arange(nt), np.arange(chq), indexing="ij")
                for side, exp, f in ((0, ek, fk), (1, ev, fv)):
                    if side not in sides:
                        continue
                    off = st + side * G.KV + pp * G.ROWB + ((cc ^ f(DA, pp)) << 4)
                    got = lds.data[off[..., None] + np.arange(16)].reshape(nt, chq, 16).view(np.uint16)
                    want = exp[:nt].reshape(nt, chq, 8)
                    if side == 0 and chq < G.CH:
                        # padding columns of a K row meet zero query columns: they must hold finite values, which a copy of
                        # the row's own first chunk is
                        pq, cq = np.meshgrid(np.arange(nt), np.arange(chq, G.CH), indexing="ij")
                        offp = st + pq * G.ROWB + ((cq ^ f(DA, pq)) << 4)
                        padv = lds.data[offp[..., None] + np.arange(16)].reshape(nt, G.CH - chq, 16).view(np.uint16)
                        need(np.array_equal(padv, np.broadcast_to(exp[:nt, None, 0:8], padv.shape)),
                             f"tile {tile}: padding columns of the K rows are not a copy of the rows' first chunk")
                    bad = np.argwhere((got != want).any(axis=2))
                    need(len(bad) == 0, f"tile {tile} {'KV'[side]}: {len(bad)} chunks differ from the final rows, first at row "
                                        f"{bad[0][0] if len(bad) else 0} chunk {bad[0][1] if len(bad) else 0}")

        # ---- the tile loop, every wavefront in the kernel's order; a barrier is a point all wavefronts reach
        kAhead = DA <= 128
        NS = G.NS
        need(not scores_ahead or scores_ahead_supported(DA, NW, QG, UK), "this instantiation has no tile loop with the scores ahead")
        for w in range(NW):
            waves[w].wait(0)                       # wait_vm<0>: the first indices
        rows = [gather_rows(w, 0) if (kAhead or scores_ahead) else None for w in range(NW)]   # (the loops with the scores ahead look rows up one iteration early at every width)
        for t in (range(-(NS - 1), ntiles) if scores_ahead else ()):
            # iteration t: this iteration's loads; K operands of tile t + 1 and V operands of tile t; the wait that lets only
            # this iteration's loads stay outstanding; concat and publication of tile t + 2
            for w in range(NW):
                step[0] += 1
                slot = (t + NS + 2) & (G.NIS - 1)
                former = t + NS + 2 - G.NIS
                need(former < 0 or former <= looked_up[w], f"indices of tile {former} are overwritten before their rows were looked up")
                need(idx_last_read[w][slot] < step[0], "an index slot is overwritten before its last reader")
                issue_idx(w, t + NS + 2)
                tile_dma(w, t + NS - 1, *rows[w])
            stage_tile[(t + NS - 1) & (NS - 1)] = t + NS - 1
            if -1 <= t < ntiles - 1:
                compute(t + 1, sides=(0,))
            if t >= 0:
                compute(t, sides=(1,))
            for w in range(NW):
                waves[w].wait((NS - 3) * (2 * G.NI + 1 + nui))
                if nui > 0 and 0 <= t + 2 < ntiles:
                    concat(w, t + 2)
                rows[w] = gather_rows(w, t + NS)
            if t + 2 < ntiles:
                for w in range(NW):
                    need(waves[w].landed(f"k:{t + 2}") and waves[w].landed(f"v:{t + 2}"),
                         f"tile {t + 2} is published while gathers of wavefront {w} are in flight")
            published[0] = t + 2
            stage_free_at[t & (NS - 1)] = step[0] + 1 if t >= 0 else stage_free_at[t & (NS - 1)]
        for t in (() if scores_ahead else range(-(NS - 1), ntiles)):
            for w in range(NW):
                step[0] += 1
                slot = (t + NS + 2) & (G.NIS - 1)
                # the slot's former content, the indices of tile t + NS + 2 - NIS, must have been looked up already
                former = t + NS + 2 - G.NIS
                need(former < 0 or former <= looked_up[w], f"indices of tile {former} are overwritten before their rows were looked up")
                need(idx_last_read[w][slot] < step[0], "an index slot is overwritten before its last reader")
                issue_idx(w, t + NS + 2)
                if not kAhead:
                    rows[w] = gather_rows(w, t + NS - 1)
                tile_dma(w, t + NS - 1, *rows[w])
            stage_tile[(t + NS - 1) & (NS - 1)] = t + NS - 1
            if t >= 0:
                compute(t)
            for w in range(NW):
                waves[w].wait((NS - 2) * (2 * G.NI + 1 + nui))
                if nui > 0 and 0 <= t + 1 < ntiles:
                    concat(w, t + 1)
                if kAhead:
                    rows[w] = gather_rows(w, t + NS)
            # lds_barrier: tile t + 1 is published, the stage of tile t is retired
            if t + 1 < ntiles:
                for w in range(NW):
                    need(waves[w].landed(f"k:{t + 1}") and waves[w].landed(f"v:{t + 1}"),
                         f"tile {t + 1} is published while gathers of wavefront {w} are in flight")
            published[0] = t + 1
            stage_free_at[t & (NS - 1)] = step[0] + 1 if t >= 0 else stage_free_at[t & (NS - 1)]
        for w in range(NW):
            waves[w].wait(0)

    # ---- epilogue
    for w in range(NW if q16 else 0):
        # lane: query lane % 16, columns 16 dt + 4 (lane / 16) + r of the kernel's order
        written = np.zeros((16, DA), bool)
        if item["part"] < 0:
            for dt in range(4):
                for r in range(0, 4, 2):
                    ci = 16 * dt + 4 * g4 + r
                    pc = np.where(ci < dgv, ci + duv, ci - dgv)
                    lds.write(l16 * QS + pc * 2, np.zeros((64, 4), np.uint8), "output staging")
                    written[l16, pc] = True
                    written[l16, pc + 1] = True
            need(written.all(), "the staged output rows have columns nobody wrote")
            for i in range(16 * G.CH // 64):
                e = i * 64 + lane
                row, c = e // G.CH, e % G.CH
                need(row.max() < 16, "copy-out past the sixteen staged rows")
                v = lds.read(row * QS + c * 16, 16, "output staging")
                ok = row < qrows[w]
                if ok.any():
                    g_out.write(qbyte0[w] + row[ok] * da * 2 + c[ok] * 16, v[ok] + 1, "output rows")
        else:
            need(buffers.get("partial") is not None, "a piece of a split history needs the workspace")
            g_ws = Memory("partial", buffers["partial"])
            QB = item["QB"]
            need(QB == 16, "sixteen queries per work item")
            ws0 = item["part"] * QB * (da + 2) * 4
            FS = DA * 4 + 16
            need(16 * FS <= G.NS * G.STAGE, "the staged accumulators must fit in the retired stages")
            for dt in range(4):
                for r in range(4):
                    ci = 16 * dt + 4 * g4 + r
                    pc = np.where(ci < dgv, ci + duv, ci - dgv)
                    lds.write(l16 * FS + pc * 4, np.zeros((64, 4), np.uint8), "accumulator staging")
                    written[l16, pc] = True
            need(written.all(), "the staged accumulators have columns nobody wrote")
            first = g4 == 0
            g_ws.write(ws0 + (QB * da + l16[first]) * 4, np.ones((16, 4), np.uint8), "piece maximum")
            g_ws.write(ws0 + (QB * da + QB + l16[first]) * 4, np.ones((16, 4), np.uint8), "piece sum")
            for i in range(16 * (DA // 4) // 64):
                e = i * 64 + lane
                row, c = e // (DA // 4), e % (DA // 4)
                v = lds.read(row * FS + c * 16, 16, "accumulator staging")
                g_ws.write(ws0 + (row * da + c * 4) * 4, v + 1, "piece accumulators")
    for w in range(0 if q16 else NW):
        if item["part"] < 0:
            qlds = w * QG * 32 * QS
            for g in range(QG):
                for dt in range(DA // 32):
                    for r in range(0, 16, 2):
                        ci = 32 * dt + 8 * (r >> 2) + 4 * hh + (r & 3)
                        pc = np.where(ci < dgv, ci + duv, np.where(ci < da, ci - dgv, ci))
                        need(((g * 32 + qn) * QS + pc * 2 + 4).max() <= NW * QG * 32 * QS, "output staging leaves its rows")
                        lds.write(qlds + (g * 32 + qn) * QS + pc * 2, np.zeros((64, 2 if uodd else 4), np.uint8), "output staging")
                        if uodd:
                            pc1 = np.where(ci + 1 < dgv, ci + 1 + duv, ci + 1 - dgv)
                            lds.write(qlds + (g * 32 + qn) * QS + pc1 * 2, np.zeros((64, 2), np.uint8), "output staging")
            for i in range(QG * 32 * G.CH // 64):
                e = i * 64 + lane
                row, c = e // G.CH, e % G.CH
                v = lds.read(qlds + row * QS + c * 16, 16, "output staging")
                ok = (row < qrows[w]) & (c < chq)
                if ok.any():
                    g_out.write(qbyte0[w] + row[ok] * da * 2 + c[ok] * 16, v[ok] + 1, "output rows")   # (+1: marks what was written)
        else:
            need(buffers.get("partial") is not None, "a piece of a split history needs the workspace")
            g_ws = Memory("partial", buffers["partial"])
            QB = item["QB"]
            ws0 = item["part"] * QB * (da + 2) * 4
            FS = DA * 4 + 16
            need(NW * QG * 32 * FS <= G.NS * G.STAGE, "the staged accumulators must fit in the retired stages")
            flds = w * QG * 32 * FS
            for g in range(QG):
                j = (w * QG + g) * 32 + qn
                for dt in range(DA // 32):
                    for r in range(16):
                        ci = 32 * dt + 8 * (r >> 2) + 4 * hh + (r & 3)
                        pc = np.where(ci < dgv, ci + duv, np.where(ci < da, ci - dgv, ci))
                        lds.write(flds + (g * 32 + qn) * FS + pc * 4, np.zeros((64, 4), np.uint8), "accumulator staging")
                low = hh == 0
                g_ws.write(ws0 + (QB * da + j[low]) * 4, np.ones((int(low.sum()), 4), np.uint8), "piece maximum")
                g_ws.write(ws0 + (QB * da + QB + j[low]) * 4, np.ones((int(low.sum()), 4), np.uint8), "piece sum")
            for i in range(QG * 32 * (DA // 4) // 64):
                e = i * 64 + lane
                row, c = e // (DA // 4), e % (DA // 4)
                v = lds.read(flds + row * FS + c * 16, 16, "accumulator staging")
                ok = c < (da >> 2)
                g_ws.write(ws0 + ((w * QG * 32 + row[ok]) * da + c[ok] * 4) * 4, v[ok] + 1, "piece accumulators")
    return {"peak_outstanding": max(wv.peak for wv in waves), "lds_bytes": G.LDS, "nui": nui, "UK": UK, "NS": G.NS}
