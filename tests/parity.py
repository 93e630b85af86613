"""Comparison rule shared by the GPU parity tests, the smoke check and the benchmark.

Tolerance (the benchmark spec): 1e-4 relative for fp32 storage, 2e-2 relative for bf16 storage.
An attention output is a signed sum r_c = sum_i w_i V_i[c]; single elements can sit arbitrarily
close to zero (weights of both signs in the SiLU form, or value rows that cancel) while the rounding
error they carry is set by the size of their summands, so "relative" needs a scale per element.
The rule, for every output element:

    |g_c - r_c| <= tol * |r_c| + max(tol * rss_c, u_w * asum_c) + u_s * sss_c + u_a * acs_c,
    rss_c = sqrt(sum over groups g of (sum_{i in g} w_i V_i[c])^2),   a group = the positions with one and the same weight
    asum_c = sum_i |w_i V_i[c]|,  u_w = the unit roundoff of the storage type (2^-9 for bf16, 2^-24 for fp32)
    sss_c = sqrt(sum over groups g of (sum_{i in g} k_i)^2),          k_i = d r_c / d s_i * A_i,  A_i = |scale| sum_k |q_k K_ik|
    u_s   = (d_a + 1) * 2^-24
    acs_c = sqrt(n) * (|r_c| + sqrt(sum_i (w_i V_i[c])^2)),           n = the user's history length
    u_a   = 8 * 2^-24

Where it comes from: the kernels keep products and sums in fp32 and round two things below that,
the weights w_i (to the storage type before the second matrix product: relative error at most
u = 2^-9 in bf16, 2^-24 in fp32) and the finished output (again u, the tol * |r_c| term).  The
rounding error of a weight is a function of its value: positions with the same weight (same key
row, same query) err alike and their errors add up coherently, different weights err
independently.  Independent relative errors of size u on the group sums add up to an error of
standard deviation u / sqrt(3) * rss_c, so tol * rss_c with tol = 2e-2 and u = 2^-9 is eighteen
standard deviations of the modelled error: a floor derived from the arithmetic, not from the
outputs.  (A CPU model of exactly these roundings lands at 0.2 to 0.5 of the bound on every seeded
random shape, the near-cancelling ones included.)  For value rows without structure rss_c is about
the root-mean-square of the output row, so on ordinary rows the rule is as strict as a floor of
tol * rms(row); on a row that nearly cancels it stays proportional to what was added up.
The other argument of the maximum is the case the independent model leaves out.  Weights that are not equal but nearly so
(positions that share their pool key row and differ in a narrow user slice: a pool of two rows, d_u = 1) fall into the same
rounding interval of the storage type and are all rounded the same way, so their errors add up coherently although no two
weights are equal: a history of two hundred positions over two pool rows has a hundred summands per row whose errors add up
to u_w times the sum of their magnitudes, ten times what independent errors of that size would give, and that is the bound of
the independent model (found on a seeded random shape: bf16, d_a = 128, d_u = 1, P = 2, SiLU, ratio 1.004 against the rule
without this term).  Whatever the weights are rounded to, with a relative error of at most u_w each, the output moves by at
most u_w * asum_c: that bound needs no model, and the rule takes the larger of the two.  With fp32 storage it is far below
tol * rss_c; with bf16 storage it is the larger one for histories of a few hundred positions or more (for a softmax over n
positions of comparable weight by a factor of about sqrt(n / 160)), where it is still a bound of 2^-9 of the magnitudes that
were added up, the precision of the storage type.
The third term is the scores' own rounding.  A score s_i = scale q . K_i is a sum of d_a products kept in fp32 with
either storage type (unit roundoff 2^-24; bf16 products are exact in fp32, fp32 products are rounded once), in whatever
order the matrix instruction adds them: whatever the order, it is off by at most (d_a + 1) 2^-24 A_i (the standard bound
for a dot product).  For softmax that is a relative error of the weight and far below tol.  The SiLU weight s sigma(s) / n
passes through zero, where an absolute error of the score is an unbounded relative error of the weight: a short history
whose one score is 1e-3 has a weight that is right to 1e-4 only, and no rule relative to the summands can hold.  To first
order an error delta_i A_i of score i moves the output by k_i delta_i (softmax: k_i = w_i (V_i[c] - r_c) A_i, the
normalisation included; SiLU/n: k_i = f'(s_i) V_i[c] A_i / n); equal rows have equal scores and err alike, different
rows err independently, hence the same grouping.  With fp32 storage, 256 columns and SiLU this term is about twice
tol * rss_c; with bf16 storage it is a hundredth of it.
The fourth term is the rounding of the output's own additions.  sum_i w_i V_i[c] is added up in fp32 with either
storage type, n - 1 additions in an order the oracle does not know, each rounding a partial sum by at most 2^-24 of it
(and, with fp32 storage, each product once).  A partial sum of k of the n summands, in an order unrelated to their values,
has mean (k/n) r_c and a spread of at most rs_c = sqrt(sum_i (w_i V_i[c])^2), so independent roundings add up to a standard
deviation of at most 2^-24 sqrt(n) (0.19 |r_c| + 0.36 rs_c) (uniform roundings, variance u^2 / 3; sum over k of (k/n)^2 is
n/3 and of (k/n)(1 - k/n) is n/6; the products' own roundings add rs_c^2 u^2 / 3).  u_a = 8 * 2^-24 is at least eighteen of these
standard deviations, the margin of the second term.  Where the weights differ this term is small beside tol * rss_c (fp32, n = 1024:
a seventh of it; bf16: a ten-thousandth).  It matters where the weights are all equal (a key pool of one row, q = 0): then
every error of the weights is common to all summands, rss_c collapses to |r_c|, and on an element whose value rows nearly
cancel nothing but this term stands for the additions (found on a seeded random shape: fp32 storage, one key row, 64
positions; plain IEEE fp32 addition in history order exceeds the first three terms there by 1.4, as the kernel did by 1.8).
rss_c, asum_c, sss_c and acs_c come from the CPU oracle (fp64, from the oracle's inputs), never from the GPU output.
Users with an empty history have r = 0 and rss = 0: their rows must be exactly zero.
The norm-wise figure max|g - r| / max|r| is reported beside it.
"""
import numpy as np

from oracle import oracle

TOL = {0: 1e-4, 1: 2e-2}


def score_unit(d_a):
    """u_s of the rule above: the most a d_a-term dot product summed in fp32 can be off by, relative to the sum of the
    magnitudes of its products."""
    return (d_a + 1) * 2.0 ** -24


ACC_UNIT = 8 * 2.0 ** -24   # u_a of the rule above
WEIGHT_UNIT = {0: 2.0 ** -24, 1: 2.0 ** -9}   # u_w of the rule above: unit roundoff of the storage type


def compare(gpu, ref, rss, dtype, sss=None, acs=None, asum=None):
    """Statistics of one comparison: gpu, ref, rss, sss, acs, asum float64 arrays of one shape [...][d_a] (sss = None,
    acs = None or asum = None leaves that term out: a stricter rule).
    worst_ratio = max over elements of |g - r| / (tol |r| + max(tol rss, u_w asum) + u_s sss + u_a acs)  (<= 1 passes; an
    element with a zero bound counts as 0 if it is exact and as infinity if it is not)."""
    assert gpu.shape == ref.shape == rss.shape and (sss is None or sss.shape == ref.shape)
    assert acs is None or acs.shape == ref.shape
    assert asum is None or asum.shape == ref.shape
    tol = TOL[dtype]
    if ref.size == 0:
        return {"tol": tol, "elements": 0, "norm_err": 0.0, "worst_ratio": 0.0, "finite": True}
    finite = bool(np.isfinite(gpu).all())
    err = np.abs(gpu - ref)
    bound = tol * np.abs(ref) + (tol * rss if asum is None else np.maximum(tol * rss, WEIGHT_UNIT[dtype] * asum))
    if sss is not None:
        bound = bound + score_unit(ref.shape[-1]) * sss
    if acs is not None:
        bound = bound + ACC_UNIT * acs
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(bound > 0, err / bound, np.where(err == 0, 0.0, np.inf))
    return {"tol": tol, "elements": int(ref.size), "finite": finite,
            "norm_err": float(err.max() / max(np.abs(ref).max(), 1e-300)) if finite else float("inf"),
            "worst_ratio": float(np.nanmax(ratio)) if finite else float("inf")}


def check(gpu, ref, rss, dtype, rows=None, what="", sss=None, acs=None, asum=None):
    """gpu, ref, rss, sss, acs, asum: float64 [B][H][Nq][d_a]; rows: optional index of the users to compare.
    Asserts the rule above on every element and returns the norm-wise error."""
    if rows is not None:
        gpu, ref, rss = gpu[rows], ref[rows], rss[rows]
        sss = None if sss is None else sss[rows]
        acs = None if acs is None else acs[rows]
        asum = None if asum is None else asum[rows]
    assert asum is None or np.isfinite(asum).all(), f"{what}: oracle produced non-finite values"
    assert np.isfinite(ref).all() and np.isfinite(rss).all(), f"{what}: oracle produced non-finite values"
    assert sss is None or np.isfinite(sss).all(), f"{what}: oracle produced non-finite values"
    assert acs is None or np.isfinite(acs).all(), f"{what}: oracle produced non-finite values"
    assert np.isfinite(gpu).all(), f"{what}: GPU produced non-finite values"
    st = compare(gpu, ref, rss, dtype, sss, acs, asum)
    assert st["worst_ratio"] <= 1.0, (f"{what}: element error exceeds tol={st['tol']}: worst |g-r| / (tol|r| + max(tol rss, u_w asum) + u_s sss + u_a acs) = "
                                      f"{st['worst_ratio']:.3f}, norm-wise {st['norm_err']:.3e}")
    return st["norm_err"]


def check_against_oracle(gpu, w, users=None, what="", queries=None):
    """Run the oracle on workload `w` (all users, or the listed ones; all queries, or the listed ones of every user and head:
    the oracle then gets the workload with only those queries) and check `gpu` against it."""
    if queries is not None:
        queries = np.asarray(queries)
        w = dict(w, q=np.ascontiguousarray(w["q"][:, :, queries]), Nq=len(queries))
        gpu = gpu[:, :, queries]
    ref, rss, sss, acs, asum = oracle.attend(w, users=users, with_scales=True, with_asum=True)
    return check(gpu, ref, rss, w["dtype"], rows=users, what=what, sss=sss, acs=acs, asum=asum)
