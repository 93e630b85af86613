"""Comparison rule shared by the GPU parity tests.

Tolerance (the benchmark spec): 1e-4 relative for fp32 storage, 2e-2 relative for bf16 storage.
"Relative" is applied per output element against a floor of the row's own scale:
    |g - r| <= tol * |r| + tol * rms(r over the d_a columns of that query)
because an attention output is a signed sum, so single elements can sit arbitrarily close
to zero while their rounding error is set by the size of the summands.  The norm-wise
figure max|g - r| / max|r| is returned as well.
"""
import numpy as np

TOL = {0: 1e-4, 1: 2e-2}


def check(gpu, ref, dtype, rows=None, what=""):
    """gpu, ref: float64 [B][H][Nq][d_a]; rows: optional index of users to compare."""
    if rows is not None:
        gpu, ref = gpu[rows], ref[rows]
    assert gpu.shape == ref.shape
    assert np.isfinite(ref).all(), f"{what}: oracle produced non-finite values"
    assert np.isfinite(gpu).all(), f"{what}: GPU produced non-finite values"
    tol = TOL[dtype]
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    bound = tol * np.abs(ref) + tol * rms
    err = np.abs(gpu - ref)
    worst = float(np.max(err - bound)) if err.size else 0.0
    norm = float(err.max() / max(np.abs(ref).max(), 1e-300)) if err.size else 0.0
    # exact zeros (empty histories) must be exact
    zero_rows = (rms[..., 0] == 0)
    assert np.all(gpu[zero_rows] == 0), f"{what}: rows that must be exactly zero are not"
    assert worst <= 0, f"{what}: element error exceeds tol={tol}: max excess {worst:.3e}, norm-wise {norm:.3e}"
    return norm
