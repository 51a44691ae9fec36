"""Helpers of the GPU parity tests: run the HIP path through the C-ABI, compare with the oracle."""
import numpy as np

import oracle

# The acceptance rule for floating point: |y_gpu - y_ref| <= 1e-3 * sum_j |W_ij||x_j| per output.
# The output is binary16: where that bound is below the spacing of binary16 subnormals (2^-24) no
# binary16 value may lie within it, so there (and only there) half that spacing is added.
REL_TOL = 1e-3
SUBNORMAL_SPACING = 2.0 ** -24


def tolerance(mag):
    tol = REL_TOL * np.asarray(mag, dtype=np.float64)
    return np.where(tol < SUBNORMAL_SPACING, tol + SUBNORMAL_SPACING / 2, tol)


def run_gemv(pm, b, x_np):
    import torch
    from paper_2402_10517_amd import binding as B
    x = torch.from_numpy(np.ascontiguousarray(x_np)).cuda()
    y = B.ap_gemv(pm, b, x)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check_against_oracle(y_gpu, idx, lut, b, x, n=8, rows=None):
    """Element-by-element comparison; rows = optional subset of output rows (sampled check)."""
    if rows is not None:
        rows = np.asarray(rows)
        y_ref, mag = oracle.gemv(idx[rows], lut[rows], b, x, n=n)
        y_gpu = y_gpu[:, rows]
    else:
        y_ref, mag = oracle.gemv(idx, lut, b, x, n=n)
    assert y_gpu.shape == y_ref.shape
    got = y_gpu.astype(np.float64)
    assert np.all(np.isfinite(got)), "non-finite output"
    err = np.abs(got - y_ref)
    tol = tolerance(mag)
    worst = float(np.max(err / tol))
    assert worst <= 1.0, "max err/tol = %.3f at %s" % (worst, np.unravel_index(np.argmax(err / tol), err.shape))
    return worst
