"""Error metric shared by the GPU parity tests.

The bound on the features is 1e-5 maximum relative error in fp32.  Sums of
signed terms can cancel to (almost) zero, where an element-wise ratio is
meaningless for any fp32 implementation, so the ratio is taken row-wise
against the largest magnitude in the row:

    err(row) = max_j |gpu - oracle| / max(max_j |oracle|, tiny)

and maximised over rows.  The oracle side is fp64.

Next to it stands the condition-aware element-wise measure: every output element is a sum
of terms c_vu * z_uj, and a float32 evaluation of a sum is accurate relative to the size of
its terms,

    err(v, j) = |gpu - oracle| / sum_u |c_vu z_uj|

with the denominator from the oracle's own loops (``oracle.aggregate_abs``).  It needs no
robust row magnitude, so it also judges rows of one or a few signed columns.  An element
whose terms are all zero must be exactly zero.
"""
import numpy as np

TOL = 1e-5


def row_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if got.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite value in GPU output"
    num = np.abs(got - want).max(axis=1)
    den = np.maximum(np.abs(want).max(axis=1), 1e-30)
    # a row that is exactly zero in the oracle must be exactly zero on the GPU
    zero = np.abs(want).max(axis=1) == 0
    if np.any(num[zero] != 0):
        return float("inf")
    return float((num[~zero] / den[~zero]).max(initial=0.0))


def assert_close(got, want, tol=TOL, what=""):
    e = row_rel_err(got, want)
    assert e <= tol, "%s: max row-relative error %.3e > %.1e" % (what, e, tol)
    return e


def cond_rel_err(got: np.ndarray, want: np.ndarray, mag: np.ndarray) -> float:
    """max over elements of |got - want| / mag, mag = size of the terms behind the element."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    mag = np.asarray(mag, np.float64)
    assert got.shape == want.shape == mag.shape, (got.shape, want.shape, mag.shape)
    if got.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite value in GPU output"
    num = np.abs(got - want)
    zero = mag == 0
    if np.any(num[zero] != 0):
        return float("inf")
    return float((num[~zero] / mag[~zero]).max(initial=0.0))


def assert_cond_close(got, want, mag, tol=TOL, what=""):
    e = cond_rel_err(got, want, mag)
    assert e <= tol, "%s: max element-wise error relative to the size of the terms %.3e > %.1e" % (what, e, tol)
    return e
