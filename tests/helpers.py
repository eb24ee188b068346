"""Comparison helpers shared by the tests (no arithmetic of the method)."""
import numpy as np


def ulp_of(x: np.ndarray) -> np.ndarray:
    """Spacing of float32 at |x| (at least the subnormal spacing)."""
    x = np.abs(np.asarray(x, dtype=np.float32))
    return np.maximum(np.spacing(x), np.float32(2.0 ** -149)).astype(np.float64)


def elementwise_close(got, ref, ulps=2.0, rel=1e-6, floor=None):
    """|got-ref| <= max(ulps*ulp(ref), rel*|ref|) per element; NaN/inf must match.

    ``floor`` (optional array) adds an absolute allowance per element, used
    where the last op of an expression is a cancelling subtraction.
    Returns the boolean array of passing elements.
    """
    got = np.asarray(got, dtype=np.float32)
    ref = np.asarray(ref, dtype=np.float32)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    g64, r64 = got.astype(np.float64), ref.astype(np.float64)
    finite = np.isfinite(r64)
    tol = np.maximum(ulps * ulp_of(ref), rel * np.abs(r64))
    if floor is not None:
        tol = np.maximum(tol, floor)
    with np.errstate(invalid="ignore"):
        ok_fin = np.abs(g64 - r64) <= tol
    same_special = (np.isnan(r64) & np.isnan(g64)) | ((r64 == g64) & ~finite)
    return np.where(finite, ok_fin, same_special)


def reduction_check(got, ref, rel=1e-5, scale=None):
    """The bar for results that contain a float32 reduction.

    Strict, per element: |got-ref| <= max(rel*|ref|, 2*ulp(ref)); NaN/inf must match.
    ``scale`` (optional array, broadcastable to ref) is the caller's explicit cancellation
    bound for the sums behind each element, sum|terms| as the oracle computes it: an
    element that misses the strict bar may still pass with |got-ref| <= rel*scale.
    There is no other fallback; in particular nothing is measured against the largest
    element of the array.

    Returns (ok, needed_scale): the boolean array of passing elements and the number of
    elements that passed only through ``scale``.
    """
    got = np.asarray(got)
    ref = np.asarray(ref)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    g64, r64 = got.astype(np.float64), ref.astype(np.float64)
    finite = np.isfinite(r64)
    tol = np.maximum(rel * np.abs(r64), 2.0 * ulp_of(ref))
    with np.errstate(invalid="ignore"):
        diff = np.abs(g64 - r64)
        strict = diff <= tol
        if scale is None:
            ok_fin = strict
        else:
            ok_fin = strict | (diff <= rel * np.broadcast_to(np.asarray(scale, dtype=np.float64), r64.shape))
    same_special = (np.isnan(r64) & np.isnan(g64)) | ((r64 == g64) & ~finite)
    ok = np.where(finite, ok_fin, same_special)
    needed = int(np.count_nonzero(finite & ok_fin & ~strict))
    return ok, needed


# (what, elements, elements that needed the cancellation scale): filled by the GPU parity
# tests, printed at the end of the session by conftest.py
SCALE_REPORT = []
