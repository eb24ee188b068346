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


def reduction_close(got, ref, rel=1e-5):
    """Per-element rel, falling back to norm-wise rel * max|ref| (cancelling sums)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    scale = np.max(np.abs(ref)) if ref.size else 0.0
    tol = np.maximum(rel * np.abs(ref), rel * scale)
    return np.abs(got - ref) <= tol
