"""Seeded synthetic inputs and the NumPy-style user programs run on them.

This module holds no arithmetic of the method (no recording, fusion, code
generation or kernels) and imports neither the GPU binding nor the CPU
evaluator: it only draws input arrays and states, as ordinary array
expressions over an array module ``xp``, the programs a user of a NumPy
drop-in replacement would write (Section 1 and Section 4.1 of the paper:
the user changes the import, not the program).  The same program text is
handed to the lazy GPU module and to the eager CPU evaluator.

The paper's own benchmark inputs are not published (its plots carry no sizes
or distributions); the configurations below are synthetic stand-ins shaped
like its samples: a long pointwise chain (Black-Scholes-like), a broadcast
normalisation, a row softmax, a two-level slice stencil (Jacobi / image
processing, Listing 6) and a dot-bounded logistic-regression step (the
MNIST / RNN pattern of Listing 2).
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 190103771

# name -> full-size shape parameters; "small" variants keep several tiles and
# a ragged tail while staying cheap for an op-by-op CPU evaluation.
FULL = {
    "chain": dict(n=1 << 20),
    "normalize": dict(rows=8192, cols=8192),
    "softmax": dict(rows=16384, cols=4096),
    "stencil": dict(rows=8192, cols=8192),
    "logreg": dict(rows=262144, cols=512),
    "blackscholes": dict(n=1 << 24),
    "cumsum": dict(n=1 << 27),
    "cumsum_axis0": dict(rows=8192, cols=8192),
    "gemm": dict(m=4096, k=4096, n=4096),
}
SMALL = {
    "chain": dict(n=100_003),
    "normalize": dict(rows=203, cols=1501),
    "softmax": dict(rows=67, cols=1000),
    "stencil": dict(rows=151, cols=1234),
    "logreg": dict(rows=3001, cols=200),
    "blackscholes": dict(n=70_001),
    "cumsum": dict(n=300_001),
    "cumsum_axis0": dict(rows=1203, cols=516),
    "gemm": dict(m=515, k=1030, n=259),
}
CONFIG_INDEX = {"chain": 0, "normalize": 1, "softmax": 2, "stencil": 3, "logreg": 4, "blackscholes": 5, "cumsum": 6, "cumsum_axis0": 7, "gemm": 8}


def rng_for(name: str, salt: int = 0) -> np.random.Generator:
    return np.random.default_rng(SEED_BASE + CONFIG_INDEX[name] + 1000 * salt)


def make_inputs(name: str, salt: int = 0, **size) -> dict:
    """Draw the input arrays of configuration ``name`` (float32, C-contiguous)."""
    p = dict(FULL[name])
    p.update(size)
    g = rng_for(name, salt)
    f32 = np.float32
    if name == "chain":
        n = p["n"]
        return dict(a=g.uniform(-1, 1, n).astype(f32), b=g.uniform(-1, 1, n).astype(f32))
    if name == "normalize":
        r, c = p["rows"], p["cols"]
        return dict(
            X=g.standard_normal((r, c), dtype=f32),
            mu=g.uniform(-0.5, 0.5, (1, c)).astype(f32),
            sigma=g.uniform(0.5, 2.0, (1, c)).astype(f32),
            gamma=g.uniform(0.5, 1.5, (c,)).astype(f32),
            beta=g.uniform(0.5, 1.5, (c,)).astype(f32),
        )
    if name == "softmax":
        r, c = p["rows"], p["cols"]
        # N(0, 4) is read as variance 4, i.e. standard deviation 2.
        return dict(X=(2.0 * g.standard_normal((r, c), dtype=f32)).astype(f32))
    if name == "stencil":
        r, c = p["rows"], p["cols"]
        return dict(I=(g.random((r, c), dtype=f32) * f32(255.0)).astype(f32))
    if name == "logreg":
        r, c = p["rows"], p["cols"]
        # N(0, 0.05) is read as variance 0.05.
        return dict(
            X=g.standard_normal((r, c), dtype=f32),
            w=(np.sqrt(0.05) * g.standard_normal(c)).astype(f32),
            y=(g.random(r) < 0.5).astype(f32),
        )
    if name == "blackscholes":
        n = p["n"]
        # option parameters in the ranges commonly used for synthetic pricing benchmarks
        return dict(S=g.uniform(5.0, 30.0, n).astype(f32), K=g.uniform(1.0, 100.0, n).astype(f32),
                    T=g.uniform(0.25, 10.0, n).astype(f32))
    if name == "cumsum":
        return dict(x=g.random(p["n"], dtype=f32))
    if name == "cumsum_axis0":
        return dict(X=g.random((p["rows"], p["cols"]), dtype=f32))
    if name == "gemm":
        return dict(A=g.standard_normal((p["m"], p["k"]), dtype=f32), B=g.standard_normal((p["k"], p["n"]), dtype=f32))
    raise KeyError(name)


# ---- user programs (array expressions over a NumPy-like module xp) ----------

def chain(xp, a, b):
    return ((a + b) * (a - b) + 2.5 * a) / (abs(b) + 1.0) - xp.exp(-a * a)


def normalize(xp, X, mu, sigma, gamma, beta):
    return xp.maximum((X - mu) / sigma * gamma + beta, 0)


def softmax(xp, X):
    m = xp.max(X, axis=1, keepdims=True)
    e = xp.exp(X - m)
    return e / xp.sum(e, axis=1, keepdims=True)


def stencil(xp, I):
    B = 0.2 * (I[1:-1, 1:-1] + I[:-2, 1:-1] + I[2:, 1:-1] + I[1:-1, :-2] + I[1:-1, 2:])
    return xp.sqrt((B[1:-1, 2:] - B[1:-1, :-2]) ** 2 + (B[2:, 1:-1] - B[:-2, 1:-1]) ** 2)


def logreg(xp, X, w, y):
    n = X.shape[0]
    p = 1.0 / (1.0 + xp.exp(-(X @ w)))
    r = p - y
    g = (X.T @ r) / n + 1e-4 * w
    return w - 0.1 * g


def blackscholes(xp, S, K, T, r=0.02, sigma=0.30):
    """European call price by the Black-Scholes formula: a long pointwise chain with log,
    sqrt, exp and erf, the shape of the paper's best-case benchmark (Section 4.2)."""
    sqrt_t = xp.sqrt(T)
    d1 = (xp.log(S / K) + (r + 0.5 * sigma * sigma) * T) / (sigma * sqrt_t)
    d2 = d1 - sigma * sqrt_t
    cdf1 = 0.5 * (1.0 + xp.erf(d1 / 1.4142135623730951))
    cdf2 = 0.5 * (1.0 + xp.erf(d2 / 1.4142135623730951))
    return S * cdf1 - K * xp.exp(-r * T) * cdf2


def prefix_sum(xp, x):
    """Running sum of a long vector: the map-scan primitive (Section 3.2) on its own."""
    return xp.cumsum(x, 0)


def prefix_sum_of_columns(xp, X):
    """Running sums down the columns of a matrix: a scan along the axis that is not contiguous."""
    return xp.cumsum(X, 0)


def matrix_product(xp, A, B):
    """The dense contraction that the paper hands to a BLAS library (Section 2, the operations better left to libraries)."""
    return A @ B


PROGRAMS = {"gemm": matrix_product, "cumsum_axis0": prefix_sum_of_columns, "cumsum": prefix_sum, "blackscholes": blackscholes, "chain": chain, "normalize": normalize, "softmax": softmax, "stencil": stencil, "logreg": logreg}


def unique_bytes(name: str, **size) -> int:
    """Unique input bytes + output bytes of one evaluation (the metric's numerator)."""
    p = dict(FULL[name])
    p.update(size)
    if name == "chain":
        return 12 * p["n"]
    if name == "blackscholes":
        return 16 * p["n"]
    if name == "cumsum":
        return 8 * p["n"]
    if name == "cumsum_axis0":
        return 8 * p["rows"] * p["cols"]
    if name == "gemm":
        return 4 * (p["m"] * p["k"] + p["k"] * p["n"] + p["m"] * p["n"])
    if name == "normalize":
        return 8 * p["rows"] * p["cols"] + 16 * p["cols"]
    if name == "softmax":
        return 8 * p["rows"] * p["cols"]
    if name == "stencil":
        return 4 * p["rows"] * p["cols"] + 4 * (p["rows"] - 4) * (p["cols"] - 4)
    if name == "logreg":
        return 4 * p["rows"] * p["cols"] + 4 * p["cols"] + 4 * p["rows"] + 4 * p["cols"]
    raise KeyError(name)


# ---- the paper's own small listings ----------------------------------------

def listing1(xp, x, y):
    """Listing 1: z = x*x + 2*x*y + y*y on int32 arrays."""
    return x * x + 2 * x * y + y * y


def mnist(xp, W, a, b):
    """Listing 2, with W of shape (200, 10) so that W.T @ a is defined and
    the builtin max read as an elementwise maximum."""
    x = xp.transpose(W).dot(xp.maximum(a, 0)) + b
    return 1.0 / (1.0 + xp.exp(-x))


# The five-point neighbourhood of the paper's Jacobi benchmark (Listing 6): (row, column) shifts of the
# windows that are added, in the listing's order; every sweep replaces the interior by a fifth of their sum.
FIVE_POINT = ((0, 0), (-1, 0), (0, 1), (0, -1), (1, 0))


def shifted_windows(grid, offsets=FIVE_POINT, margin=1):
    """Views of `grid` with `margin` cells cut off all round, shifted by each (row, column) offset."""
    rows, cols = grid.shape
    return [grid[margin + dr:rows - margin + dr, margin + dc:cols - margin + dc] for dr, dc in offsets]


def stencil_sum(windows, weight=0.2):
    total = windows[0]
    for w in windows[1:]:
        total = total + w
    return weight * total


def jacobi_sweep(xp, grid):
    """Right-hand side of one sweep of Listing 6."""
    return stencil_sum(shifted_windows(grid))


def jacobi(xp, grid, iterations):
    """Listing 6 in full: the views are taken once, every sweep assigns through the unshifted one."""
    windows = shifted_windows(grid)
    for _ in range(iterations):
        windows[0][:] = stencil_sum(windows)
    return grid


def inner_product(xp, a, b):
    """Listing 5: map a[i]*b[i], reduce with +."""
    return xp.sum(a * b)
