"""Program tables shared by the GPU parity tests and the host-side planning
tests: NumPy-style programs over an array module xp, with their inputs."""
import numpy as np

from paper_1901_03771_amd import workloads as wl

f32 = np.float32


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(f32)


ELEMENTWISE_CASES = {
    "unary_mix": (lambda xp, a: xp.sqrt(abs(a)) + xp.tanh(a) - xp.log(abs(a) + 1.0) + xp.exp(-abs(a)) + (-a) ** 2,
                  lambda: dict(a=_rand((37, 129), 1))),
    "bcast_col": (lambda xp, a, b: a * b - b, lambda: dict(a=_rand((45, 33), 2), b=_rand((45, 1), 3))),
    "bcast_row_col": (lambda xp, a, b: xp.maximum(a, b) + xp.minimum(a, b), lambda: dict(a=_rand((1, 257), 4), b=_rand((19, 1), 5))),
    "bcast_3d": (lambda xp, a, b, c: (a + b) / (abs(c) + 1.0), lambda: dict(a=_rand((3, 1, 65), 6), b=_rand((5, 1), 7), c=_rand((3, 5, 65), 8))),
    "scalar_ops": (lambda xp, a: (2.0 - a) / 3.0 + 0.5 * a - 1, lambda: dict(a=_rand((1000,), 9))),
    "transpose_add": (lambda xp, a, b: a.T + b, lambda: dict(a=_rand((40, 70), 10), b=_rand((70, 40), 11))),
    "transpose_3d": (lambda xp, a, b: xp.transpose(a, (2, 0, 1)) * b, lambda: dict(a=_rand((4, 5, 6), 12), b=_rand((6, 4, 5), 13))),
    "slice_step": (lambda xp, a: a[1::2, ::3] - a[:-1:2, 1::3], lambda: dict(a=_rand((40, 60), 14))),
    "slice_shift_rows": (lambda xp, a: a[1:] - a[:-1], lambda: dict(a=_rand((50, 64), 15))),
    "slice_of_lazy": (lambda xp, a, b: ((a + b)[2:-3, 5:] * 2.0)[::2], lambda: dict(a=_rand((31, 47), 16), b=_rand((31, 47), 17))),
    "jacobi": (lambda xp, grid: wl.jacobi_sweep(xp, grid), lambda: dict(grid=_rand((67, 300), 18))),
    "diamond": (lambda xp, a: (lambda t: t * t + t)(a + 1.0), lambda: dict(a=_rand((513,), 19))),
    "nan_inf": (lambda xp, a, b: xp.maximum(a, b) / b,
                lambda: dict(a=np.array([1, np.nan, 3, -np.inf, 0, 5], f32), b=np.array([2, 1, np.nan, 1, 0, np.inf], f32))),
    "outer": (lambda xp, a, b: a * b, lambda: dict(a=_rand((300, 1), 20), b=_rand((1, 500), 21))),
}



REDUCTION_CASES = [((37, 211), 1, True), ((37, 211), 1, False), ((37, 211), 0, False), ((37, 211), None, False),
                   ((6, 7, 50), (0, 2), True), ((6, 7, 50), 1, False), ((5, 70000), 1, False),
                   ((20000, 3), 0, False), ((4, 5, 6), (1, 2), False), ((1, 1), None, True)]

ROWRED_PROGRAMS = [
    lambda xp, a: (a - xp.max(a, axis=1, keepdims=True)) / (xp.sum(abs(a), axis=1, keepdims=True) + 1.0),
    lambda xp, a: 1.0 / xp.sum(a * a, axis=1, keepdims=True),
    lambda xp, a: xp.sum(xp.exp(a - xp.max(a, axis=1, keepdims=True)), axis=1),
    lambda xp, a: a[:, 1:] / (xp.sum(abs(a[:, 1:] - a[:, :-1]), axis=1, keepdims=True) + 1.0),
    lambda xp, a: xp.max(a, axis=1) - xp.min(a, axis=1),
    lambda xp, a: a - xp.max(a, axis=1),            # (50,50): the row maxima broadcast along rows, not row-resident
    lambda xp, a: xp.sum(a, axis=1, keepdims=True) * xp.sum(a, axis=0, keepdims=True),
]

DOT_CASES = [
    (lambda xp, A, v, u: A @ v, "row-dot"),
    (lambda xp, A, v, u: A.T @ u, "column-accumulate"),
    (lambda xp, A, v, u: xp.dot(v, v), "inner product"),
    (lambda xp, A, v, u: xp.sum(v * v), "Listing 5 inner product"),
    (lambda xp, A, v, u: A[::2, 1::2] @ v[1::2], "strided views"),
    (lambda xp, A, v, u: xp.tanh(A @ (v * 2.0 + 1.0)) + u, "lazy vector operand + epilogue"),
    (lambda xp, A, v, u: (A @ v) * (A @ v) + u, "dot used twice"),
    (lambda xp, A, v, u: A.T @ (A @ v), "dot feeding dot"),
    # slices that start at or beyond their step (the shift is not absorbed by the stride pattern)
    (lambda xp, A, v, u: A[3:, 5:] @ v[5:], "offset matrix and vector"),
    (lambda xp, A, v, u: A.T[7:, 2:] @ u[2:], "offset transposed matrix"),
    (lambda xp, A, v, u: A[1::2, 48:51:2] @ v[100:104:2], "offset and step"),
    (lambda xp, A, v, u: xp.dot(v[5:], v[:-5]), "inner product of two windows of one array"),
    (lambda xp, A, v, u: A[10:20, 5:] @ xp.transpose(A[30:31, 5:], (1, 0)), "matrix times a column taken from itself"),
]

# long contractions with few rows (planned as two-stage reductions): (name, shapes of A and v, program)
LONG_DOT_CASES = [
    ("inner product of 300001", (300001,), (300001,), lambda xp, A, v: xp.sqrt(abs(xp.dot(A, v))) + 1.0),
    ("three rows of 100003", (3, 100003), (100003,), lambda xp, A, v: xp.dot(A, v) * 2.0 - 1.0),
    ("windows of long rows", (5, 70000), (70000,), lambda xp, A, v: xp.dot(A[1:4, 7::2], v[7::2])),
    ("inner product of two windows of one array", (200000,), (200000,), lambda xp, A, v: xp.dot(A[5:], A[:-5])),
]

# arrays with a few columns (points, pixels) and contractions over a few terms (written out inside the
# point function): (name, {array name: shape}, program)
NARROW_CASES = [
    ("points minus centroid", dict(x=(5003, 3), c=(3,)), lambda xp, x, c: x - c),
    ("points scaled per row", dict(x=(5003, 3), c=(5003, 1)), lambda xp, x, c: x * c + 1.0),
    ("two columns", dict(x=(4099, 2), c=(2,)), lambda xp, x, c: xp.maximum(x, c) * 2.0),
    ("one column", dict(x=(4099, 1), c=(1,)), lambda xp, x, c: x + c),
    ("seven columns", dict(x=(3001, 7), c=(7,)), lambda xp, x, c: x * c - 1.0),
    ("five columns, stencil along rows", dict(x=(3001, 5), c=(5,)), lambda xp, x, c: x[2:] - x[:-2] + c),
    ("three columns, shifted columns", dict(x=(3001, 5), c=(3,)), lambda xp, x, c: x[:, 2:] + x[:, :-2] * c),
    ("61 columns", dict(x=(1001, 61), c=(61,)), lambda xp, x, c: x / (abs(c) + 1.0)),
    ("3-d, three channels last", dict(x=(37, 41, 3), c=(3,)), lambda xp, x, c: x * c + x),
    ("rotate points", dict(x=(5003, 3), c=(3, 3)), lambda xp, x, c: xp.dot(x, c)),
    ("rotate and shift", dict(x=(5003, 3), c=(3, 3), d=(3,)), lambda xp, x, c, d: xp.dot(x * 2.0, c) + d),
    ("weights of three", dict(x=(5003, 3), c=(3,)), lambda xp, x, c: xp.tanh(xp.dot(x, c))),
    ("transposed operand", dict(x=(3, 5003), c=(3,)), lambda xp, x, c: xp.dot(xp.transpose(x, (1, 0)), c) - 1.0),
    ("eight terms, wide result", dict(x=(301, 8), c=(8, 1030)), lambda xp, x, c: xp.dot(x, c)),
    ("one term (outer product)", dict(x=(301, 1), c=(1, 130)), lambda xp, x, c: xp.dot(x, c) + 1.0),
    ("no term (empty contraction)", dict(x=(5, 0), c=(0, 7)), lambda xp, x, c: xp.dot(x, c) + 1.0),
    ("softmax of a small product", dict(x=(2003, 4), c=(4, 6)),
     lambda xp, x, c: xp.exp(xp.dot(x, c) - xp.max(xp.dot(x, c), axis=1, keepdims=True)) / xp.sum(xp.exp(xp.dot(x, c) - xp.max(xp.dot(x, c), axis=1, keepdims=True)), axis=1, keepdims=True)),
    ("small product feeding a large one", dict(x=(257, 3), c=(3, 12), d=(12, 40)), lambda xp, x, c, d: xp.dot(xp.dot(x, c), d[:, :33])),
    ("scan of a small product", dict(x=(1003, 3), c=(3, 3)), lambda xp, x, c: xp.cumsum(xp.dot(x, c), 0)),
]

# (shape, axis): inclusive scans along the contiguous axis, along outer axes, over long lines
SCAN_CASES = [((1000,), 0), ((37, 211), 1), ((37, 211), 0), ((4, 5, 6), 1), ((4, 5, 6), 0), ((4, 5, 6), -1), ((3, 100000), 1),
              ((1 << 21,), 0), ((5, 1), 1), ((1, 7), 0), ((1,), 0), ((600, 1030), 1), ((2, 5000), 0),
              # long lines along an axis that is not contiguous: a thread per (line, chunk)
              ((1000, 300), 0), ((4100, 7), 0), ((3, 2000, 5), 1), ((129, 1), 0), ((70000, 2), 0),
              # batches of eight steps with a ragged tail: chunked (four lines per thread, one line per thread)
              # and in one pass over the lines (enough lines for that: 2^14 threads of four lines, 2^15 of one)
              ((1003, 300), 0), ((1003, 301), 0), ((139, 65540), 0), ((131, 33001), 0), ((5, 143, 13108), 1),
              # few lines, four to a lane: one pass over tiles of neighbouring lines kept in registers (several
              # tiles and groups of tiles per chain, ragged last tile and last column block, outer dimensions,
              # fewer lines than a tile is wide)
              ((8200, 1028), 0), ((3, 2000, 520), 1), ((70000, 8), 0), ((5000, 12), 0), ((2, 131, 3, 64), 1), ((20000, 132), 0)]
