"""Pins for the CPU oracle (oracle/eager.cpp) against things other than itself:
the paper's worked example, closed forms, brute force on tiny arrays written
here as plain Python loops, exact rational arithmetic, and NumPy as a third
opinion.  A dropped term, a wrong sign or index, or a transposed operand in
the oracle fails at least one of these."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle as ora
from paper_1901_03771_amd import workloads as wl
from helpers import elementwise_close, ulp_of

f32 = np.float32
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed=0):
    return np.random.default_rng(1901 + seed)


# ---------------------------------------------------------------- broadcast --
BROADCAST_TABLE = [
    ((10, 20), (20,), (10, 20)),
    ((64, 48), (1, 48), (64, 48)),
    ((64, 48), (48,), (64, 48)),
    ((32, 16), (32, 1), (32, 16)),
    ((3, 1), (1, 4), (3, 4)),
    ((5,), (5,), (5,)),
    ((0, 3), (1, 3), (0, 3)),
    ((2, 1, 4), (3, 1), (2, 3, 4)),
    ((7, 1, 5), (1, 6, 1), (7, 6, 5)),
    ((2, 3), (2,), None),
    ((4,), (5,), None),
    ((2, 3), (3, 2), None),
]


@pytest.mark.parametrize("sa,sb,expect", BROADCAST_TABLE)
def test_broadcast_table(sa, sb, expect):
    a = ora.array(np.ones(sa, f32))
    b = ora.array(np.ones(sb, f32))
    if expect is None:
        with pytest.raises(ora.OracleError):
            ora.add(a, b)
    else:
        assert ora.add(a, b).shape == expect


def test_broadcast_values_brute_force():
    # hand loop: out[i][j][k] = a[i][0][k] - b[j][0]
    g = rng(1)
    a = g.standard_normal((2, 1, 4)).astype(f32)
    b = g.standard_normal((3, 1)).astype(f32)
    got = (ora.array(a) - ora.array(b)).numpy()
    for i, j, k in itertools.product(range(2), range(3), range(4)):
        assert got[i, j, k] == f32(a[i, 0, k] - b[j, 0])


def test_scalar_broadcast_rank0():
    a = np.arange(5, dtype=f32)
    got = (ora.array(a) + 1.5).numpy()
    assert got.shape == (5,)
    assert np.array_equal(got, a + f32(1.5))


# ------------------------------------------------------ paper's Listing 1 ----
def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                rows.append(np.array(line.split(), dtype=np.int32))
    return rows


def test_listing1_literal_values():
    x, y, z = _read_golden("listing1_literal.txt")
    got = wl.listing1(ora, ora.array(x), ora.array(y)).numpy()
    assert got.dtype == np.int32
    assert np.array_equal(got, z)


def test_listing1_shape_reading_ring_identity_with_wraparound():
    # Listing 3 reads x as [10][20], y as [20]; z == (x+y)^2 holds exactly in
    # the ring Z/2^32, overflow included.
    g = rng(2)
    x = g.integers(-2**31, 2**31 - 1, (10, 20), dtype=np.int64).astype(np.int32)
    y = g.integers(-2**31, 2**31 - 1, (20,), dtype=np.int64).astype(np.int32)
    got = wl.listing1(ora, ora.array(x), ora.array(y)).numpy()
    # Python big ints, reduced mod 2^32, then reinterpreted as signed
    for i, j in itertools.product(range(10), range(20)):
        v = (int(x[i, j]) + int(y[j])) ** 2 % (1 << 32)
        v = v - (1 << 32) if v >= (1 << 31) else v
        assert int(got[i, j]) == v


def test_int32_abs_neg_edge():
    x = np.array([-2**31, -5, 0, 7, 2**31 - 1], dtype=np.int32)
    assert np.array_equal(abs(ora.array(x)).numpy(), np.array([-2**31, 5, 0, 7, 2**31 - 1], np.int32))
    assert np.array_equal((-ora.array(x)).numpy(), np.array([-2**31, 5, 0, -7, -(2**31 - 1)], np.int32))


def test_float_scalar_with_int_array_is_rejected():
    with pytest.raises(ora.OracleError):
        ora.array(np.arange(3, dtype=np.int32)) * 0.5
    with pytest.raises(ora.OracleError):
        ora.array(np.arange(3, dtype=np.int32)) + ora.array(np.ones(3, f32))


# ----------------------------------------------------------------- identities --
def test_identities():
    g = rng(3)
    x = (g.standard_normal(1000) * 100).astype(f32)
    X = ora.array(x)
    assert np.all((X - X).numpy() == 0)
    assert np.array_equal((X * 1.0).numpy(), x)
    assert np.array_equal(ora.maximum(X, X).numpy(), x)
    assert np.array_equal(abs(-X).numpy(), abs(X).numpy())
    assert np.array_equal(ora.sqrt(ora.square(X)).numpy(), np.abs(x))  # |x| ~ 100: x^2 is far from over/underflow
    assert np.array_equal((X + 0.0).numpy(), x)
    assert np.array_equal((X / 1.0).numpy(), x)
    assert np.array_equal((-(-X)).numpy(), x)


def test_sub_is_not_commuted_and_div_is_not_flipped():
    a, b = ora.array(np.array([7.0], f32)), ora.array(np.array([2.0], f32))
    assert (a - b).numpy()[0] == 5.0 and (b - a).numpy()[0] == -5.0
    assert (a / b).numpy()[0] == 3.5 and (b / a).numpy()[0] == f32(2.0) / f32(7.0)
    assert (10 - a).numpy()[0] == 3.0 and (14 / a).numpy()[0] == 2.0


def test_f32_rounding_is_single_op():
    # 1 + 2^-24 rounds to 1 in binary32 (ties to even); a double-precision
    # intermediate would keep it.
    one, tiny = ora.array(np.array([1.0], f32)), ora.array(np.array([2.0**-24], f32))
    assert ((one + tiny) - one).numpy()[0] == 0.0
    # scalar 0.2 is rounded to binary32 before use
    assert (one * 0.2).numpy()[0] == f32(0.2)
    assert float((one * 0.2).numpy()[0]) != 0.2


def test_maximum_nan_and_minimum():
    a = np.array([1.0, np.nan, 3.0, -0.0, 5.0], f32)
    b = np.array([2.0, 1.0, np.nan, 0.0, -5.0], f32)
    mx = ora.maximum(ora.array(a), ora.array(b)).numpy()
    mn = ora.minimum(ora.array(a), ora.array(b)).numpy()
    assert mx[0] == 2 and np.isnan(mx[1]) and np.isnan(mx[2]) and mx[3] == 0 and mx[4] == 5
    assert mn[0] == 1 and np.isnan(mn[1]) and np.isnan(mn[2]) and mn[3] == 0 and mn[4] == -5


# ----------------------------------------------- transcendentals, exact pins --
def _exp_fraction(x: Fraction, terms=60) -> Fraction:
    s, t = Fraction(0), Fraction(1)
    for k in range(terms):
        s += t
        t = t * x / (k + 1)
    return s


def _round_f32(q: Fraction) -> np.float32:
    # nearest binary32 to an exact rational (value well inside the normal range)
    lo = np.float32(float(q))
    cands = [lo, np.nextafter(lo, f32(np.inf)), np.nextafter(lo, f32(-np.inf))]
    return min(cands, key=lambda c: abs(Fraction(float(c)) - q))


@pytest.mark.parametrize("xv", [0.0, 1.0, -1.0, 0.5, -0.3125, 2.75, -7.5, 0.001953125])
def test_exp_is_correctly_rounded_on_exact_rational_series(xv):
    got = ora.exp(ora.array(np.array([xv], f32))).numpy()[0]
    want = _round_f32(_exp_fraction(Fraction(xv)))
    assert got == want


def test_erf_against_high_precision_series():
    from decimal import Decimal, getcontext
    getcontext().prec = 60

    def pi_machin():
        def arctan_inv(n):  # arctan(1/n)
            x = Decimal(1) / n
            s_, t, k = Decimal(0), x, 0
            while abs(t) > Decimal(10) ** -58:
                s_ += t / (2 * k + 1) if k % 2 == 0 else -t / (2 * k + 1)
                t *= x * x
                k += 1
            return s_
        return 16 * arctan_inv(5) - 4 * arctan_inv(239)

    def erf_dec(x):
        x = Decimal(x)
        s_, term, n = Decimal(0), x, 0
        while abs(term) > Decimal(10) ** -55:
            s_ += term / (2 * n + 1)
            n += 1
            term = -term * x * x / n
        return 2 * s_ / pi_machin().sqrt()

    xs = np.array([0.0, 0.125, -0.5, 0.75, 1.0, -1.5, 2.25, 3.0], f32)
    got = ora.erf(ora.array(xs)).numpy()
    for x, g_ in zip(xs, got):
        want = erf_dec(float(x))
        assert abs(Decimal(float(g_)) - want) <= Decimal(float(np.spacing(f32(abs(float(want)))))) * Decimal("0.51") + Decimal(10) ** -45
    assert got[0] == 0 and np.array_equal(ora.erf(ora.array(-xs)).numpy(), -got)          # odd
    big = ora.erf(ora.array(np.array([6.0, -6.0, np.inf], f32))).numpy()
    assert big.tolist() == [1.0, -1.0, 1.0]


def test_blackscholes_limits_and_float64_reference():
    import math
    inp = wl.make_inputs("blackscholes", n=2000)
    got = wl.blackscholes(ora, *(ora.array(inp[k]) for k in ("S", "K", "T"))).numpy()
    S, K, T = (inp[k].astype(np.float64) for k in ("S", "K", "T"))
    r, sig = 0.02, 0.30
    d1 = (np.log(S / K) + (r + 0.5 * sig * sig) * T) / (sig * np.sqrt(T))
    d2 = d1 - sig * np.sqrt(T)
    N = np.vectorize(lambda v: 0.5 * (1 + math.erf(v / math.sqrt(2))))
    want = S * N(d1) - K * np.exp(-r * T) * N(d2)
    assert np.max(np.abs(got - want)) < 2e-5            # prices of order 10, f32 arithmetic
    assert np.all(got >= -1e-5) and np.all(got <= inp["S"] + 1e-5)   # 0 <= call <= S
    # deep in the money: call -> S - K exp(-rT)
    deep = wl.blackscholes(ora, ora.array(np.array([1000.0], f32)), ora.array(np.array([1.0], f32)), ora.array(np.array([1.0], f32))).numpy()
    assert abs(float(deep[0]) - (1000.0 - math.exp(-0.02))) < 1e-3


def test_log_tanh_special_values_and_inverse():
    x = np.array([0.25, 1.0, 3.0, 10.0], f32)
    lg = ora.log(ora.array(x)).numpy()
    assert lg[1] == 0.0
    assert np.all(elementwise_close(ora.exp(ora.array(lg)).numpy(), x, ulps=4))
    th = ora.tanh(ora.array(np.array([0.0, 20.0, -20.0, 0.5], f32))).numpy()
    assert th[0] == 0 and th[1] == 1 and th[2] == -1
    e1, e2 = np.exp(np.float64(0.5)), np.exp(np.float64(-0.5))
    assert abs(float(th[3]) - (e1 - e2) / (e1 + e2)) < 1e-7
    assert np.isnan(ora.log(ora.array(np.array([-1.0], f32))).numpy()[0])
    assert np.isnan(ora.sqrt(ora.array(np.array([-1.0], f32))).numpy()[0])


# ------------------------------------------------------------------- sums ----
@pytest.mark.parametrize("n", [0, 1, 2, 1000, 5793, 70000])
def test_sum_arange_int(n):
    s = ora.sum(ora.array(np.arange(n, dtype=np.int32)))
    assert s.dtype == np.int64 and s.shape == ()
    assert int(s.numpy()) == n * (n - 1) // 2


@pytest.mark.parametrize("n", [1, 17, 4096, 5793])
def test_sum_arange_f32_exact(n):
    s = ora.sum(ora.array(np.arange(n, dtype=f32)))
    assert s.dtype == f32
    assert float(s.numpy()) == n * (n - 1) / 2


def test_sum_accumulates_in_double():
    # 2^24 + 1 + 1 ... : a binary32 accumulator would stall at 2^24.
    x = np.ones(1 << 12, f32)
    x[0] = 2.0**24
    assert float(ora.sum(ora.array(x)).numpy()) == float(f32(2.0**24 + (1 << 12) - 1))


def test_sum_ones_by_axis_and_keepdims():
    x = ora.array(np.ones((3, 4, 5), f32))
    for axis, shape, val in [(0, (4, 5), 3), (1, (3, 5), 4), (2, (3, 4), 5), (-1, (3, 4), 5), ((0, 2), (4,), 15), (None, (), 60)]:
        r = ora.sum(x, axis=axis)
        assert r.shape == shape and np.all(r.numpy() == val)
    assert ora.sum(x, axis=1, keepdims=True).shape == (3, 1, 5)
    assert ora.sum(x, axis=(0, 2), keepdims=True).shape == (1, 4, 1)
    with pytest.raises(ora.OracleError):
        ora.sum(x, axis=3)
    with pytest.raises(ora.OracleError):
        ora.sum(x, axis=(1, 1))


def test_reduce_brute_force_axes():
    g = rng(4)
    x = g.integers(-50, 50, (3, 4, 5)).astype(f32)  # small ints: every order of summation is exact
    X = ora.array(x)
    got = ora.sum(X, axis=1).numpy()
    for i, k in itertools.product(range(3), range(5)):
        assert got[i, k] == sum(float(x[i, j, k]) for j in range(4))
    gmx = ora.max(X, axis=(0, 2)).numpy()
    gmn = ora.min(X, axis=0).numpy()
    for j in range(4):
        assert gmx[j] == max(x[i, j, k] for i in range(3) for k in range(5))
    for j, k in itertools.product(range(4), range(5)):
        assert gmn[j, k] == min(x[i, j, k] for i in range(3))


def test_reduce_empty():
    e = ora.array(np.zeros((0, 3), f32))
    assert np.array_equal(ora.sum(e, axis=0).numpy(), np.zeros(3, f32))
    with pytest.raises(ora.OracleError):
        ora.max(e, axis=0)
    assert ora.max(e, axis=1).shape == (0,)


def test_reduce_max_propagates_nan():
    x = np.array([[1.0, np.nan, 2.0], [1.0, 5.0, 2.0]], f32)
    m = ora.max(ora.array(x), axis=1).numpy()
    assert np.isnan(m[0]) and m[1] == 5


# ------------------------------------------------------------------- scans ---
def test_scan_closed_forms_and_brute_force():
    # cumsum(ones) = 1..n; cumsum(arange) = triangular numbers (exact in f32 for n <= 5793)
    n = 5000
    assert np.array_equal(ora.cumsum(ora.array(np.ones(n, f32)), 0).numpy(), np.arange(1, n + 1, dtype=f32))
    tri = ora.cumsum(ora.array(np.arange(n, dtype=f32)), 0).numpy()
    assert np.array_equal(tri, (np.arange(n, dtype=np.int64) * np.arange(1, n + 1, dtype=np.int64) // 2).astype(f32))
    ti = ora.cumsum(ora.array(np.arange(70000, dtype=np.int32)), 0)
    assert ti.dtype == np.int64
    k = np.arange(70000, dtype=np.int64)
    assert np.array_equal(ti.numpy(), k * (k + 1) // 2)
    # last prefix equals the reduction; differences of prefixes give the terms back (small ints: exact)
    g = rng(20)
    x = g.integers(-9, 10, (4, 5, 6)).astype(f32)
    for axis in (0, 1, 2, -1):
        c = ora.cumsum(ora.array(x), axis).numpy()
        assert c.shape == x.shape
        ax = axis % 3
        assert np.array_equal(np.take(c, -1, axis=ax), ora.sum(ora.array(x), axis=ax).numpy())
        assert np.array_equal(np.diff(c, axis=ax), np.delete(x, 0, axis=ax))
        # brute force against nested Python loops
        for idx in itertools.product(range(4), range(5), range(6)):
            lo = list(idx)
            s = 0.0
            for j in range(idx[ax] + 1):
                lo[ax] = j
                s += float(x[tuple(lo)])
            assert c[idx] == s
    # running extrema against Python's max/min on prefixes, and through a strided view
    y = g.standard_normal((3, 17)).astype(f32)
    cm = ora.cummax(ora.array(y), 1).numpy()
    cn = ora.cummin(ora.array(y)[:, ::2], 1).numpy()
    for i in range(3):
        for j in range(17):
            assert cm[i, j] == max(y[i, :j + 1])
        for j in range(9):
            assert cn[i, j] == min(y[i, :2 * j + 1:2])
    # binary64 accumulation: a binary32 running sum would stall at 2^24
    big = np.ones(1 << 12, f32)
    big[0] = 2.0**24
    assert float(ora.cumsum(ora.array(big), 0).numpy()[-1]) == float(f32(2.0**24 + (1 << 12) - 1))
    with pytest.raises(ora.OracleError):
        ora.cumsum(ora.array(x), 3)
    # NumPy third opinion (NumPy accumulates in binary32, hence a tolerance)
    z = g.standard_normal((7, 300)).astype(f32)
    assert np.allclose(ora.cumsum(ora.array(z), 1).numpy(), np.cumsum(z.astype(np.float64), axis=1), rtol=1e-6, atol=1e-5)
    assert np.array_equal(ora.cummax(ora.array(z), 0).numpy(), np.maximum.accumulate(z, axis=0))


# ------------------------------------------------------------------ slices ---
def test_slice_brute_force_1d_against_python_range():
    n = 6
    x = np.arange(100, 100 + n, dtype=np.int32)
    X = ora.array(x)
    vals = [None] + list(range(-n - 1, n + 2))
    for st, sp, step in itertools.product(vals, vals, (None, 1, 2, 3)):
        want = [int(x[i]) for i in range(n)[st:sp:step]]
        got = X[st:sp:step].numpy()
        assert got.tolist() == want, (st, sp, step)


def test_slice_brute_force_2d():
    x = np.arange(42, dtype=np.int32).reshape(6, 7)
    X = ora.array(x)
    g = rng(5)
    for _ in range(300):
        r0, r1 = int(g.integers(-8, 9)), int(g.integers(-8, 9))
        c0, c1 = int(g.integers(-9, 10)), int(g.integers(-9, 10))
        sr, sc = int(g.integers(1, 4)), int(g.integers(1, 4))
        got = X[r0:r1:sr, c0:c1:sc].numpy()
        rows = list(range(6)[r0:r1:sr])
        cols = list(range(7)[c0:c1:sc])
        assert got.shape == (len(rows), len(cols))
        for i, r in enumerate(rows):
            for j, c in enumerate(cols):
                assert got[i, j] == r * 7 + c
    assert X[1:3].shape == (2, 7)           # trailing dims taken whole
    assert X[2:5][1:, 3:].numpy()[0, 0] == 3 * 7 + 3  # slice of a slice
    with pytest.raises(ora.OracleError):
        X[::-1]
    with pytest.raises(ora.OracleError):
        X[:, :, :]


def test_slice_assignment_aliases_like_numpy():
    x = np.arange(30, dtype=f32).reshape(5, 6)
    X = ora.array(x)
    V = X[1:-1, 2:]                 # view taken before the write
    X[1:-1, 2:] = V * 2.0 + 1.0      # reads the destination itself
    want = x.copy()
    want[1:-1, 2:] = want[1:-1, 2:] * 2 + 1
    assert np.array_equal(X.numpy(), want)
    assert np.array_equal(V.numpy(), want[1:-1, 2:])       # the old view sees the new contents
    # overlapping source and destination: the right-hand side is finished first
    y = np.arange(10, dtype=np.int32)
    Y = ora.array(y)
    Y[1:] = Y[:-1]
    want = y.copy(); want[1:] = y[:-1]
    assert np.array_equal(Y.numpy(), want)
    with pytest.raises(ora.OracleError):
        Y[2:5] = Y[:2]
    # Listing 6: closed form on a constant grid (fixed point) and against NumPy on random data
    const = ora.array(np.full((9, 11), 2.5, f32))
    assert np.all(wl.jacobi(ora, const, 3).numpy() == 2.5)
    g = rng(21)
    grid = g.random((12, 9)).astype(f32)
    got = wl.jacobi(ora, ora.array(grid), 4).numpy()
    ref = grid.copy()
    assert np.array_equal(got, wl.jacobi(np, ref, 4))
    # hand loop for one sweep
    one = wl.jacobi(ora, ora.array(grid), 1).numpy()
    for i in range(1, 11):
        for j in range(1, 8):
            s_ = f32(f32(f32(f32(grid[i, j] + grid[i - 1, j]) + grid[i, j + 1]) + grid[i, j - 1]) + grid[i + 1, j])
            assert one[i, j] == f32(f32(0.2) * s_)
    assert np.array_equal(one[0], grid[0]) and np.array_equal(one[:, -1], grid[:, -1])


def test_ops_read_through_views():
    x = np.arange(30, dtype=f32).reshape(5, 6)
    X = ora.array(x)
    got = (X[1:-1, 2:] - X[:-2, :-2]).numpy()
    for i, j in itertools.product(range(3), range(4)):
        assert got[i, j] == x[i + 1, j + 2] - x[i, j]


# --------------------------------------------------------------- transpose ---
def test_transpose_rule_and_involution():
    x = np.arange(12, dtype=np.int32).reshape(3, 4)
    T = ora.array(x).T
    assert T.shape == (4, 3)
    t = T.numpy()
    for i, j in itertools.product(range(4), range(3)):
        assert t[i, j] == x[j, i]
    assert np.array_equal(T.T.numpy(), x)
    y = np.arange(24, dtype=np.int32).reshape(2, 3, 4)
    p = ora.transpose(ora.array(y), (1, 2, 0))
    assert p.shape == (3, 4, 2)
    pn = p.numpy()
    for i, j, k in itertools.product(range(3), range(4), range(2)):
        assert pn[i, j, k] == y[k, i, j]
    with pytest.raises(ora.OracleError):
        ora.transpose(ora.array(y), (0, 0, 1))


# --------------------------------------------------------------------- dot ---
def test_dot_ones_onehot_and_hand_loop():
    g = rng(6)
    w = g.standard_normal(9).astype(f32)
    ones = np.ones((4, 9), f32)
    z = (ora.array(ones) @ ora.array(w)).numpy()
    exact = float(f32(sum(Fraction(float(v)) for v in w)))  # exactly rounded sum
    assert np.all(z == f32(exact))
    sel = np.zeros((5, 9), f32)
    idx = [3, 0, 8, 8, 2]
    for i, k in enumerate(idx):
        sel[i, k] = 1
    assert np.array_equal((ora.array(sel) @ ora.array(w)).numpy(), w[idx])
    # non-symmetric hand loop, catches a transposed operand
    A = g.integers(-4, 5, (3, 5)).astype(f32)
    v = g.integers(-4, 5, 5).astype(f32)
    got = ora.dot(ora.array(A), ora.array(v)).numpy()
    for i in range(3):
        assert got[i] == sum(float(A[i, k]) * float(v[k]) for k in range(5))
    u = g.integers(-4, 5, 3).astype(f32)
    gotT = (ora.array(A).T @ ora.array(u)).numpy()
    for k in range(5):
        assert gotT[k] == sum(float(A[i, k]) * float(u[i]) for i in range(3))
    B = g.integers(-4, 5, (5, 2)).astype(f32)
    gotM = (ora.array(A) @ ora.array(B)).numpy()
    for i, j in itertools.product(range(3), range(2)):
        assert gotM[i, j] == sum(float(A[i, k]) * float(B[k, j]) for k in range(5))
    with pytest.raises(ora.OracleError):
        ora.array(A) @ ora.array(u)


def test_inner_product_listing5_equals_dot():
    g = rng(7)
    a = g.integers(-8, 9, 301).astype(f32)
    b = g.integers(-8, 9, 301).astype(f32)
    ip = wl.inner_product(ora, ora.array(a), ora.array(b)).numpy()
    d = ora.dot(ora.array(a), ora.array(b)).numpy()
    assert ip.shape == () and d.shape == ()
    assert float(ip) == float(d) == float(sum(int(x) * int(y) for x, y in zip(a, b)))


# ----------------------------------------------------- the five programs ----
def test_chain_equals_hand_written_scalar_loop():
    inp = wl.make_inputs("chain", n=257)
    got = wl.chain(ora, ora.array(inp["a"]), ora.array(inp["b"])).numpy()
    import math
    for i in range(257):
        a, b = f32(inp["a"][i]), f32(inp["b"][i])
        t = f32(f32(f32(a + b) * f32(a - b)) + f32(f32(2.5) * a))
        d = f32(f32(abs(b)) + f32(1.0))
        e = f32(math.exp(float(f32(f32(-a) * a))))
        assert got[i] == f32(f32(t / d) - e)


def test_normalize_against_hand_loop_and_numpy():
    inp = wl.make_inputs("normalize", rows=7, cols=13)
    got = wl.normalize(ora, *(ora.array(inp[k]) for k in ("X", "mu", "sigma", "gamma", "beta"))).numpy()
    for i, j in itertools.product(range(7), range(13)):
        v = f32(f32(f32(f32(inp["X"][i, j] - inp["mu"][0, j]) / inp["sigma"][0, j]) * inp["gamma"][j]) + inp["beta"][j])
        assert got[i, j] == (v if v > 0 else f32(0))
    want = wl.normalize(np, **inp)
    assert want.dtype == f32 and np.array_equal(got, want)


def test_softmax_properties():
    inp = wl.make_inputs("softmax", rows=9, cols=300)
    X = inp["X"]
    out = wl.softmax(ora, ora.array(X)).numpy()
    assert np.all(np.abs(out.astype(np.float64).sum(axis=1) - 1) < 1e-6)
    # the row maximum maps to exp(0)/s = 1/s exactly
    e = np.exp((X - X.max(axis=1, keepdims=True)).astype(np.float64))
    j = X.argmax(axis=1)
    s = out[np.arange(9), j]
    assert np.all(elementwise_close(s, (1.0 / e.sum(axis=1)).astype(f32), ulps=2))
    # shift invariance by an exactly representable per-row constant
    shifted = wl.softmax(ora, ora.array((X.astype(np.float64) * 0 + np.round(X * 4) / 4 + 8).astype(f32))).numpy()
    base = wl.softmax(ora, ora.array((np.round(X * 4) / 4).astype(f32))).numpy()
    assert np.array_equal(shifted, base)
    # equal values -> 1/ncols
    flat = wl.softmax(ora, ora.array(np.full((2, 64), 3.25, f32))).numpy()
    assert np.all(flat == f32(1.0 / 64))


def test_stencil_constant_and_ramp_closed_forms():
    c = f32(37.5)
    out = wl.stencil(ora, ora.array(np.full((9, 11), c, f32))).numpy()
    assert out.shape == (5, 7) and np.all(out == 0)
    # ramp along columns: every five-term sum is an exact integer, B[r,c] = fl(0.2f*(5c+5));
    # vertical differences vanish, so out = |B[., q+2] - B[., q]|.
    R, C = 8, 40
    ramp = np.tile(np.arange(C, dtype=f32), (R, 1))
    out = wl.stencil(ora, ora.array(ramp)).numpy()
    B = np.array([f32(0.2) * f32(5 * c + 5) for c in range(C - 2)], dtype=f32)
    for q in range(C - 4):
        d = f32(B[q + 2] - B[q])
        assert np.all(out[:, q] == f32(np.sqrt(f32(f32(d * d) + f32(0)))))
    outT = wl.stencil(ora, ora.array(np.ascontiguousarray(ramp.T))).numpy()
    assert np.array_equal(outT, out.T)


def test_stencil_brute_force_13_point():
    g = rng(8)
    I = (g.random((7, 8)) * 255).astype(f32)
    out = wl.stencil(ora, ora.array(I)).numpy()
    assert out.shape == (3, 4)

    def B(r, c):  # value of the blurred image at its own index (r, c)
        s = f32(f32(f32(f32(I[r + 1, c + 1] + I[r, c + 1]) + I[r + 2, c + 1]) + I[r + 1, c]) + I[r + 1, c + 2])
        return f32(f32(0.2) * s)

    for p, q in itertools.product(range(3), range(4)):
        dx = f32(B(p + 1, q + 2) - B(p + 1, q))
        dy = f32(B(p + 2, q + 1) - B(p, q + 1))
        assert out[p, q] == f32(np.sqrt(f32(f32(dx * dx) + f32(dy * dy))))


def test_jacobi_sweep_matches_numpy_views():
    g = rng(9)
    grid = g.random((12, 9)).astype(f32)
    got = wl.jacobi_sweep(ora, ora.array(grid)).numpy()
    want = wl.jacobi_sweep(np, grid)
    assert want.dtype == f32 and np.array_equal(got, want)


def test_logreg_zero_weights_closed_form():
    inp = wl.make_inputs("logreg", rows=64, cols=8)
    X, y = inp["X"], inp["y"]
    w0 = np.zeros(8, f32)
    got = wl.logreg(ora, ora.array(X), ora.array(w0), ora.array(y)).numpy()
    # w = 0 -> p = 0.5 exactly, r = 0.5 - y in {+-0.5}; g = X.T r / n; w' = -0.1 g
    r = (0.5 - y).astype(np.float64)
    gT = np.array([f32(sum(float(X[i, k]) * r[i] for i in range(64))) for k in range(8)], dtype=f32)
    want = f32(0) - f32(0.1) * (gT / f32(64) + f32(1e-4) * w0)
    assert np.array_equal(got, want.astype(f32))


def test_logreg_against_float64_reference():
    inp = wl.make_inputs("logreg", rows=500, cols=40)
    got = wl.logreg(ora, *(ora.array(inp[k]) for k in ("X", "w", "y"))).numpy()
    X, w, y = (inp[k].astype(np.float64) for k in ("X", "w", "y"))
    p = 1 / (1 + np.exp(-(X @ w)))
    want = w - 0.1 * ((X.T @ (p - y)) / 500 + 1e-4 * w)
    assert np.max(np.abs(got - want)) < 1e-6


def test_mnist_listing2_against_float64():
    g = rng(10)
    W = g.standard_normal((200, 10)).astype(f32)
    a = g.standard_normal(200).astype(f32)
    b = g.standard_normal(10).astype(f32)
    got = wl.mnist(ora, ora.array(W), ora.array(a), ora.array(b)).numpy()
    x = W.astype(np.float64).T @ np.maximum(a, 0).astype(np.float64) + b
    assert np.max(np.abs(got - 1 / (1 + np.exp(-x)))) < 1e-6


# ------------------------------------------------- NumPy as a third opinion --
def test_numpy_third_opinion_elementwise_bit_exact():
    g = rng(11)
    a = (g.standard_normal((33, 65)) * 10).astype(f32)
    b = (g.standard_normal((65,)) * 10).astype(f32)
    A, B = ora.array(a), ora.array(b)
    assert np.array_equal((A + B).numpy(), a + b)
    assert np.array_equal((A - B).numpy(), a - b)
    assert np.array_equal((A * B).numpy(), a * b)
    assert np.array_equal((A / B).numpy(), a / b)
    assert np.array_equal(abs(A).numpy(), np.abs(a))
    assert np.array_equal((-A).numpy(), -a)
    assert np.array_equal(ora.sqrt(abs(A)).numpy(), np.sqrt(np.abs(a)))
    assert np.array_equal(ora.maximum(A, B).numpy(), np.maximum(a, b))
    assert np.array_equal(ora.minimum(A, B).numpy(), np.minimum(a, b))
    assert np.array_equal((A ** 2).numpy(), a ** 2)
    assert np.all(elementwise_close(ora.exp(A / 10.0).numpy(), np.exp(a / f32(10)), ulps=2))
    assert np.all(elementwise_close(ora.tanh(A / 10.0).numpy(), np.tanh(a / f32(10)), ulps=2))
    assert np.all(elementwise_close(ora.log(abs(A) + 1.0).numpy(), np.log(np.abs(a) + f32(1)), ulps=2))
    i = g.integers(-2**31, 2**31 - 1, (7, 9), dtype=np.int64).astype(np.int32)
    j = g.integers(-2**31, 2**31 - 1, (9,), dtype=np.int64).astype(np.int32)
    with np.errstate(over="ignore"):
        assert np.array_equal((ora.array(i) * ora.array(j) - ora.array(i)).numpy(), i * j - i)
        assert np.array_equal((ora.array(i) * 3 + 1).numpy(), i * np.int32(3) + np.int32(1))


def test_numpy_third_opinion_reductions_and_programs():
    g = rng(12)
    x = g.standard_normal((37, 211)).astype(f32)
    X = ora.array(x)
    assert np.allclose(ora.sum(X, axis=1).numpy(), x.sum(axis=1, dtype=np.float64), rtol=1e-6, atol=1e-6)
    assert np.array_equal(ora.max(X, axis=0).numpy(), x.max(axis=0))
    assert np.array_equal(ora.min(X, axis=1, keepdims=True).numpy(), x.min(axis=1, keepdims=True))
    for name in ("chain", "softmax", "stencil"):
        inp = wl.make_inputs(name, **wl.SMALL[name]) if name != "chain" else wl.make_inputs(name, n=4099)
        if name == "softmax":
            inp = wl.make_inputs(name, rows=11, cols=257)
        if name == "stencil":
            inp = wl.make_inputs(name, rows=23, cols=41)
        got = wl.PROGRAMS[name](ora, **{k: ora.array(v) for k, v in inp.items()}).numpy()
        want = wl.PROGRAMS[name](np, **inp)
        assert want.dtype == f32
        tol = dict(ulps=4, rel=2e-6)
        floor = 4 * ulp_of(np.ones(1, f32)) if name == "chain" else None  # final op subtracts two O(1) values
        assert np.all(elementwise_close(got, want, floor=floor, **tol)), name


# ------------------------------------------------------------- threading ----
def test_threads_do_not_change_results():
    inp = wl.make_inputs("softmax", rows=40, cols=123)
    ora.set_threads(1)
    one = wl.softmax(ora, ora.array(inp["X"])).numpy()
    ora.set_threads(4)
    try:
        four = wl.softmax(ora, ora.array(inp["X"])).numpy()
    finally:
        ora.set_threads(1)
    assert np.array_equal(one, four)


# ---- reshape ---------------------------------------------------------------------------------

def test_reshape_is_row_major_relabelling():
    # brute force: element number `lin` in row-major order keeps its number under the new shape
    g = np.random.default_rng(77)
    x = g.standard_normal((4, 6, 5)).astype(f32)
    for shape in [(120,), (6, 20), (2, 3, 4, 5), (5, -1), (-1,), (1, 120, 1)]:
        got = ora.array(x).reshape(*shape).numpy()
        want = tuple(120 // 5 if v == -1 and len(shape) == 2 else (120 if v == -1 else v) for v in shape)
        assert got.shape == want
        flat_src = [x[i, j, k] for i in range(4) for j in range(6) for k in range(5)]
        assert got.ravel().tolist() == flat_src
    # a transposed, stepped view is read in ITS row-major order
    v = ora.array(x).T[::2, 1:, :]
    src = x.T[::2, 1:, :]
    got = v.reshape(-1).numpy()
    assert got.tolist() == [src[i, j, k] for i in range(src.shape[0]) for j in range(src.shape[1]) for k in range(src.shape[2])]
    assert np.array_equal(ora.array(x).T.reshape(10, 12).numpy(), x.T.reshape(10, 12))       # NumPy as third opinion
    i = np.arange(24, dtype=np.int32).reshape(2, 12)
    assert np.array_equal(ora.array(i).reshape(4, 6).numpy(), i.reshape(4, 6))
    # a copy: writing through the result leaves the operand alone
    a = ora.array(x)
    r = a.reshape(6, 20)
    r[0:1] = ora.array(np.zeros((1, 20), f32))
    assert np.array_equal(a.numpy(), x)
    for bad in [(7, 17), (-1, -1), (0, -1), (-2, 60)]:
        with pytest.raises(Exception):
            ora.array(x).reshape(*bad)
    assert ora.array(np.zeros((0, 4), f32)).reshape(4, 0).numpy().shape == (4, 0)


# ---- random programs against NumPy ---------------------------------------------------------

def test_random_programs_match_numpy_bit_for_bit():
    # every op of a recipe rounds once, so the evaluator and NumPy (a library routine per op, the
    # special case the evaluator reduces to) must agree in every bit of every intermediate;
    # only the sign of a zero returned by maximum/minimum on equal operands is left open
    import warnings
    import fuzz
    checked = 0
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")          # NumPy warns about float overflow; inf is the expected value
        for seed in range(400):
            dtype, shapes, steps, res = fuzz.make_recipe(seed)
            leaves = fuzz.make_leaves(seed, dtype, shapes)
            ref = fuzz.apply(fuzz.NumpyModule, steps, leaves)
            got = fuzz.apply(ora, steps, [ora.array(x) for x in leaves])
            for i, (g, r) in enumerate(zip(got, ref)):
                assert fuzz.same_bits(g.numpy(), r, zero_signs=False), (seed, i, steps)
                checked += 1
    assert checked > 2000


def test_random_programs_with_reshapes_match_numpy():
    import warnings
    import fuzz
    n = 0
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        for seed in range(400000, 400300):
            dtype, shapes, steps, res = fuzz.make_recipe(seed, reshape=True, assign=(seed % 2 == 0))
            n += sum(1 for st in steps if st[0] == "reshape")
            leaves = fuzz.make_leaves(seed, dtype, shapes)
            ref = fuzz.apply(fuzz.NumpyModule, steps, [x.copy() for x in leaves])
            got = fuzz.apply(ora, steps, [ora.array(x.copy()) for x in leaves])
            for i, (g, r) in enumerate(zip(got, ref)):
                assert fuzz.same_bits(g.numpy(), r, zero_signs=False), (seed, i, steps)
    assert n > 100


def test_random_programs_with_slice_assignments_match_numpy():
    # the same with writes through views: overlapping sources, values that were computed before a
    # write, views that must show it (NumPy's eager semantics are the definition)
    import warnings
    import fuzz
    assigns = 0
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        for seed in range(5000, 5300):
            dtype, shapes, steps, res = fuzz.make_recipe(seed, assign=True)
            assigns += sum(1 for st in steps if st[0] == "assign")
            leaves = fuzz.make_leaves(seed, dtype, shapes)
            ref = fuzz.apply(fuzz.NumpyModule, steps, [x.copy() for x in leaves])
            got = fuzz.apply(ora, steps, [ora.array(x.copy()) for x in leaves])
            for i, (g, r) in enumerate(zip(got, ref)):
                assert fuzz.same_bits(g.numpy(), r, zero_signs=False), (seed, i, steps)
    assert assigns > 200


def test_random_programs_assigning_into_evaluated_values_match_numpy():
    # writes into arrays that are results of earlier operations (evaluated first), among them values that an
    # earlier assignment stored into another array: each is an array of its own, as in NumPy
    import warnings
    import fuzz
    into_values = 0
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        for seed in range(800000, 800400):
            dtype, shapes, steps, res = fuzz.make_recipe(seed, max_steps=14, assign=True, assign_values=True, reshape=(seed % 3 == 0))
            into_values += sum(1 for st in steps if st[0] == "assign" and st[1] >= len(shapes))
            leaves = fuzz.make_leaves(seed, dtype, shapes)
            ref = fuzz.apply(fuzz.NumpyModule, steps, [x.copy() for x in leaves])
            got = fuzz.apply(ora, steps, [ora.array(x.copy()) for x in leaves])
            for i, (g, r) in enumerate(zip(got, ref)):
                assert fuzz.same_bits(g.numpy(), r, zero_signs=False), (seed, i, steps)
    assert into_values > 50


def test_mean_is_the_sum_divided_by_the_number_of_terms():
    # closed forms (exact: every partial sum is a small integer or a dyadic fraction), NumPy in binary64
    # as the third opinion, and the decomposition over two axes
    f32 = np.float32
    for n in (1, 2, 7, 1000, 4097):
        assert ora.mean(ora.array(np.arange(n, dtype=f32))).numpy() == f32((n - 1) / 2)
    c = np.full((64, 32), 0.375, f32)
    assert np.array_equal(ora.mean(ora.array(c), axis=0).numpy(), np.full(32, 0.375, f32))
    assert np.array_equal(ora.mean(ora.array(c), axis=1, keepdims=True).numpy(), np.full((64, 1), 0.375, f32))
    x = np.random.default_rng(11).standard_normal((37, 50, 6)).astype(f32)
    for axis, keep in [(None, False), (0, True), (1, False), (-1, False), ((0, 2), True), ((0, 1, 2), False)]:
        got = ora.mean(ora.array(x), axis=axis, keepdims=keep).numpy()
        ref = np.mean(x.astype(np.float64), axis=axis, keepdims=keep)
        assert got.shape == ref.shape and got.dtype == f32
        assert np.all(np.abs(got - ref) <= 1e-6 * np.abs(ref) + 1e-7), axis
    rows = ora.mean(ora.array(x[:, :, 0]), axis=1).numpy()
    assert abs(float(ora.mean(ora.array(rows)).numpy()) - float(ora.mean(ora.array(x[:, :, 0])).numpy())) < 1e-6
    assert ora.array(x).mean(axis=1).shape == (37, 6)


def test_var_std_and_clip_follow_their_definitions():
    # variance: closed form for 0..n-1 ((n^2 - 1) / 12, every intermediate exact for small n), shift invariance,
    # NumPy in binary64; clip: bounds reached exactly, order of the two bounds as NumPy applies them
    f32 = np.float32
    for n in (2, 5, 9, 33):
        got = float(ora.var(ora.array(np.arange(n, dtype=f32))).numpy())
        assert abs(got - (n * n - 1) / 12.0) <= 1e-6 * (n * n) / 12.0
    x = np.random.default_rng(12).standard_normal((41, 30)).astype(f32)
    for axis, keep in [(None, False), (0, True), (1, False), ((0, 1), False)]:
        for name in ("var", "std"):
            got = getattr(ora, name)(ora.array(x), axis=axis, keepdims=keep).numpy()
            ref = getattr(np, name)(x.astype(np.float64), axis=axis, keepdims=keep)
            assert got.shape == ref.shape and np.all(np.abs(got - ref) <= 2e-6 * np.abs(ref)), (name, axis)
    shifted = ora.var(ora.array(x + f32(8)), axis=1).numpy()
    assert np.all(np.abs(shifted - ora.var(ora.array(x), axis=1).numpy()) <= 1e-4)
    assert float(ora.var(ora.array(np.full(17, 3.5, f32))).numpy()) == 0.0
    c = ora.clip(ora.array(x), -0.5, 0.25).numpy()
    assert np.array_equal(c, np.clip(x, f32(-0.5), f32(0.25))) and c.max() == f32(0.25) and c.min() == f32(-0.5)
    assert np.array_equal(ora.clip(ora.array(x), 1.0, -1.0).numpy(), np.clip(x, f32(1.0), f32(-1.0)))   # lo > hi: everything becomes hi
