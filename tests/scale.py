"""Cancellation scales for the reduction tolerance, computed by the CPU oracle.

A float32 sum of n terms carries an error of order (rounding unit) x sum|terms|,
so "1e-5 relative" is a per-element bar only while the terms do not cancel.
Where they do (a dot product of signed values, a sum that lands near zero) the
bar is stated against sum|terms| instead.  This module runs a NumPy-style
program a second time on the oracle, op by op, carrying beside every value v
a magnitude M >= |v|:

    leaf, scalar          M = |v|
    a + b, a - b          M = M_a + M_b
    a * b                 M = M_a * M_b
    a / b                 M = (M_a + |a / b| * (M_b - |b|)) / |b|
    neg, abs              M = M_a
    square                M = M_a * M_a
    f(a) (exp log sqrt    M = |f(a)| + |f'(a)| * (M_a - |a|)   (first order: only the
          tanh erf)                                              excess of M_a over |a| is amplified)
    maximum, minimum      M = maximum(M_a, M_b)
    sum, dot, cumsum      the same operation applied to the magnitudes
    max, min, cummax ...  max of the magnitudes
    views, reshape        applied to both

so M is what the program would yield if no addition ever cancelled; with
positive terms throughout M = |v| and the scaled bar equals the per-element
one.  No expected value comes from here: only the width of the band around the
oracle's value where the per-element bar does not apply.
"""
import math

import numpy as np

import oracle as ora


def _is_num(x):
    return isinstance(x, (int, float, np.integer, np.floating))


class Tracked:
    """A value of the oracle and the magnitude that bounds it."""

    __array_priority__ = 2000

    def __init__(self, v, m):
        self.v, self.m = v, m

    @property
    def shape(self):
        return self.v.shape

    @property
    def ndim(self):
        return self.v.ndim

    # -- operators ----------------------------------------------------------
    def __add__(self, o): return _addsub("add", self, o)
    def __radd__(self, o): return _addsub("add", o, self)
    def __sub__(self, o): return _addsub("sub", self, o)
    def __rsub__(self, o): return _addsub("sub", o, self)
    def __mul__(self, o): return _mul(self, o)
    def __rmul__(self, o): return _mul(o, self)
    def __truediv__(self, o): return _div(self, o)
    def __rtruediv__(self, o): return _div(o, self)
    def __neg__(self): return Tracked(-self.v, self.m)
    def __abs__(self): return Tracked(abs(self.v), self.m)
    def __matmul__(self, o): return dot(self, o)

    def __pow__(self, e):
        assert e == 2
        return square(self)

    def __getitem__(self, key):
        return Tracked(self.v[key], self.m[key])

    @property
    def T(self):
        return Tracked(self.v.T, self.m.T)

    def reshape(self, *shape):
        return Tracked(self.v.reshape(*shape), self.m.reshape(*shape))

    def sum(self, axis=None, keepdims=False): return sum(self, axis, keepdims)
    def max(self, axis=None, keepdims=False): return max(self, axis, keepdims)
    def min(self, axis=None, keepdims=False): return min(self, axis, keepdims)
    def mean(self, axis=None, keepdims=False): return mean(self, axis, keepdims)
    def dot(self, o): return dot(self, o)
    def cumsum(self, axis=None): return cumsum(self, axis)


def _pair(x):
    """(value, magnitude) of an operand; Python numbers stay Python numbers."""
    if isinstance(x, Tracked):
        return x.v, x.m
    if _is_num(x):
        return x, type(x)(abs(x))
    raise TypeError(type(x))


def _addsub(name, a, b):
    (av, am), (bv, bm) = _pair(a), _pair(b)
    return Tracked(ora.binary(name, av, bv), ora.binary("add", am, bm))


def _mul(a, b):
    (av, am), (bv, bm) = _pair(a), _pair(b)
    return Tracked(ora.binary("mul", av, bv), ora.binary("mul", am, bm))


def _div(a, b):
    (av, am), (bv, bm) = _pair(a), _pair(b)
    q = ora.binary("div", av, bv)
    absb = abs(bv) if not _is_num(bv) else abs(bv)
    excess_b = ora.binary("sub", bm, absb) if not (_is_num(bm) and _is_num(absb)) else bm - absb
    m = ora.binary("div", ora.binary("add", am, ora.binary("mul", abs(q), excess_b)), absb)
    return Tracked(q, m)


def _first_order(fv, dabs, a):
    """|f(a)| + |f'(a)| * (M_a - |a|)."""
    return abs(fv) + dabs * (a.m - abs(a.v))


def exp(a):
    fv = ora.exp(a.v)
    return Tracked(fv, _first_order(fv, fv, a))


def log(a):
    fv = ora.log(a.v)
    return Tracked(fv, _first_order(fv, 1.0 / abs(a.v), a))


def sqrt(a):
    fv = ora.sqrt(a.v)
    return Tracked(fv, _first_order(fv, 0.5 / fv, a))


def tanh(a):
    fv = ora.tanh(a.v)
    return Tracked(fv, _first_order(fv, 1.0 - fv * fv, a))


def erf(a):
    fv = ora.erf(a.v)
    return Tracked(fv, _first_order(fv, (2.0 / math.sqrt(math.pi)) * ora.exp(-(a.v * a.v)), a))


def square(a): return Tracked(ora.square(a.v), a.m * a.m)
def negative(a): return -a
def absolute(a): return abs(a)
def add(a, b): return _addsub("add", a, b)
def subtract(a, b): return _addsub("sub", a, b)
def multiply(a, b): return _mul(a, b)
def divide(a, b): return _div(a, b)


def maximum(a, b):
    (av, am), (bv, bm) = _pair(a), _pair(b)
    return Tracked(ora.maximum(av, bv), ora.maximum(am, bm))


def minimum(a, b):
    (av, am), (bv, bm) = _pair(a), _pair(b)
    return Tracked(ora.minimum(av, bv), ora.maximum(am, bm))


def sum(a, axis=None, keepdims=False):  # noqa: A001
    return Tracked(ora.sum(a.v, axis, keepdims), ora.sum(a.m, axis, keepdims))


def max(a, axis=None, keepdims=False):  # noqa: A001
    return Tracked(ora.max(a.v, axis, keepdims), ora.max(a.m, axis, keepdims))


def min(a, axis=None, keepdims=False):  # noqa: A001
    return Tracked(ora.min(a.v, axis, keepdims), ora.max(a.m, axis, keepdims))


def mean(a, axis=None, keepdims=False):
    return Tracked(ora.mean(a.v, axis, keepdims), ora.mean(a.m, axis, keepdims))


def var(a, axis=None, keepdims=False):
    d = a - mean(a, axis, True)
    return mean(d * d, axis, keepdims)


def std(a, axis=None, keepdims=False):
    return sqrt(var(a, axis, keepdims))


def clip(a, lo, hi):
    return minimum(maximum(a, lo), hi)


def cumsum(a, axis=None): return Tracked(ora.cumsum(a.v, axis), ora.cumsum(a.m, axis))
def cummax(a, axis=None): return Tracked(ora.cummax(a.v, axis), ora.cummax(a.m, axis))
def cummin(a, axis=None): return Tracked(ora.cummin(a.v, axis), ora.cummax(a.m, axis))


def dot(a, b):
    return Tracked(ora.dot(a.v, b.v), ora.dot(a.m, b.m))


def transpose(a, perm=None):
    return Tracked(ora.transpose(a.v, perm), ora.transpose(a.m, perm))


def reshape(a, shape):
    return Tracked(ora.reshape(a.v, shape), ora.reshape(a.m, shape))


def leaf(x):
    x = np.ascontiguousarray(x)
    return Tracked(ora.array(x), ora.array(np.abs(x)))


def of(program, arrays):
    """Runs `program(xp, **arrays)` with tracked operands; returns (oracle value, magnitude) as NumPy arrays."""
    import sys
    out = program(sys.modules[__name__], **{k: leaf(v) for k, v in arrays.items()})
    return out.v.numpy(), out.m.numpy().astype(np.float64)
