"""ORACLE -- test infrastructure only.

Python face of the eager CPU evaluator in ``eager.cpp``: an ``Array`` class
with NumPy-like operators so that a NumPy-style program (Section 1, Listing 1
of the paper) runs op by op, one materialised host array per operation.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the GPU
library and the GPU library imports nothing from here.
"""
from __future__ import annotations

import builtins
import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_eager.so")
_SRC = os.path.join(_HERE, "eager.cpp")

_DT = {np.dtype(np.float32): 0, np.dtype(np.int32): 1, np.dtype(np.int64): 2}
_NP = {0: np.float32, 1: np.int32, 2: np.int64}
_UNARY = {"neg": 0, "abs": 1, "exp": 2, "log": 3, "sqrt": 4, "square": 5, "tanh": 6, "erf": 7}
_BINARY = {"add": 0, "sub": 1, "mul": 2, "div": 3, "maximum": 4, "minimum": 5}
_REDUCE = {"sum": 0, "max": 1, "min": 2}


class OracleError(Exception):
    pass


def build() -> str:
    """Compile eager.cpp (plain g++, no fast-math, no FMA contraction)."""
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-o", _SO, _SRC]
    subprocess.check_call(cmd)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
            build()
        L = ctypes.CDLL(_SO)
        P, I, D = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        L.ora_last_error.restype = ctypes.c_char_p
        L.ora_from_host.restype = P
        L.ora_from_host.argtypes = [P, I, I, P]
        L.ora_scalar.restype = P
        L.ora_scalar.argtypes = [D, I]
        L.ora_free.argtypes = [P]
        L.ora_ndim.argtypes = [P]
        L.ora_dtype.argtypes = [P]
        L.ora_shape.argtypes = [P, P]
        L.ora_copy_out.argtypes = [P, P]
        L.ora_unary.restype = P
        L.ora_unary.argtypes = [I, P]
        L.ora_binary.restype = P
        L.ora_binary.argtypes = [I, P, P]
        L.ora_slice.restype = P
        L.ora_slice.argtypes = [P, I, P, P, P, P, P]
        L.ora_transpose.restype = P
        L.ora_transpose.argtypes = [P, P]
        L.ora_reshape.restype = P
        L.ora_reshape.argtypes = [P, I, P]
        L.ora_reduce.restype = P
        L.ora_reduce.argtypes = [I, P, P, I, I]
        L.ora_dot.restype = P
        L.ora_dot.argtypes = [P, P]
        L.ora_scan.restype = P
        L.ora_scan.argtypes = [I, P, I]
        L.ora_assign.restype = I
        L.ora_assign.argtypes = [P, P]
        L.ora_set_threads.argtypes = [I]
        _lib = L
    return _lib


def set_threads(n: int) -> None:
    lib().ora_set_threads(int(n))


def get_threads() -> int:
    return int(lib().ora_get_threads())


def _check(ptr):
    if not ptr:
        raise OracleError(lib().ora_last_error().decode())
    return ptr


class Array:
    """One eagerly computed host array (or a view of one)."""

    __array_priority__ = 1000

    def __init__(self, ptr):
        self._p = ctypes.c_void_p(_check(ptr))

    def __del__(self):
        try:
            lib().ora_free(self._p)
        except Exception:
            pass

    # -- inspection ---------------------------------------------------------
    @property
    def shape(self):
        n = lib().ora_ndim(self._p)
        s = (ctypes.c_int64 * builtins.max(n, 1))()
        lib().ora_shape(self._p, s)
        return tuple(int(s[i]) for i in range(n))

    @property
    def ndim(self):
        return int(lib().ora_ndim(self._p))

    @property
    def dtype(self):
        return np.dtype(_NP[lib().ora_dtype(self._p)])

    def numpy(self) -> np.ndarray:
        out = np.empty(self.shape, dtype=self.dtype)
        lib().ora_copy_out(self._p, out.ctypes.data_as(ctypes.c_void_p))
        return out

    # -- operators ----------------------------------------------------------
    def __add__(self, o): return binary("add", self, o)
    def __radd__(self, o): return binary("add", o, self)
    def __sub__(self, o): return binary("sub", self, o)
    def __rsub__(self, o): return binary("sub", o, self)
    def __mul__(self, o): return binary("mul", self, o)
    def __rmul__(self, o): return binary("mul", o, self)
    def __truediv__(self, o): return binary("div", self, o)
    def __rtruediv__(self, o): return binary("div", o, self)
    def __neg__(self): return unary("neg", self)
    def __abs__(self): return unary("abs", self)
    def __matmul__(self, o): return dot(self, o)

    def __pow__(self, e):
        if e == 2:
            return unary("square", self)
        raise OracleError("only **2 is supported")

    def __getitem__(self, key):
        return slice_(self, key)

    def __setitem__(self, key, value):
        dst = slice_(self, key)
        if lib().ora_assign(dst._p, _operand(value)._p):
            raise OracleError(lib().ora_last_error().decode())

    @property
    def T(self):
        return transpose(self)

    def reshape(self, *shape):
        return reshape(self, shape[0] if len(shape) == 1 and not isinstance(shape[0], int) else shape)

    def mean(self, axis=None, keepdims=False): return mean(self, axis, keepdims)
    def sum(self, axis=None, keepdims=False): return reduce("sum", self, axis, keepdims)
    def max(self, axis=None, keepdims=False): return reduce("max", self, axis, keepdims)
    def min(self, axis=None, keepdims=False): return reduce("min", self, axis, keepdims)
    def dot(self, o): return dot(self, o)
    def cumsum(self, axis=None): return cumsum(self, axis)


def array(x) -> Array:
    a = np.ascontiguousarray(x)
    if a.dtype not in _DT:
        raise OracleError(f"unsupported dtype {a.dtype}")
    shape = (ctypes.c_int64 * builtins.max(a.ndim, 1))(*a.shape)
    return Array(lib().ora_from_host(a.ctypes.data_as(ctypes.c_void_p), _DT[a.dtype], a.ndim, shape))


def _operand(x):
    """Arrays pass through; Python numbers become weak scalars."""
    if isinstance(x, Array):
        return x
    if isinstance(x, (bool, np.bool_)):
        raise OracleError("bool scalars are not supported")
    if isinstance(x, (int, np.integer)):
        return Array(lib().ora_scalar(float(int(x)), 1))
    if isinstance(x, (float, np.floating)):
        return Array(lib().ora_scalar(float(x), 0))
    if isinstance(x, np.ndarray):
        return array(x)
    raise OracleError(f"unsupported operand {type(x)}")


def unary(name: str, a) -> Array:
    a = _operand(a)
    return Array(lib().ora_unary(_UNARY[name], a._p))


def binary(name: str, a, b) -> Array:
    a, b = _operand(a), _operand(b)
    return Array(lib().ora_binary(_BINARY[name], a._p, b._p))


def slice_(a: Array, key) -> Array:
    if not isinstance(key, tuple):
        key = (key,)
    n = len(key)
    I64, U8 = ctypes.c_int64 * builtins.max(n, 1), ctypes.c_uint8 * builtins.max(n, 1)
    start, stop, step, hs, he = I64(), I64(), I64(), U8(), U8()
    for d, k in enumerate(key):
        if not isinstance(k, slice):
            raise OracleError("only slice objects are supported as indices")
        step[d] = 1 if k.step is None else int(k.step)
        hs[d] = k.start is not None
        he[d] = k.stop is not None
        start[d] = 0 if k.start is None else int(k.start)
        stop[d] = 0 if k.stop is None else int(k.stop)
    return Array(lib().ora_slice(a._p, n, start, stop, step, hs, he))


def transpose(a: Array, perm: Optional[Sequence[int]] = None) -> Array:
    p = None if perm is None else (ctypes.c_int * len(perm))(*perm)
    return Array(lib().ora_transpose(a._p, p))


def reshape(a: Array, shape) -> Array:
    """Row-major reshape; always a copy (Section 2 of the paper lists reshape among the operations)."""
    shape = [int(shape)] if isinstance(shape, int) else [int(v) for v in shape]
    arr = (ctypes.c_int64 * builtins.max(len(shape), 1))(*shape)
    return Array(_check(lib().ora_reshape(a._p, len(shape), arr)))


def reduce(name: str, a: Array, axis=None, keepdims=False) -> Array:
    if axis is None:
        axes = []
    elif isinstance(axis, int):
        axes = [axis]
    else:
        axes = list(axis)
        if not axes:
            raise OracleError("empty axis tuple")
    arr = (ctypes.c_int * builtins.max(len(axes), 1))(*axes)
    return Array(lib().ora_reduce(_REDUCE[name], a._p, arr, len(axes), int(bool(keepdims))))


def scan(name: str, a: Array, axis: int) -> Array:
    return Array(lib().ora_scan(_REDUCE[name], a._p, int(axis)))


def _scan_axis(name, a, axis):
    # axis=None: NumPy's scan over the flattened array
    return scan(name, reshape(a, (-1,)), 0) if axis is None else scan(name, a, axis)


def cumsum(a, axis=None): return _scan_axis("sum", a, axis)
def cummax(a, axis=None): return _scan_axis("max", a, axis)
def cummin(a, axis=None): return _scan_axis("min", a, axis)


def dot(a: Array, b: Array) -> Array:
    return Array(lib().ora_dot(_operand(a)._p, _operand(b)._p))


# NumPy-style free functions, so a program can be written against a module.
def add(a, b): return binary("add", a, b)
def subtract(a, b): return binary("sub", a, b)
def multiply(a, b): return binary("mul", a, b)
def divide(a, b): return binary("div", a, b)
def maximum(a, b): return binary("maximum", a, b)
def minimum(a, b): return binary("minimum", a, b)
def negative(a): return unary("neg", a)
def absolute(a): return unary("abs", a)
def exp(a): return unary("exp", a)
def log(a): return unary("log", a)
def sqrt(a): return unary("sqrt", a)
def square(a): return unary("square", a)
def tanh(a): return unary("tanh", a)
def erf(a): return unary("erf", a)
def sum(a, axis=None, keepdims=False): return reduce("sum", a, axis, keepdims)  # noqa: A001


def mean(a, axis=None, keepdims=False):
    """Arithmetic mean over the given axes of a float32 array: the sum (accumulated in binary64 and
    rounded once, as `sum` is) divided by the number of terms in one binary32 division."""
    shape = a.shape
    dims = range(len(shape)) if axis is None else ([axis] if isinstance(axis, int) else list(axis))
    terms = 1
    for d in dims:
        terms *= shape[d]
    return reduce("sum", a, axis, keepdims) / float(terms)


def var(a, axis=None, keepdims=False):
    """Population variance (NumPy's default, ddof = 0): the mean of the squared deviations from the
    mean, in two passes as NumPy computes it."""
    d = a - mean(a, axis, True)
    return mean(d * d, axis, keepdims)


def std(a, axis=None, keepdims=False):
    """Square root of the population variance."""
    return sqrt(var(a, axis, keepdims))


def clip(a, lo, hi):
    """NumPy's clip with two bounds: minimum(maximum(a, lo), hi)."""
    return minimum(maximum(a, lo), hi)
def max(a, axis=None, keepdims=False): return reduce("max", a, axis, keepdims)  # noqa: A001
def min(a, axis=None, keepdims=False): return reduce("min", a, axis, keepdims)  # noqa: A001
