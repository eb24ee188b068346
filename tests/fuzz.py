"""Seeded random array programs for differential tests.

A recipe is a list of steps over a pool of arrays: exactly rounded pointwise
ops (+ - * / neg abs square sqrt maximum minimum) with NumPy broadcasting and
Python scalars, slices with steps, transpositions, max/min reductions over
random axes, running max/min, and - for int32 programs - wrap-around sums and
prefix sums.  Every op in a recipe rounds once (or not at all), so any two
correct evaluators agree bit for bit, whatever they fuse: the GPU library is
compared with the CPU evaluator exactly, and the CPU evaluator with NumPy.

Shapes are tracked here by hand-written NumPy rules (no array library is
called while a recipe is built); `apply` runs a recipe on any array module
with NumPy's names.
"""
from __future__ import annotations

import random

import numpy as np

DIMS = [1, 1, 2, 3, 5, 7, 16, 33, 64, 130]
BIG_DIMS = [1, 2, 3, 5, 17, 130, 257, 1030, 2051, 4100]   # several tiles of every kernel, ragged tails


def _broadcast(a, b):
    n = max(len(a), len(b))
    a2, b2 = (1,) * (n - len(a)) + tuple(a), (1,) * (n - len(b)) + tuple(b)
    out = []
    for x, y in zip(a2, b2):
        if x != y and x != 1 and y != 1:
            return None
        out.append(max(x, y))
    return tuple(out)


def make_recipe(seed: int, max_steps: int = 10, assign: bool = False, big: bool = False, empty: bool = False,
                reshape: bool = False, assign_values: bool = False):
    """Returns (dtype, leaf_shapes, steps, result_index); steps are tuples whose first entry names the op.
    assign=True adds slice assignments into leaves and views of leaves (values: an array of the same
    shape, an expression of the destination itself, or a shifted and possibly overlapping view)."""
    r = random.Random(seed)
    dtype = "i32" if r.random() < 0.3 else "f32"
    nleaf = r.randint(1, 3)
    rank = r.randint(1, 4)
    dims, limit = (BIG_DIMS, 3_000_000) if big else (DIMS, 60000)
    base = [r.choice(dims) for _ in range(rank)]
    while int(np.prod(base)) > limit:
        base[r.randrange(rank)] = r.choice(dims[:6])
    leaf_shapes = [tuple(base)]
    for _ in range(nleaf - 1):
        # a broadcast-compatible partner: trailing dims of the base, some replaced by 1
        k = r.randint(0, rank)
        s = [d if r.random() < 0.7 else 1 for d in base[rank - k:]] if k else []
        leaf_shapes.append(tuple(s) if s else (1,))
    shapes = list(leaf_shapes)      # pool shapes
    final = [False] * len(shapes)   # i64 results cannot feed further ops
    storage = [True] * len(shapes)  # leaves and views of leaves: valid destinations of an assignment
    computed = [False] * len(shapes)  # results of operations (not leaves, not views)
    steps = []

    def pick(pred=lambda i: True):
        c = [i for i in range(len(shapes)) if not final[i] and pred(i)]
        return r.choice(c) if c else None

    nsteps = r.randint(3, max_steps)
    for _ in range(nsteps):
        kind = r.choices(["unary", "binary", "scalar", "slice", "transpose", "reduce", "scan", "materialize", "assign", "reshape"],
                         weights=[3, 6, 3, 3, 2, 2, 1, 1, 3 if assign else 0, 3 if reshape else 0])[0]
        if kind == "assign":
            t = r.choice([i for i in range(len(shapes)) if storage[i]])
            st_ = shapes[t]
            key, key2, out = [], [], []
            for d in st_:
                n = r.randint(1, d)                       # extent of the destination along this dimension
                step = r.choice([1, 1, 2]) if (n - 1) * 2 < d else 1
                span = (n - 1) * step + 1
                lo = r.randint(0, d - span)
                lo2 = r.randint(0, d - span)
                key.append((lo, lo + span, step))
                key2.append((lo2, lo2 + span, step))
                out.append(n)
            same = [i for i in range(len(shapes)) if not final[i] and shapes[i] == tuple(out)]
            mode = r.choice(["self", "shift", "shiftexpr"] + (["pool"] * 2 if same else []))
            steps.append(("assign", t, tuple(key), mode, r.choice(same) if mode == "pool" else tuple(key2)))
            continue
        a = pick()
        if a is None:
            break
        sa = shapes[a]
        if len(sa) == 0 and kind in ("slice", "transpose", "reduce", "scan"):
            kind = "unary"
        if 0 in sa and kind == "reduce" and dtype != "i32":
            kind = "unary"                                  # max/min of nothing is an error; an empty i32 sum is 0
        if kind == "reshape":
            # flatten, merge two neighbouring dimensions, or split one by a divisor
            new = list(sa)
            how = r.choice(["flat", "merge", "split"])
            if how == "merge" and len(sa) >= 2:
                i = r.randrange(len(sa) - 1)
                new = list(sa[:i]) + [sa[i] * sa[i + 1]] + list(sa[i + 2:])
            elif how == "split" and len(sa) >= 1 and len(sa) < 5:
                i = r.randrange(len(sa))
                divs = [f for f in (2, 3, 4, 5, 7, 8, 10, 13, 16) if sa[i] % f == 0 and sa[i] > 0]
                if divs:
                    f = r.choice(divs)
                    new = list(sa[:i]) + ([f, sa[i] // f] if r.random() < 0.5 else [sa[i] // f, f]) + list(sa[i + 1:])
            else:
                new = [int(np.prod(sa))] if len(sa) else [1]
            given = list(new)
            if given and int(np.prod(sa)) > 0 and r.random() < 0.3:
                given[r.randrange(len(given))] = -1          # one extent left to be inferred
            steps.append(("reshape", a, tuple(given)))
            shapes.append(tuple(new))
        elif kind == "unary":
            op = r.choice(["neg", "abs", "square"] + (["sqrtabs"] if dtype == "f32" else []))
            steps.append(("unary", op, a))
            shapes.append(sa)
        elif kind == "binary":
            # broadcasting two transposed operands can multiply extents: keep results within bounds
            b = pick(lambda i: _broadcast(shapes[i], sa) is not None and int(np.prod(_broadcast(shapes[i], sa))) <= 2 * limit)
            op = r.choice(["add", "sub", "mul", "maximum", "minimum"] + (["divsafe"] if dtype == "f32" else []))
            steps.append(("binary", op, a, b))
            shapes.append(_broadcast(sa, shapes[b]))
        elif kind == "scalar":
            op = r.choice(["add", "sub", "mul", "maximum", "minimum"])
            v = r.choice([-3, -1, 0, 2, 7]) if dtype == "i32" or r.random() < 0.3 else r.choice([-1.5, 0.25, 0.1, 3.0])
            steps.append(("scalar", op, a, v, r.random() < 0.5))
            shapes.append(sa)
        elif kind == "slice":
            key, out = [], []
            for d in sa:
                if d <= 1 or r.random() < 0.3:
                    key.append((None, None, None))
                    out.append(d)
                    continue
                lo = r.randint(0, d - 1)
                hi = r.randint(lo + 1, d)
                st = r.choice([1, 1, 2, 3])
                if empty and r.random() < 0.15:
                    hi = lo                                 # an empty window: every later op sees extent 0
                neg = r.random() < 0.3                      # negative indices address from the end
                key.append((lo - d if neg else lo, hi - d if (neg and hi < d) else hi, st))
                out.append((hi - lo + st - 1) // st)
            steps.append(("slice", a, tuple(key)))
            shapes.append(tuple(out))
        elif kind == "transpose":
            perm = list(range(len(sa)))
            r.shuffle(perm)
            steps.append(("transpose", a, tuple(perm)))
            shapes.append(tuple(sa[p] for p in perm))
        elif kind == "reduce":
            ops = ["max", "min"] + (["sum"] if dtype == "i32" else [])
            op = "sum" if 0 in sa else r.choice(ops)
            naxes = r.randint(0, len(sa))                  # 0: all axes (axis=None)
            axes = tuple(sorted(r.sample(range(len(sa)), naxes))) if naxes else None
            keep = r.random() < 0.5
            red = set(range(len(sa))) if axes is None else set(axes)
            out = tuple((1 if i in red else d) for i, d in enumerate(sa) if keep or i not in red)
            steps.append(("reduce", op, a, axes, keep))
            shapes.append(out)
            if op == "sum":
                final.append(True)
                storage.append(False)
                computed.append(True)
                continue
        elif kind == "scan":
            op = r.choice(["cummax", "cummin"] + (["cumsum"] if dtype == "i32" else []))
            steps.append(("scan", op, a, r.randrange(len(sa))))
            shapes.append(sa)
            if op == "cumsum":
                final.append(True)
                storage.append(False)
                computed.append(True)
                continue
        else:
            steps.append(("materialize", a))
            # assign_values: an evaluated result is an array like any other and may be assigned into
            # (also one that an earlier assignment wrote straight into another array's storage)
            if assign_values and computed[a] and len(sa) >= 1 and all(d >= 1 for d in sa):
                storage[a] = True
            continue
        final.append(False)
        while len(storage) < len(shapes):
            storage.append(kind in ("slice", "transpose") and storage[a])
        while len(computed) < len(shapes):
            computed.append(kind not in ("slice", "transpose"))
    if not steps or steps[-1][0] == "materialize":
        steps.append(("unary", "neg", 0))
        shapes.append(shapes[0])
        final.append(False)
        computed.append(True)
    return dtype, leaf_shapes, steps, len(shapes) - 1


def make_tail(seed: int, dtype: str, shape):
    """One more step for a float recipe whose result is only reproducible up to rounding: a
    transcendental function, a float sum, or a contraction.  Returns (step, kind of comparison)."""
    r = random.Random(seed * 7919 + 1)
    if dtype != "f32":
        return None, None
    c = ["exp", "tanh", "erf", "log"] + (["sum"] * 3 if len(shape) >= 1 else []) + (["dot"] * 3 if len(shape) in (1, 2) else [])
    k = r.choice(c)
    if k == "sum":
        naxes = r.randint(0, len(shape))
        axes = tuple(sorted(r.sample(range(len(shape)), naxes))) if naxes else None
        return ("tail", "sum", axes, r.random() < 0.5), "reduction"
    if k == "dot":
        return ("tail", "dot", r.choice(["self_t", "column"]) if len(shape) == 2 else "inner"), "reduction"
    return ("tail", k), "elementwise"


def apply_tail(xp, step, x):
    if step[1] == "sum":
        return xp.sum(x, axis=step[2], keepdims=step[3])
    if step[1] == "dot":
        if step[2] == "inner":
            return xp.dot(x, x)
        if step[2] == "self_t":
            return xp.dot(x, xp.transpose(x, (1, 0)))
        return xp.dot(x, xp.transpose(x[0:1], (1, 0)))
    x = xp.minimum(xp.maximum(x, -30.0), 30.0)       # keep exp finite and the functions' arguments tame
    if step[1] == "log":
        return xp.log(abs(x) + 0.5)
    return getattr(xp, step[1])(x)


def make_leaves(seed: int, dtype: str, leaf_shapes):
    g = np.random.default_rng(1000003 * seed + 17)
    out = []
    for s in leaf_shapes:
        if dtype == "i32":
            # mostly small values (products stay meaningful), a few extreme ones (wrap-around)
            x = g.integers(-50, 50, s).astype(np.int32)
            m = g.random(s) < 0.02
            x[m] = g.integers(-2**31, 2**31 - 1, s, dtype=np.int64).astype(np.int32)[m]
        else:
            x = g.uniform(-2.0, 2.0, s).astype(np.float32)
            x[g.random(s) < 0.02] = 0.0
        out.append(x)
    return out


def apply(xp, steps, leaves):
    """Runs the recipe on arrays of module `xp` (NumPy's names); returns the pool."""
    pool = list(leaves)
    for st in steps:
        k = st[0]
        if k == "unary":
            x = pool[st[2]]
            pool.append({"neg": lambda: -x, "abs": lambda: abs(x), "square": lambda: xp.square(x),
                         "sqrtabs": lambda: xp.sqrt(abs(x))}[st[1]]())
        elif k == "binary":
            x, y = pool[st[2]], pool[st[3]]
            pool.append({"add": lambda: x + y, "sub": lambda: x - y, "mul": lambda: x * y,
                         "maximum": lambda: xp.maximum(x, y), "minimum": lambda: xp.minimum(x, y),
                         "divsafe": lambda: x / (abs(y) + 1.0)}[st[1]]())
        elif k == "scalar":
            x, v, left = pool[st[2]], st[3], st[4]
            if st[1] in ("maximum", "minimum"):
                f = getattr(xp, st[1])
                pool.append(f(v, x) if left else f(x, v))
            else:
                pool.append({"add": (lambda: v + x) if left else (lambda: x + v), "sub": (lambda: v - x) if left else (lambda: x - v),
                             "mul": (lambda: v * x) if left else (lambda: x * v)}[st[1]]())
        elif k == "slice":
            pool.append(pool[st[1]][tuple(slice(*t) for t in st[2])])
        elif k == "transpose":
            pool.append(xp.transpose(pool[st[1]], st[2]))
        elif k == "reshape":
            pool.append(xp.reshape(pool[st[1]], st[2]))
        elif k == "reduce":
            pool.append(getattr(xp, st[1])(pool[st[2]], axis=st[3], keepdims=st[4]))
        elif k == "scan":
            pool.append(getattr(xp, st[1])(pool[st[2]], st[3]))
        elif k == "materialize":
            if hasattr(pool[st[1]], "materialize"):
                pool[st[1]].materialize()
        elif k == "assign":
            key = tuple(slice(*t) for t in st[2])
            dst = pool[st[1]]
            if st[3] == "pool":
                val = pool[st[4]]
            elif st[3] == "self":
                val = dst[key] * 2 - 1
            else:
                val = dst[tuple(slice(*t) for t in st[4])]
                if st[3] == "shiftexpr":
                    val = val + 1
            dst[key] = val
    return pool


class NumpyModule:
    """NumPy under the names the recipes use; scalars keep the array's element type (the rule of
    both evaluators: a Python scalar never promotes an array)."""
    square = staticmethod(np.square)
    sqrt = staticmethod(np.sqrt)
    transpose = staticmethod(np.transpose)

    @staticmethod
    def reshape(a, shape):
        return np.reshape(a, shape).copy()        # the evaluators' reshape is an array of its own

    @staticmethod
    def maximum(a, b):
        a, b = NumpyModule._pair(a, b)
        return np.maximum(a, b)

    @staticmethod
    def minimum(a, b):
        a, b = NumpyModule._pair(a, b)
        return np.minimum(a, b)

    @staticmethod
    def _pair(a, b):
        if isinstance(a, (int, float)):
            a = b.dtype.type(a)
        if isinstance(b, (int, float)):
            b = a.dtype.type(b)
        return a, b

    @staticmethod
    def max(a, axis=None, keepdims=False): return np.max(a, axis=axis, keepdims=keepdims)
    @staticmethod
    def min(a, axis=None, keepdims=False): return np.min(a, axis=axis, keepdims=keepdims)
    @staticmethod
    def sum(a, axis=None, keepdims=False): return np.sum(a, axis=axis, keepdims=keepdims, dtype=np.int64)
    @staticmethod
    def cummax(a, axis): return np.maximum.accumulate(a, axis=axis)
    @staticmethod
    def cummin(a, axis): return np.minimum.accumulate(a, axis=axis)
    @staticmethod
    def cumsum(a, axis): return np.cumsum(a, axis=axis, dtype=np.int64)


def same_bits(got: np.ndarray, ref: np.ndarray, zero_signs: bool = True) -> bool:
    """Equal shape, element type and bit patterns; NaNs compare equal whatever their payload.
    zero_signs=False also lets +0 and -0 compare equal (which of two equal operands a maximum or
    minimum returns is not fixed by NumPy's documentation; none of the recipe's ops turns a
    difference in the sign of a zero into anything but a difference in the sign of a zero)."""
    got, ref = np.asarray(got), np.asarray(ref)
    if got.shape != ref.shape or got.dtype != ref.dtype:
        return False
    if got.dtype == np.float32:
        nan = np.isnan(ref)
        if not np.array_equal(np.isnan(got), nan):
            return False
        g, r = got.view(np.uint32)[~nan], ref.view(np.uint32)[~nan]
        if not zero_signs:
            g, r = np.where(g == 0x80000000, 0, g), np.where(r == 0x80000000, 0, r)
        return bool(np.array_equal(g, r))
    return bool(np.array_equal(got, ref))


# ---- contractions on integer-valued floats: exact whatever the summation order ---------------

def make_dot_case(seed: int):
    """A random contraction whose operands are windows (offset, step, optional transposition in
    memory) of float arrays holding integers in [-3, 3]: every partial sum is an integer below
    2**24, so any correct kernel returns the same bits.  Returns (arrays, program(xp, **arrays))."""
    r = random.Random(seed * 104729 + 7)
    g = np.random.default_rng(seed + 424242)
    dims = [1, 2, 3, 5, 16, 33, 64, 130, 257, 600]
    kind = r.choice(["gemm", "gemm", "rowdot", "colacc", "inner", "pair"])
    M, K, N = r.choice(dims), r.choice(dims), r.choice(dims)
    if kind == "pair":
        M, K = r.choice([5, 64, 257, 600, 3000]), r.choice([3, 16, 64, 130, 512])

    def window(rows, cols):
        """An integer-valued array and the slicing that cuts a (rows, cols) window out of it,
        possibly stored transposed."""
        sr, sc = r.choice([1, 1, 2, 3]), r.choice([1, 1, 2])
        o_r, o_c = r.randint(0, 7), r.randint(0, 9)
        tr = r.random() < 0.4
        full = (o_r + (rows - 1) * sr + 1 + r.randint(0, 3), o_c + (cols - 1) * sc + 1 + r.randint(0, 3))
        arr = g.integers(-3, 4, full[::-1] if tr else full).astype(np.float32)
        key = (slice(o_r, o_r + (rows - 1) * sr + 1, sr), slice(o_c, o_c + (cols - 1) * sc + 1, sc))
        return arr, (lambda xp, a: (xp.transpose(a, (1, 0)) if tr else a)[key])

    def vector(n):
        st, off = r.choice([1, 1, 2, 5]), r.randint(0, 11)
        arr = g.integers(-3, 4, (off + (n - 1) * st + 1 + r.randint(0, 3),)).astype(np.float32)
        return arr, (lambda xp, a: a[off:off + (n - 1) * st + 1:st])

    arrays, epi = {}, r.choice(["none", "bias", "relu", "scale"])
    if kind == "gemm":
        arrays["A"], fa = window(M, K)
        arrays["B"], fb = window(K, N)
        arrays["c"] = g.integers(-3, 4, (N,)).astype(np.float32)
        core = lambda xp, A, B, c: xp.dot(fa(xp, A), fb(xp, B))
    elif kind == "rowdot":
        arrays["A"], fa = window(M, K)
        arrays["B"], fb = vector(K)
        arrays["c"] = g.integers(-3, 4, (M,)).astype(np.float32)
        core = lambda xp, A, B, c: xp.dot(fa(xp, A), fb(xp, B))
    elif kind == "colacc":
        arrays["A"], fa = window(K, M)                       # (K, M) window used transposed: (M, K) . (K,)
        arrays["B"], fb = vector(K)
        arrays["c"] = g.integers(-3, 4, (M,)).astype(np.float32)
        core = lambda xp, A, B, c: xp.dot(xp.transpose(fa(xp, A), (1, 0)), fb(xp, B))
    elif kind == "inner":
        arrays["A"], fa = vector(K)
        arrays["B"], fb = vector(K)
        arrays["c"] = g.integers(-3, 4, (1,)).astype(np.float32)
        core = lambda xp, A, B, c: xp.dot(fa(xp, A), fb(xp, B))
        epi = "none"
    else:
        # the logistic-regression pattern with exact arithmetic: r = relu(X.w) - y, g = X^T.r
        arrays["A"], fa = window(M, K)
        arrays["B"], fb = vector(K)
        arrays["c"] = g.integers(0, 2, (M,)).astype(np.float32)
        def core(xp, A, B, c):
            X = fa(xp, A)
            rres = xp.maximum(xp.dot(X, fb(xp, B)), 0) - c
            return xp.dot(xp.transpose(X, (1, 0)), rres)
        epi = "none"

    def program(xp, A, B, c):
        out = core(xp, A, B, c)
        if epi == "bias":
            return out + c
        if epi == "relu":
            return xp.maximum(out + c, 0)
        if epi == "scale":
            return (out - c) * 0.5
        return out
    return kind, arrays, program
