"""Thin ctypes binding over the C-ABI library (include/grumpy_hip.h).

Argument marshalling only: every step of the path (recording, shape and
broadcast inference, partitioning, code generation, kernels) runs inside
libgrumpy_hip.so.  PyTorch is used for device memory and the stream.  There is
no CPU fallback: if the library is missing, loading fails.

``Array`` mirrors the part of ``numpy.ndarray`` the paper's programs use
(Section 4.1: an ndarray object that stands for one DAG node), and the module
exposes NumPy-named functions so that a program written against ``numpy`` runs
unchanged with this module passed in its place.
"""
from __future__ import annotations

import builtins
import atexit
import ctypes
import weakref
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("GRUMPY_HIP_LIB", os.path.join(_HERE, "libgrumpy_hip.so"))

GR_F32, GR_I32, GR_I64 = 0, 1, 2
GR_NEG, GR_ABS, GR_EXP, GR_LOG, GR_SQRT, GR_SQUARE, GR_TANH, GR_ERF = range(8)
GR_ADD, GR_SUB, GR_MUL, GR_DIV, GR_MAXIMUM, GR_MINIMUM, GR_POW_INT = range(16, 23)
_UNARY = {"neg": 0, "abs": 1, "exp": 2, "log": 3, "sqrt": 4, "square": 5, "tanh": 6, "erf": 7}
_BINARY = {"add": 16, "sub": 17, "mul": 18, "div": 19, "maximum": 20, "minimum": 21}
_REDUCE = {"sum": 32, "max": 33, "min": 34}
STATUS = {0: "GR_OK", 1: "GR_ERR_HANDLE", 2: "GR_ERR_SHAPE", 3: "GR_ERR_DTYPE", 4: "GR_ERR_AXIS",
          5: "GR_ERR_UNSUPPORTED", 6: "GR_ERR_ARG", 7: "GR_ERR_COMPILE", 8: "GR_ERR_HIP", 9: "GR_ERR_OOM",
          10: "GR_ERR_ALIAS", 11: "GR_ERR_NODEVICE"}

# every symbol include/grumpy_hip.h declares
SYMBOLS = [
    "gr_ctx_create", "gr_ctx_destroy", "gr_ctx_set_stream", "gr_ctx_set_allocator", "gr_ctx_set_option", "gr_sync",
    "gr_last_error", "gr_array_from_device", "gr_array_lend_buffer", "gr_scalar", "gr_unary", "gr_binary", "gr_binary_scalar", "gr_slice", "gr_transpose", "gr_reshape",
    "gr_reduce", "gr_scan", "gr_dot", "gr_materialize", "gr_materialize_into", "gr_materialize_into_static", "gr_static_scratch_bytes", "gr_program_create", "gr_program_run", "gr_program_destroy", "gr_assign", "gr_ndim", "gr_shape", "gr_dtype_of",
    "gr_is_materialized", "gr_data_ptr", "gr_retain", "gr_release", "gr_plan_describe", "gr_plan_source",
    "gr_plan_compile", "gr_compile_wait", "gr_stats", "gr_profile_reset", "gr_profile_read", "gr_stream_copy", "gr_stream_read",
]


class GrError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status
        self.code = STATUS.get(status, str(status))


class Stats(ctypes.Structure):
    _fields_ = [("nodes_recorded", ctypes.c_uint64), ("nodes_alive", ctypes.c_uint64),
                ("materialize_calls", ctypes.c_uint64), ("groups_executed", ctypes.c_uint64),
                ("kernel_launches", ctypes.c_uint64), ("cache_hits", ctypes.c_uint64),
                ("cache_misses", ctypes.c_uint64), ("compile_ms", ctypes.c_double),
                ("bytes_allocated", ctypes.c_uint64), ("disk_hits", ctypes.c_uint64),
                ("nodes_merged", ctypes.c_uint64), ("interp_launches", ctypes.c_uint64),
                ("assign_swaps", ctypes.c_uint64), ("plan_hits", ctypes.c_uint64), ("pool_bytes", ctypes.c_uint64)]


_lib = None
_TORCH_DTYPES = {}
_I64_ARRAYS = [ctypes.c_int64 * builtins.max(n, 1) for n in range(9)]


def lib():
    """Loads libgrumpy_hip.so (built in-tree by build.py); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    P, I, I64, U64, SZ = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64, ctypes.c_size_t
    PP = ctypes.POINTER
    sig = {
        "gr_ctx_create": [PP(P), I, P], "gr_ctx_destroy": [P], "gr_ctx_set_stream": [P, P],
        "gr_ctx_set_allocator": [P, P, P, P], "gr_ctx_set_option": [P, ctypes.c_char_p, I64], "gr_sync": [P],
        "gr_array_from_device": [P, P, I, I, PP(I64), PP(I64), PP(U64)],
        "gr_scalar": [P, ctypes.c_double, I, PP(U64)],
        "gr_unary": [P, I, U64, PP(U64)], "gr_binary": [P, I, U64, U64, PP(U64)],
        "gr_binary_scalar": [P, I, U64, ctypes.c_double, I, I, PP(U64)],
        "gr_slice": [P, U64, I, PP(I64), PP(I64), PP(I64), PP(ctypes.c_uint8), PP(ctypes.c_uint8), PP(U64)],
        "gr_transpose": [P, U64, PP(I), PP(U64)],
        "gr_reshape": [P, U64, I, PP(I64), PP(U64)],
        "gr_reduce": [P, I, U64, PP(I), I, I, PP(U64)], "gr_dot": [P, U64, U64, PP(U64)],
        "gr_scan": [P, I, U64, I, PP(U64)],
        "gr_materialize": [P, U64], "gr_assign": [P, U64, U64], "gr_materialize_into": [P, U64, P, SZ],
        "gr_array_lend_buffer": [P, U64, P, SZ],
        "gr_materialize_into_static": [P, U64, P, SZ], "gr_static_scratch_bytes": [PP(SZ)],
        "gr_program_create": [P, U64, PP(U64), I, PP(P)], "gr_program_run": [P, PP(P), P], "gr_program_destroy": [P],
        "gr_ndim": [P, U64, PP(I)], "gr_shape": [P, U64, PP(I64)], "gr_dtype_of": [P, U64, PP(I)],
        "gr_is_materialized": [P, U64, PP(I)], "gr_data_ptr": [P, U64, PP(P), PP(I64)],
        "gr_retain": [P, U64], "gr_release": [P, U64],
        "gr_plan_describe": [P, U64, ctypes.c_char_p, SZ, PP(SZ)],
        "gr_plan_source": [P, U64, I, ctypes.c_char_p, SZ, PP(SZ)], "gr_plan_compile": [P, U64],
        "gr_compile_wait": [P],
        "gr_stats": [P, PP(Stats)], "gr_profile_reset": [P],
        "gr_profile_read": [P, ctypes.c_char_p, PP(U64), PP(ctypes.c_double)],
        "gr_stream_copy": [P, P, P, SZ], "gr_stream_read": [P, P, SZ, P],
    }
    for name, argtypes in sig.items():
        fn = getattr(L, name)
        fn.argtypes = argtypes
        fn.restype = I
    L.gr_last_error.argtypes = [P]
    L.gr_last_error.restype = ctypes.c_char_p
    _lib = L
    _bind_fast_paths(L)
    return L


def _torch():
    import torch
    return torch


# Contexts still open when the interpreter exits are closed while the HIP runtime is still up
# (a context may have compilations running on host threads).
_LIVE = weakref.WeakSet()


@atexit.register
def _close_live_contexts():
    for c in list(_LIVE):
        try:
            c.close()
        except Exception:
            pass


class Context:
    """One gr_ctx.  device=-1 records, plans and generates code without a GPU."""

    def __init__(self, device: Optional[int] = None, stream: Optional[int] = None):
        L = lib()
        if device is None:
            torch = _torch()
            if not torch.cuda.is_available():
                raise RuntimeError("no GPU visible; pass device=-1 for a device-less context")
            device = torch.cuda.current_device()
        if stream is None and device >= 0:
            torch = _torch()
            if torch.cuda.is_available() and device < torch.cuda.device_count():
                stream = torch.cuda.current_stream(device).cuda_stream
        self._p = ctypes.c_void_p()
        st = L.gr_ctx_create(ctypes.byref(self._p), int(device), ctypes.c_void_p(stream or 0))
        if st:
            raise GrError(st, L.gr_last_error(None).decode())
        self._addr = self._p.value or 0  # what the C fast paths read; 0 once closed
        self.device = int(device)
        self._programs = set()  # recorded requests (Program): they die with the context
        _LIVE.add(self)

    def program(self, root: "Array", leaves: Sequence["Array"]) -> "Program":
        """Records the evaluation of ``root`` for replay on new data in place of ``leaves`` (gr_program_create)."""
        return Program(root, leaves)

    def close(self):
        self._addr = 0
        for prog in list(getattr(self, "_programs", ())):
            prog._p = None              # the library frees a context's programs with it
        if self._p:
            lib().gr_ctx_destroy(self._p)
            self._p = ctypes.c_void_p()
        _LIVE.discard(self)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, st: int):
        if st:
            raise GrError(st, lib().gr_last_error(self._p).decode())

    def last_error(self) -> str:
        return lib().gr_last_error(self._p).decode()

    def set_allocator(self, alloc, free):
        """Installs Python callables alloc(nbytes) -> device address or None, free(address) as the
        context's device allocator (results of gr_materialize, temporaries, workspaces)."""
        ALLOC = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
        FREE = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)

        def _alloc(n, user):
            try:
                return alloc(n)
            except Exception:
                return None

        def _free(ptr, user):
            try:
                free(ptr)
            except Exception:
                pass

        self._allocator = (ALLOC(_alloc), FREE(_free))  # kept alive: the library calls them until close()
        self.check(lib().gr_ctx_set_allocator(self._p, ctypes.cast(self._allocator[0], ctypes.c_void_p),
                                              ctypes.cast(self._allocator[1], ctypes.c_void_p), None))

    def use_torch_allocator(self):
        """Routes the context's allocations through PyTorch's caching allocator."""
        torch = _torch()
        dev = self.device
        self.set_allocator(lambda n: torch.cuda.caching_allocator_alloc(n, dev, torch.cuda.current_stream(dev)),
                           lambda ptr: torch.cuda.caching_allocator_delete(ptr))

    def set_option(self, key: str, value: int):
        self.check(lib().gr_ctx_set_option(self._p, key.encode(), int(value)))

    def set_stream(self, stream: int):
        self.check(lib().gr_ctx_set_stream(self._p, ctypes.c_void_p(stream)))

    def sync(self):
        self.check(lib().gr_sync(self._p))

    def compile_wait(self):
        """Blocks until every compilation running in the background has finished."""
        self.check(lib().gr_compile_wait(self._p))

    def stats(self) -> dict:
        s = Stats()
        self.check(lib().gr_stats(self._p, ctypes.byref(s)))
        return {k: getattr(s, k) for k, _ in Stats._fields_}

    def profile_reset(self):
        self.check(lib().gr_profile_reset(self._p))

    def profile_read(self, prefix: str = ""):
        n, ms = ctypes.c_uint64(), ctypes.c_double()
        self.check(lib().gr_profile_read(self._p, prefix.encode(), ctypes.byref(n), ctypes.byref(ms)))
        return int(n.value), float(ms.value)

    # -- leaves ---------------------------------------------------------------
    def from_device(self, ptr: int, dtype: int, shape: Sequence[int], strides: Optional[Sequence[int]] = None,
                    owner=None) -> "Array":
        n = len(shape)
        T = _I64_ARRAYS[n]
        h = ctypes.c_uint64()
        st = _lib.gr_array_from_device(self._p, ptr, dtype, n, T(*shape), None if strides is None else T(*strides),
                                       ctypes.byref(h))
        if st:
            self.check(st)
        a = Array(self, h.value)
        a._owner = owner  # keeps the device memory of the leaf alive as long as the handle
        return a

    def array(self, t, second=None) -> "Array":
        """Wraps a torch tensor that lives on this context's GPU (borrowed, any strides).  ``second``: a second
        tensor of the same shape lent to the library (gr_array_lend_buffer): stencil sweeps assigned into the array
        then alternate between the two tensors instead of going through a temporary; ``Array.current(t, second)``
        tells which of them holds the contents."""
        if second is not None:
            a = self.array(t)
            if tuple(second.shape) != tuple(t.shape) or second.dtype != t.dtype or not second.is_contiguous():
                raise ValueError("the second buffer must be a contiguous tensor of the same shape and element type")
            self.check(lib().gr_array_lend_buffer(self._p, a.h, second.data_ptr(), second.numel() * second.element_size()))
            a._owner = (t, second)
            return a
        try:
            dt = _TORCH_DTYPES[t.dtype]
        except (KeyError, AttributeError):
            torch = _torch()
            if not isinstance(t, torch.Tensor):
                raise TypeError("expected a torch.Tensor on the GPU")
            _TORCH_DTYPES.update({torch.float32: GR_F32, torch.int32: GR_I32, torch.int64: GR_I64})
            if t.dtype not in _TORCH_DTYPES:
                raise GrError(3, f"unsupported dtype {t.dtype}")
            dt = _TORCH_DTYPES[t.dtype]
        if not t.is_cuda:
            raise ValueError("tensor must live in device memory")
        return self.from_device(t.data_ptr(), dt, t.shape, t.stride(), owner=t)

    def spec(self, shape: Sequence[int], dtype: int = GR_F32, strides: Optional[Sequence[int]] = None) -> "Array":
        """A leaf with a placeholder address, for planning on a device-less context."""
        return self.from_device(0x10000, dtype, tuple(shape), strides)

    def scalar(self, v) -> "Array":
        h = ctypes.c_uint64()
        if isinstance(v, bool):
            raise GrError(5, "bool scalars are not supported")
        is_int = isinstance(v, int) or type(v).__name__.startswith(("int", "uint"))
        self.check(lib().gr_scalar(self._p, float(v), int(is_int), ctypes.byref(h)))
        return Array(self, h.value)

    # -- streaming ceiling kernels ----------------------------------------------
    def stream_copy(self, dst, src):
        self.check(lib().gr_stream_copy(self._p, ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()),
                                        src.numel() * src.element_size()))

    def stream_read(self, src, sink):
        self.check(lib().gr_stream_read(self._p, ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                                        ctypes.c_void_p(sink.data_ptr())))


class _DeviceExport:
    """Zero-copy hand-over of a materialised node's storage (CUDA array interface, version 2)."""

    def __init__(self, owner, ptr, shape, byte_strides, typestr):
        self.owner = owner  # keeps the handle, hence the storage, alive
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": typestr, "data": (ptr, False), "version": 2,
                                         "strides": byte_strides if len(shape) else None}


class Program:
    """A request recorded once and run many times on new data (gr_program_*): ``root`` is evaluated with the
    tensors given to ``run`` in place of ``leaves`` (same element type, shape and strides), launches only."""

    def __init__(self, root: "Array", leaves: Sequence["Array"]):
        self.ctx = root.ctx
        n = len(leaves)
        arr = (ctypes.c_uint64 * builtins.max(n, 1))(*[l.h for l in leaves])
        p = ctypes.c_void_p()
        self.ctx.check(lib().gr_program_create(self.ctx._p, root.h, arr, n, ctypes.byref(p)))
        self._p = p.value
        self._n = n
        self._keep = root._owner        # inputs that are not rebound stay bound to their memory
        self.ctx._programs.add(self)

    def run(self, tensors, out):
        """Launches the recorded kernels on ``tensors`` (one per rebindable leaf, in order) into ``out``."""
        if len(tensors) != self._n:
            raise ValueError(f"expected {self._n} inputs")
        ptrs = tuple(t.data_ptr() for t in tensors)
        if _fastbind is not None:
            st = _fastbind.program_run(self._p, ptrs, out.data_ptr())
        else:
            st = _lib.gr_program_run(self._p, (ctypes.c_void_p * builtins.max(self._n, 1))(*ptrs), out.data_ptr())
        if st:
            self.ctx.check(st)
        return out

    def close(self):
        if self._p and self.ctx._p:
            lib().gr_program_destroy(self._p)
        self._p = None
        self.ctx._programs.discard(self)


class _PyArrayBase:
    """The recording calls through ctypes alone (GRUMPY_NO_FASTBIND=1): what _fastbind.ArrayBase does in C."""

    __slots__ = ("ctx", "h", "_owner", "_view")

    def __init__(self, ctx: Context, handle: int):
        self.ctx = ctx
        self.h = handle
        self._owner = None
        self._view = False

    def __del__(self):
        try:
            p = self.ctx._p
            if p:
                _lib.gr_release(p, self.h)
        except Exception:
            pass

    def materialize(self):
        self.ctx.check(lib().gr_materialize(self.ctx._p, self.h))
        if not self._view:
            self._owner = None  # the node now has storage of its own and has let go of its inputs
        return self

    def _materialize_into(self, ptr, nbytes, tensor, static=False):
        had = ctypes.c_int(1)
        if not self._view:
            self.ctx.check(_lib.gr_is_materialized(self.ctx._p, self.h, ctypes.byref(had)))
        fn = _lib.gr_materialize_into_static if static else _lib.gr_materialize_into
        self.ctx.check(fn(self.ctx._p, self.h, ptr, nbytes))
        if not had.value:
            self._owner = tensor
        return self

    def __add__(self, o): return _binary_slow(GR_ADD, self, o)
    def __radd__(self, o): return _binary_slow(GR_ADD, o, self)
    def __sub__(self, o): return _binary_slow(GR_SUB, self, o)
    def __rsub__(self, o): return _binary_slow(GR_SUB, o, self)
    def __mul__(self, o): return _binary_slow(GR_MUL, self, o)
    def __rmul__(self, o): return _binary_slow(GR_MUL, o, self)
    def __truediv__(self, o): return _binary_slow(GR_DIV, self, o)
    def __rtruediv__(self, o): return _binary_slow(GR_DIV, o, self)
    def __neg__(self): return _unary_slow(GR_NEG, self)
    def __abs__(self): return _unary_slow(GR_ABS, self)
    def __matmul__(self, o): return dot(self, o)
    def __pow__(self, e): return _pow_slow(self, e)
    def __getitem__(self, key): return slice_(self, key)
    def __setitem__(self, key, value): _setitem_slow(self, key, value)

    @property
    def T(self):
        return transpose(self)


class _ArrayMethods:
    """Everything of an Array that is not on the recording fast path."""

    __slots__ = ()

    # -- inspection -----------------------------------------------------------
    @property
    def ndim(self) -> int:
        n = ctypes.c_int()
        self.ctx.check(lib().gr_ndim(self.ctx._p, self.h, ctypes.byref(n)))
        return n.value

    @property
    def shape(self):
        n = self.ndim
        s = (ctypes.c_int64 * builtins.max(n, 1))()
        self.ctx.check(lib().gr_shape(self.ctx._p, self.h, s))
        return tuple(int(s[i]) for i in range(n))

    @property
    def dtype_code(self) -> int:
        d = ctypes.c_int()
        self.ctx.check(lib().gr_dtype_of(self.ctx._p, self.h, ctypes.byref(d)))
        return d.value

    @property
    def is_materialized(self) -> bool:
        f = ctypes.c_int()
        self.ctx.check(lib().gr_is_materialized(self.ctx._p, self.h, ctypes.byref(f)))
        return bool(f.value)

    def data_ptr(self):
        p = ctypes.c_void_p()
        st = (ctypes.c_int64 * 8)()
        self.ctx.check(lib().gr_data_ptr(self.ctx._p, self.h, ctypes.byref(p), st))
        return p.value or 0, tuple(int(st[i]) for i in range(self.ndim))

    def current(self, *tensors):
        """Which of the given tensors is this array's storage right now (after sweeps over a lent second buffer)."""
        ptr, _ = self.data_ptr()
        for t in tensors:
            if t.data_ptr() == ptr:
                return t
        raise LookupError("the array's storage is none of the given tensors")

    def copy(self) -> "Array":
        """An evaluated array with storage of its own (allocated and owned by the library) holding
        this array's values; multiplying by one is exact for every value."""
        return (self * 1).materialize()

    # -- materialisation --------------------------------------------------------
    def materialize_into(self, t) -> "Array":
        """Evaluates into the caller's tensor (gr_materialize_into).  An array that had no storage is bound to the
        tensor, which then is what keeps it alive; one that had (and every view) is copied."""
        return self._materialize_into(t.data_ptr(), t.numel() * t.element_size(), t, False)

    def materialize_into_static(self, t) -> "Array":
        """materialize_into for callers that must not allocate device memory (gr_materialize_into_static)."""
        return self._materialize_into(t.data_ptr(), t.numel() * t.element_size(), t, True)

    def torch(self, copy: bool = True):
        """Evaluates the node (its storage then belongs to the library and lives as long as the node,
        Section 2) and returns its value as a torch tensor on the context's device: a copy by default,
        with copy=False a tensor that shares the node's storage (and keeps this handle alive)."""
        torch = _torch()
        dt = {GR_F32: (torch.float32, "<f4", 4), GR_I32: (torch.int32, "<i4", 4), GR_I64: (torch.int64, "<i8", 8)}[self.dtype_code]
        shape = self.shape
        if 0 in shape:
            return torch.empty(shape, dtype=dt[0], device=f"cuda:{self.ctx.device}")
        self.materialize()
        ptr, strides = self.data_ptr()
        view = torch.as_tensor(_DeviceExport(self, ptr, shape, tuple(s * dt[2] for s in strides), dt[1]),
                               device=f"cuda:{self.ctx.device}")
        return view.clone() if copy else view

    def numpy(self):
        return self.torch(copy=False).cpu().numpy()

    def plan(self) -> str:
        need = ctypes.c_size_t()
        self.ctx.check(lib().gr_plan_describe(self.ctx._p, self.h, None, 0, ctypes.byref(need)))
        buf = ctypes.create_string_buffer(need.value)
        self.ctx.check(lib().gr_plan_describe(self.ctx._p, self.h, buf, need.value, ctypes.byref(need)))
        return buf.value.decode()

    def source(self, index: int = 0) -> str:
        need = ctypes.c_size_t()
        self.ctx.check(lib().gr_plan_source(self.ctx._p, self.h, index, None, 0, ctypes.byref(need)))
        buf = ctypes.create_string_buffer(need.value)
        self.ctx.check(lib().gr_plan_source(self.ctx._p, self.h, index, buf, need.value, ctypes.byref(need)))
        return buf.value.decode()

    def compile(self) -> "Array":
        self.ctx.check(lib().gr_plan_compile(self.ctx._p, self.h))
        return self

    # -- NumPy-named methods --------------------------------------------------------
    def mean(self, axis=None, keepdims=False): return mean(self, axis, keepdims)
    def var(self, axis=None, keepdims=False): return var(self, axis, keepdims)
    def std(self, axis=None, keepdims=False): return std(self, axis, keepdims)
    def clip(self, lo, hi): return clip(self, lo, hi)
    def sum(self, axis=None, keepdims=False): return reduce("sum", self, axis, keepdims)
    def max(self, axis=None, keepdims=False): return reduce("max", self, axis, keepdims)
    def min(self, axis=None, keepdims=False): return reduce("min", self, axis, keepdims)
    def dot(self, o): return dot(self, o)
    def cumsum(self, axis=None): return cumsum(self, axis)

    def reshape(self, *shape):
        return reshape(self, shape[0] if len(shape) == 1 and not isinstance(shape[0], int) else shape)


def _load_fastbind():
    """The C type with the recording fast paths (built in-tree by build.py).  GRUMPY_NO_FASTBIND=1
    selects the ctypes-only route instead; a missing module is an error, not a silent fallback."""
    if os.environ.get("GRUMPY_NO_FASTBIND") == "1":
        return None
    try:
        from . import _fastbind
    except ImportError as e:
        raise ImportError(f"{e}: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or set GRUMPY_NO_FASTBIND=1 for the ctypes-only binding)") from None
    return _fastbind


_fastbind = _load_fastbind()


class Array(_PyArrayBase if _fastbind is None else _fastbind.ArrayBase, _ArrayMethods):
    """Handle of one DAG node."""

    __slots__ = ()
    __array_priority__ = 1000


def _bind_fast_paths(L):
    if _fastbind is None:
        return
    names = ["gr_unary", "gr_binary", "gr_binary_scalar", "gr_slice", "gr_transpose", "gr_dot", "gr_assign",
             "gr_materialize", "gr_release", "gr_reduce", "gr_ndim", "gr_shape", "gr_materialize_into",
             "gr_materialize_into_static", "gr_is_materialized", "gr_program_run"]
    _fastbind.bind({n: ctypes.cast(getattr(L, n), ctypes.c_void_p).value for n in names})
    _fastbind.set_hooks(_binary_slow, slice_, _setitem_slow, _pow_slow, _reduce_slow)


def _result(ctx: Context, handle: int, a=None, b=None, view: bool = False) -> "Array":
    """Wraps the handle of a freshly recorded node.  The recorded DAG outlives the handles of its leaves
    (``z = ctx.array(tensor) * 2`` drops the leaf's handle at once), so a result carries what keeps its
    operands' leaves alive: one owner as it is, two different ones as a pair."""
    r = Array(ctx, handle)
    oa = a._owner if isinstance(a, Array) else None
    ob = b._owner if isinstance(b, Array) else None
    if oa is None or ob is None or oa is ob:
        owner = oa if oa is not None else ob
    else:
        owner = (oa, ob)
    if owner is not None:
        r._owner = owner
    if view:
        r._view = True
    return r


def _ctx_of(*xs) -> Context:
    for x in xs:
        if isinstance(x, Array):
            return x.ctx
    raise TypeError("no array operand")


def _operand(ctx: Context, x) -> Array:
    if isinstance(x, Array):
        if x.ctx is not ctx:
            raise ValueError("arrays belong to different contexts")
        return x
    return ctx.scalar(x)


def _unary_slow(op: int, a) -> Array:
    ctx = _ctx_of(a)
    h = ctypes.c_uint64()
    st = _lib.gr_unary(ctx._p, op, a.h, ctypes.byref(h))
    if st:
        ctx.check(st)
    return _result(ctx, h.value, a)


def _binary_slow(op: int, a, b) -> Array:
    h = ctypes.c_uint64()
    if isinstance(a, Array):
        ctx = a.ctx
        if isinstance(b, Array):
            if b.ctx is not ctx:
                raise ValueError("arrays belong to different contexts")
            st = _lib.gr_binary(ctx._p, op, a.h, b.h, ctypes.byref(h))
        else:
            st = _lib.gr_binary_scalar(ctx._p, op, a.h, float(_number(b)), _is_int(b), 0, ctypes.byref(h))
    elif isinstance(b, Array):
        ctx = b.ctx
        st = _lib.gr_binary_scalar(ctx._p, op, b.h, float(_number(a)), _is_int(a), 1, ctypes.byref(h))
    else:
        raise TypeError("no array operand")
    if st:
        ctx.check(st)
    return _result(ctx, h.value, a, b)


def _pow_slow(a, e) -> Array:
    if isinstance(a, Array) and _is_int(e) and not isinstance(e, bool):
        return _binary_slow(GR_POW_INT, a, e)  # the library records x ** 2 as square(x), as NumPy evaluates it
    raise GrError(5, "only array ** integer is recorded")


def _setitem_slow(a, key, value):
    if not isinstance(value, Array):
        raise GrError(5, "only arrays can be assigned")
    dst = slice_(a, key)
    a.ctx.check(lib().gr_assign(a.ctx._p, dst.h, value.h))


_unary = _unary_slow if _fastbind is None else _fastbind.unary
_binary = _binary_slow if _fastbind is None else _fastbind.binary


def unary(name: str, a) -> Array:
    return _unary(_UNARY[name], a)


def binary(name: str, a, b) -> Array:
    return _binary(_BINARY[name], a, b)


def _number(v):
    if isinstance(v, bool):
        raise GrError(5, "bool scalars are not supported")
    if not isinstance(v, (int, float)) and not hasattr(v, "__float__"):
        raise TypeError(f"unsupported operand {type(v)}")
    return v


def _is_int(v) -> int:
    return int(isinstance(v, int) or type(v).__name__.startswith(("int", "uint")))


def slice_(a: Array, key) -> Array:
    if not isinstance(key, tuple):
        key = (key,)
    n = len(key)
    I64, U8 = ctypes.c_int64 * builtins.max(n, 1), ctypes.c_uint8 * builtins.max(n, 1)
    start, stop, step, hs, he = I64(), I64(), I64(), U8(), U8()
    for d, k in enumerate(key):
        if not isinstance(k, slice):
            raise GrError(5, "only slice objects are supported as indices")
        step[d] = 1 if k.step is None else int(k.step)
        hs[d] = k.start is not None
        he[d] = k.stop is not None
        start[d] = 0 if k.start is None else int(k.start)
        stop[d] = 0 if k.stop is None else int(k.stop)
    h = ctypes.c_uint64()
    a.ctx.check(lib().gr_slice(a.ctx._p, a.h, n, start, stop, step, hs, he, ctypes.byref(h)))
    return _result(a.ctx, h.value, a, view=True)


def transpose(a: Array, axes: Optional[Sequence[int]] = None) -> Array:
    p = None if axes is None else (ctypes.c_int * len(axes))(*axes)
    h = ctypes.c_uint64()
    a.ctx.check(lib().gr_transpose(a.ctx._p, a.h, p, ctypes.byref(h)))
    return _result(a.ctx, h.value, a, view=True)


def reshape(a: Array, shape) -> Array:
    """Row-major reshape; the result is an array of its own (a fused copy when it is evaluated)."""
    shape = [int(shape)] if isinstance(shape, int) else [int(v) for v in shape]
    arr = (ctypes.c_int64 * builtins.max(len(shape), 1))(*shape)
    h = ctypes.c_uint64()
    a.ctx.check(lib().gr_reshape(a.ctx._p, a.h, len(shape), arr, ctypes.byref(h)))
    return _result(a.ctx, h.value, a)


def reduce(name: str, a: Array, axis=None, keepdims=False) -> Array:
    return _reduce(_REDUCE[name], a, axis, keepdims)


def _reduce_slow(op: int, a: Array, axis=None, keepdims=False) -> Array:
    if axis is None:
        axes = []
    elif isinstance(axis, int):
        axes = [axis]
    else:
        axes = list(axis)
        if not axes:
            raise GrError(4, "empty axis tuple")
    arr = (ctypes.c_int * builtins.max(len(axes), 1))(*axes)
    h = ctypes.c_uint64()
    a.ctx.check(lib().gr_reduce(a.ctx._p, op, a.h, arr, len(axes), int(bool(keepdims)), ctypes.byref(h)))
    return _result(a.ctx, h.value, a)


_reduce = _reduce_slow if _fastbind is None else _fastbind.reduce


def scan(name: str, a: Array, axis: int) -> Array:
    h = ctypes.c_uint64()
    a.ctx.check(lib().gr_scan(a.ctx._p, _REDUCE[name], a.h, int(axis), ctypes.byref(h)))
    return _result(a.ctx, h.value, a)


def _scan_axis(name, a, axis):
    # axis=None: NumPy's scan over the flattened array
    return scan(name, reshape(a, (-1,)), 0) if axis is None else scan(name, a, axis)


def cumsum(a, axis=None): return _scan_axis("sum", a, axis)
def cummax(a, axis=None): return _scan_axis("max", a, axis)
def cummin(a, axis=None): return _scan_axis("min", a, axis)


def dot(a: Array, b: Array) -> Array:
    if not isinstance(a, Array) or not isinstance(b, Array):
        raise TypeError("dot: both operands must be arrays")
    h = ctypes.c_uint64()
    a.ctx.check(lib().gr_dot(a.ctx._p, a.h, b.h, ctypes.byref(h)))
    return _result(a.ctx, h.value, a, b)


# NumPy-named functions
def add(a, b): return _binary(GR_ADD, a, b)
def subtract(a, b): return _binary(GR_SUB, a, b)
def multiply(a, b): return _binary(GR_MUL, a, b)
def divide(a, b): return _binary(GR_DIV, a, b)
def maximum(a, b): return _binary(GR_MAXIMUM, a, b)
def minimum(a, b): return _binary(GR_MINIMUM, a, b)
def negative(a): return _unary(GR_NEG, a)
def absolute(a): return _unary(GR_ABS, a)
def exp(a): return _unary(GR_EXP, a)
def log(a): return _unary(GR_LOG, a)
def sqrt(a): return _unary(GR_SQRT, a)
def square(a): return _unary(GR_SQUARE, a)
def tanh(a): return _unary(GR_TANH, a)
def erf(a): return _unary(GR_ERF, a)
def sum(a, axis=None, keepdims=False): return _reduce(32, a, axis, keepdims)  # noqa: A001
def max(a, axis=None, keepdims=False): return _reduce(33, a, axis, keepdims)  # noqa: A001


def mean(a, axis=None, keepdims=False):
    """NumPy's mean of a float32 array, recorded as the sum over the axes divided by their element count."""
    extents = a.shape
    count = 1
    for d in (range(len(extents)) if axis is None else ((axis,) if isinstance(axis, int) else tuple(axis))):
        count *= extents[d]
    return _reduce(32, a, axis, keepdims) / float(count)


def var(a, axis=None, keepdims=False):
    """NumPy's var (ddof = 0): the mean of the squared deviations from the mean."""
    d = a - mean(a, axis, True)
    return mean(d * d, axis, keepdims)


def std(a, axis=None, keepdims=False):
    return sqrt(var(a, axis, keepdims))


def clip(a, lo, hi):
    """NumPy's clip with two bounds."""
    return minimum(maximum(a, lo), hi)
def min(a, axis=None, keepdims=False): return _reduce(34, a, axis, keepdims)  # noqa: A001
