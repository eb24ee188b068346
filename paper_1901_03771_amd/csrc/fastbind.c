/* CPython type behind the binding's Array class: the recording calls of the C ABI
 * (gr_unary, gr_binary, gr_binary_scalar, gr_slice, gr_transpose, gr_dot, gr_reduce, gr_assign,
 * gr_materialize, gr_release, gr_ndim, gr_shape) reached through the number and mapping protocols without
 * ctypes in between.  Argument marshalling only: a user program that records a few dozen
 * operations per sweep spends its host time here, and at small array sizes that time, not
 * the kernels, bounds the throughput.
 *
 * The library itself is not linked: lazy.py loads it once (ctypes) and hands the addresses
 * of the entry points to bind(), so that both routes call the same library instance.
 * Everything unusual (operands that are neither arrays nor Python numbers, index keys that
 * are not slices, errors) is passed to Python callables registered with set_hooks(). */
#define PY_SSIZE_T_CLEAN
#include <Python.h>
#include <structmember.h>

#include "../../include/grumpy_hip.h"

typedef struct {
  PyObject_HEAD
  PyObject* ctx;   /* the binding's Context object (attribute _addr: address of the gr_ctx, 0 once closed) */
  unsigned long long h;
  PyObject* owner; /* whatever keeps alive the device memory of the leaves this node still reads: a leaf's
                      tensor, or a tuple of the operands' owners */
  char view;       /* a slice or transpose: it reads its base's storage also once evaluated */
} ArrayObject;

static PyTypeObject ArrayBase_Type;

static __typeof__(&gr_unary) p_unary;
static __typeof__(&gr_binary) p_binary;
static __typeof__(&gr_binary_scalar) p_binary_scalar;
static __typeof__(&gr_slice) p_slice;
static __typeof__(&gr_transpose) p_transpose;
static __typeof__(&gr_dot) p_dot;
static __typeof__(&gr_assign) p_assign;
static __typeof__(&gr_materialize) p_materialize;
static __typeof__(&gr_materialize_into) p_materialize_into;
static __typeof__(&gr_materialize_into_static) p_materialize_into_static;
static __typeof__(&gr_is_materialized) p_is_materialized;
static __typeof__(&gr_program_run) p_program_run;
static __typeof__(&gr_release) p_release;
static __typeof__(&gr_reduce) p_reduce;
static __typeof__(&gr_ndim) p_ndim;
static __typeof__(&gr_shape) p_shape;

static PyObject* hook_binary;   /* (op, a, b) -> Array, for operands this file does not marshal */
static PyObject* hook_getitem;  /* (a, key) -> Array */
static PyObject* hook_setitem;  /* (a, key, value) -> None */
static PyObject* hook_pow;      /* (a, e) -> Array */
static PyObject* hook_reduce;   /* (op, a, axis, keepdims) -> Array */
static PyObject* str_addr;
static PyObject* str_check;

#define IS_ARRAY(o) PyObject_TypeCheck((o), &ArrayBase_Type)

/* Address of the gr_ctx behind a Context object; NULL with an exception set if it is closed. */
static gr_ctx* ctx_of(PyObject* ctx) {
  PyObject* a = PyObject_GetAttr(ctx, str_addr);
  if (!a) return NULL;
  void* p = PyLong_AsVoidPtr(a);
  Py_DECREF(a);
  if (!p && !PyErr_Occurred()) PyErr_SetString(PyExc_RuntimeError, "the context of this array has been closed");
  return (gr_ctx*)p;
}

/* Raises the binding's error for a non-zero status (Context.check does). */
static PyObject* raise_status(PyObject* ctx, int st) {
  PyObject* code = PyLong_FromLong(st);
  if (!code) return NULL;
  PyObject* r = PyObject_CallMethodObjArgs(ctx, str_check, code, NULL);
  Py_DECREF(code);
  if (r) { Py_DECREF(r); PyErr_SetString(PyExc_RuntimeError, "library call failed"); }
  return NULL;
}

/* The recorded DAG outlives the handles of its leaves (z = ctx.array(tensor) * 2 drops the leaf's handle at
 * once), so every result carries what its operands carry: one owner as it is, two different ones as a pair. */
static PyObject* merged_owner(PyObject* a, PyObject* b) {
  if (a == Py_None) a = NULL;
  if (b == Py_None) b = NULL;
  if (!a) { Py_XINCREF(b); return b; }
  if (!b || a == b) { Py_INCREF(a); return a; }
  return PyTuple_Pack(2, a, b);
}

static PyObject* new_array(PyTypeObject* type, PyObject* ctx, unsigned long long h, PyObject* owner_a, PyObject* owner_b, int view) {
  ArrayObject* a = (ArrayObject*)type->tp_alloc(type, 0);
  PyObject* owner = NULL;
  if (a && (owner_a || owner_b)) {
    owner = merged_owner(owner_a, owner_b);
    if (!owner && PyErr_Occurred()) { Py_DECREF(a); a = NULL; }
  }
  if (!a) {
    gr_ctx* c = ctx_of(ctx);
    if (c) p_release(c, h); else PyErr_Clear();
    return PyErr_NoMemory();
  }
  Py_INCREF(ctx);
  a->ctx = ctx;
  a->h = h;
  a->owner = owner;
  a->view = (char)view;
  return (PyObject*)a;
}

static int array_init(ArrayObject* self, PyObject* args, PyObject* kw) {
  PyObject* ctx;
  unsigned long long h;
  if (kw && PyDict_Size(kw)) { PyErr_SetString(PyExc_TypeError, "Array(ctx, handle)"); return -1; }
  if (!PyArg_ParseTuple(args, "OK", &ctx, &h)) return -1;
  Py_INCREF(ctx);
  Py_XSETREF(self->ctx, ctx);
  self->h = h;
  return 0;
}

static void array_dealloc(ArrayObject* self) {
  if (self->ctx) {
    PyObject *et, *ev, *tb;
    PyErr_Fetch(&et, &ev, &tb);
    PyObject* a = PyObject_GetAttr(self->ctx, str_addr);
    if (a) {
      void* p = PyLong_AsVoidPtr(a);
      Py_DECREF(a);
      if (p && p_release) p_release((gr_ctx*)p, self->h);
    }
    PyErr_Clear();
    PyErr_Restore(et, ev, tb);
  }
  Py_CLEAR(self->ctx);
  Py_CLEAR(self->owner);
  Py_TYPE(self)->tp_free((PyObject*)self);
}

/* A Python number as the library's scalar: 1 = taken, 0 = not a plain number (use the hook). */
static int as_scalar(PyObject* o, double* v, int* is_int) {
  if (PyFloat_CheckExact(o)) { *v = PyFloat_AS_DOUBLE(o); *is_int = 0; return 1; }
  if (PyLong_CheckExact(o)) {
    double d = PyLong_AsDouble(o);
    if (d == -1.0 && PyErr_Occurred()) { PyErr_Clear(); return 0; }
    *v = d; *is_int = 1;
    return 1;
  }
  return 0;
}

static PyObject* do_binary(int op, PyObject* a, PyObject* b) {
  gr_array out = 0;
  int st;
  if (IS_ARRAY(a)) {
    ArrayObject* x = (ArrayObject*)a;
    if (IS_ARRAY(b)) {
      ArrayObject* y = (ArrayObject*)b;
      if (x->ctx != y->ctx) { PyErr_SetString(PyExc_ValueError, "arrays belong to different contexts"); return NULL; }
      gr_ctx* c = ctx_of(x->ctx);
      if (!c) return NULL;
      st = p_binary(c, (gr_op)op, x->h, y->h, &out);
    } else {
      double v; int is_int;
      if (!as_scalar(b, &v, &is_int)) return PyObject_CallFunction(hook_binary, "iOO", op, a, b);
      gr_ctx* c = ctx_of(x->ctx);
      if (!c) return NULL;
      st = p_binary_scalar(c, (gr_op)op, x->h, v, is_int, 0, &out);
    }
    if (st) return raise_status(x->ctx, st);
    return new_array(Py_TYPE(a), x->ctx, out, x->owner, IS_ARRAY(b) ? ((ArrayObject*)b)->owner : NULL, 0);
  }
  if (IS_ARRAY(b)) {
    ArrayObject* y = (ArrayObject*)b;
    double v; int is_int;
    if (!as_scalar(a, &v, &is_int)) return PyObject_CallFunction(hook_binary, "iOO", op, a, b);
    gr_ctx* c = ctx_of(y->ctx);
    if (!c) return NULL;
    st = p_binary_scalar(c, (gr_op)op, y->h, v, is_int, 1, &out);
    if (st) return raise_status(y->ctx, st);
    return new_array(Py_TYPE(b), y->ctx, out, y->owner, NULL, 0);
  }
  return PyObject_CallFunction(hook_binary, "iOO", op, a, b);
}

static PyObject* do_unary(int op, PyObject* a) {
  if (!IS_ARRAY(a)) { PyErr_SetString(PyExc_TypeError, "no array operand"); return NULL; }
  ArrayObject* x = (ArrayObject*)a;
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  gr_array out = 0;
  int st = p_unary(c, (gr_op)op, x->h, &out);
  if (st) return raise_status(x->ctx, st);
  return new_array(Py_TYPE(a), x->ctx, out, x->owner, NULL, 0);
}

static PyObject* nb_add(PyObject* a, PyObject* b) { return do_binary(GR_ADD, a, b); }
static PyObject* nb_sub(PyObject* a, PyObject* b) { return do_binary(GR_SUB, a, b); }
static PyObject* nb_mul(PyObject* a, PyObject* b) { return do_binary(GR_MUL, a, b); }
static PyObject* nb_div(PyObject* a, PyObject* b) { return do_binary(GR_DIV, a, b); }
static PyObject* nb_neg(PyObject* a) { return do_unary(GR_NEG, a); }
static PyObject* nb_abs(PyObject* a) { return do_unary(GR_ABS, a); }

static PyObject* nb_pow(PyObject* a, PyObject* e, PyObject* mod) {
  if (mod == Py_None && IS_ARRAY(a) && PyLong_CheckExact(e)) {
    int overflow = 0;
    long v = PyLong_AsLongAndOverflow(e, &overflow);
    if (!overflow && v == 2) return do_unary(GR_SQUARE, a);  /* NumPy evaluates x**2 as square(x) */
  }
  return PyObject_CallFunction(hook_pow, "OO", a, e);
}

static PyObject* nb_matmul(PyObject* a, PyObject* b) {
  if (!IS_ARRAY(a) || !IS_ARRAY(b)) { PyErr_SetString(PyExc_TypeError, "dot: both operands must be arrays"); return NULL; }
  ArrayObject *x = (ArrayObject*)a, *y = (ArrayObject*)b;
  if (x->ctx != y->ctx) { PyErr_SetString(PyExc_ValueError, "arrays belong to different contexts"); return NULL; }
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  gr_array out = 0;
  int st = p_dot(c, x->h, y->h, &out);
  if (st) return raise_status(x->ctx, st);
  return new_array(Py_TYPE(a), x->ctx, out, x->owner, y->owner, 0);
}

/* Index key -> gr_slice arguments.  1 = parsed, 0 = not a tuple of slices of ints (use the hook), -1 = error. */
static int parse_key(PyObject* key, int* n, int64_t* start, int64_t* stop, int64_t* step, uint8_t* hs, uint8_t* he) {
  PyObject* single[1] = {key};
  PyObject** items = single;
  Py_ssize_t cnt = 1;
  if (PyTuple_Check(key)) { items = &PyTuple_GET_ITEM(key, 0); cnt = PyTuple_GET_SIZE(key); }
  if (cnt > GR_MAX_NDIM) return 0;
  for (Py_ssize_t d = 0; d < cnt; ++d) {
    if (!PySlice_Check(items[d])) return 0;
    PySliceObject* s = (PySliceObject*)items[d];
    PyObject* parts[3] = {s->start, s->stop, s->step};
    long long v[3] = {0, 0, 1};
    for (int q = 0; q < 3; ++q) {
      if (parts[q] == Py_None) continue;
      if (!PyLong_Check(parts[q])) return 0;
      int overflow = 0;
      v[q] = PyLong_AsLongLongAndOverflow(parts[q], &overflow);
      if (overflow) return 0;
      if (v[q] == -1 && PyErr_Occurred()) return -1;
    }
    start[d] = v[0]; stop[d] = v[1]; step[d] = v[2];
    hs[d] = s->start != Py_None; he[d] = s->stop != Py_None;
  }
  *n = (int)cnt;
  return 1;
}

static PyObject* array_subscript(PyObject* a, PyObject* key) {
  ArrayObject* x = (ArrayObject*)a;
  int64_t start[GR_MAX_NDIM], stop[GR_MAX_NDIM], step[GR_MAX_NDIM];
  uint8_t hs[GR_MAX_NDIM], he[GR_MAX_NDIM];
  int n = 0;
  int ok = parse_key(key, &n, start, stop, step, hs, he);
  if (ok < 0) return NULL;
  if (!ok) return PyObject_CallFunction(hook_getitem, "OO", a, key);
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  gr_array out = 0;
  int st = p_slice(c, x->h, n, start, stop, step, hs, he, &out);
  if (st) return raise_status(x->ctx, st);
  return new_array(Py_TYPE(a), x->ctx, out, x->owner, NULL, 1);
}

static int array_ass_subscript(PyObject* a, PyObject* key, PyObject* value) {
  ArrayObject* x = (ArrayObject*)a;
  if (!value) { PyErr_SetString(PyExc_TypeError, "array elements cannot be deleted"); return -1; }
  int64_t start[GR_MAX_NDIM], stop[GR_MAX_NDIM], step[GR_MAX_NDIM];
  uint8_t hs[GR_MAX_NDIM], he[GR_MAX_NDIM];
  int n = 0;
  int ok = IS_ARRAY(value) && ((ArrayObject*)value)->ctx == x->ctx ? parse_key(key, &n, start, stop, step, hs, he) : 0;
  if (ok < 0) return -1;
  if (!ok) {
    PyObject* r = PyObject_CallFunction(hook_setitem, "OOO", a, key, value);
    if (!r) return -1;
    Py_DECREF(r);
    return 0;
  }
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return -1;
  gr_array dst = 0;
  int st = p_slice(c, x->h, n, start, stop, step, hs, he, &dst);
  if (!st) {
    st = p_assign(c, dst, ((ArrayObject*)value)->h);
    p_release(c, dst);
  }
  if (st) { raise_status(x->ctx, st); return -1; }
  return 0;
}

static PyObject* array_materialize(PyObject* a, PyObject* unused) {
  ArrayObject* x = (ArrayObject*)a;
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  int st = p_materialize(c, x->h);
  if (st) return raise_status(x->ctx, st);
  if (!x->view) Py_CLEAR(x->owner);  /* the node now has storage of its own and has let go of its inputs */
  Py_INCREF(a);
  return a;
}

/* _materialize_into(address, bytes, tensor, static): gr_materialize_into (or its non-allocating variant) into the
 * caller's buffer.  An array that had no storage is bound to that buffer and lets go of its inputs: the tensor
 * becomes what keeps it alive.  One that had storage (and every view) is only copied and keeps what it had. */
static PyObject* array_materialize_into(PyObject* a, PyObject* args) {
  ArrayObject* x = (ArrayObject*)a;
  unsigned long long ptr, nbytes;
  PyObject* tensor;
  int is_static = 0;
  if (!PyArg_ParseTuple(args, "KKO|p", &ptr, &nbytes, &tensor, &is_static)) return NULL;
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  int had = 1;
  if (!x->view) {
    int st0 = p_is_materialized(c, x->h, &had);
    if (st0) return raise_status(x->ctx, st0);
  }
  int st = (is_static ? p_materialize_into_static : p_materialize_into)(c, x->h, (void*)(uintptr_t)ptr, (size_t)nbytes);
  if (st) return raise_status(x->ctx, st);
  if (!had) { Py_INCREF(tensor); Py_XSETREF(x->owner, tensor); }
  Py_INCREF(a);
  return a;
}

static PyObject* array_T(PyObject* a, void* unused) {
  ArrayObject* x = (ArrayObject*)a;
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  gr_array out = 0;
  int st = p_transpose(c, x->h, NULL, &out);
  if (st) return raise_status(x->ctx, st);
  return new_array(Py_TYPE(a), x->ctx, out, x->owner, NULL, 1);
}

static PyObject* array_ndim(PyObject* a, void* unused) {
  ArrayObject* x = (ArrayObject*)a;
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  int n = 0;
  int st = p_ndim(c, x->h, &n);
  if (st) return raise_status(x->ctx, st);
  return PyLong_FromLong(n);
}

static PyObject* array_shape(PyObject* a, void* unused) {
  ArrayObject* x = (ArrayObject*)a;
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  int n = 0;
  int64_t shape[GR_MAX_NDIM];
  int st = p_ndim(c, x->h, &n);
  if (!st) st = p_shape(c, x->h, shape);
  if (st) return raise_status(x->ctx, st);
  PyObject* t = PyTuple_New(n);
  if (!t) return NULL;
  for (int d = 0; d < n; ++d) {
    PyObject* v = PyLong_FromLongLong(shape[d]);
    if (!v) { Py_DECREF(t); return NULL; }
    PyTuple_SET_ITEM(t, d, v);
  }
  return t;
}

/* reduce(op, a, axis, keepdims): axis None (all axes), an int, or a sequence of ints */
static PyObject* mod_reduce(PyObject* m, PyObject* args) {
  int op, keep;
  PyObject *a, *axis;
  if (!PyArg_ParseTuple(args, "iOOp", &op, &a, &axis, &keep)) return NULL;
  if (!IS_ARRAY(a)) { PyErr_SetString(PyExc_TypeError, "no array operand"); return NULL; }
  ArrayObject* x = (ArrayObject*)a;
  int axes[GR_MAX_NDIM + 1], n = 0;
  if (axis == Py_None) n = 0;
  else if (PyLong_Check(axis)) {
    axes[0] = (int)PyLong_AsLong(axis);
    if (PyErr_Occurred()) return NULL;
    n = 1;
  } else {
    PyObject* seq = PySequence_Fast(axis, "axis must be None, an int or a sequence of ints");
    if (!seq) return NULL;
    Py_ssize_t cnt = PySequence_Fast_GET_SIZE(seq);
    if (cnt == 0 || cnt > GR_MAX_NDIM) {
      Py_DECREF(seq);
      return PyObject_CallFunction(hook_reduce, "iOOi", op, a, axis, keep);
    }
    for (Py_ssize_t i = 0; i < cnt; ++i) {
      axes[i] = (int)PyLong_AsLong(PySequence_Fast_GET_ITEM(seq, i));
      if (PyErr_Occurred()) { Py_DECREF(seq); return NULL; }
    }
    n = (int)cnt;
    Py_DECREF(seq);
  }
  gr_ctx* c = ctx_of(x->ctx);
  if (!c) return NULL;
  gr_array out = 0;
  int st = p_reduce(c, (gr_op)op, x->h, axes, n, keep, &out);
  if (st) return raise_status(x->ctx, st);
  return new_array(Py_TYPE(a), x->ctx, out, x->owner, NULL, 0);
}

/* program_run(program address, tuple of input addresses, output address) -> status: gr_program_run without
 * ctypes in between (a replayed request of a small array costs less than marshalling its arguments twice) */
static PyObject* mod_program_run(PyObject* m, PyObject* args) {
  unsigned long long prog, out;
  PyObject* ptrs;
  if (!PyArg_ParseTuple(args, "KO!K", &prog, &PyTuple_Type, &ptrs, &out)) return NULL;
  void* v[64];
  Py_ssize_t n = PyTuple_GET_SIZE(ptrs);
  if (n > 64) { PyErr_SetString(PyExc_ValueError, "more than 64 inputs"); return NULL; }
  for (Py_ssize_t i = 0; i < n; ++i) {
    v[i] = PyLong_AsVoidPtr(PyTuple_GET_ITEM(ptrs, i));
    if (!v[i] && PyErr_Occurred()) return NULL;
  }
  return PyLong_FromLong(p_program_run((gr_program*)(uintptr_t)prog, v, (void*)(uintptr_t)out));
}

static PyNumberMethods array_as_number = {
    .nb_add = nb_add, .nb_subtract = nb_sub, .nb_multiply = nb_mul, .nb_true_divide = nb_div,
    .nb_negative = nb_neg, .nb_absolute = nb_abs, .nb_power = nb_pow, .nb_matrix_multiply = nb_matmul,
};
static PyMappingMethods array_as_mapping = {.mp_subscript = array_subscript, .mp_ass_subscript = array_ass_subscript};
static PyMethodDef array_methods[] = {
    {"materialize", array_materialize, METH_NOARGS, "Evaluates the node (gr_materialize) and returns self."},
    {"_materialize_into", array_materialize_into, METH_VARARGS, "Evaluates the node into a caller's buffer (gr_materialize_into[_static]) and returns self."},
    {NULL, NULL, 0, NULL}};
static PyMemberDef array_members[] = {
    {"ctx", T_OBJECT, offsetof(ArrayObject, ctx), READONLY, "the Context the node belongs to"},
    {"h", T_ULONGLONG, offsetof(ArrayObject, h), READONLY, "the node's handle"},
    {"_owner", T_OBJECT, offsetof(ArrayObject, owner), 0, "keeps alive the device memory of the leaves this node still reads"},
    {"_view", T_BOOL, offsetof(ArrayObject, view), 0, "a slice or transpose (reads its base's storage also once evaluated)"},
    {NULL, 0, 0, 0, NULL}};
static PyGetSetDef array_getset[] = {{"T", array_T, NULL, "transposed view (axes reversed)", NULL},
                                     {"ndim", array_ndim, NULL, "number of dimensions", NULL},
                                     {"shape", array_shape, NULL, "extents", NULL},
                                     {NULL, NULL, NULL, NULL, NULL}};

static PyTypeObject ArrayBase_Type = {
    PyVarObject_HEAD_INIT(NULL, 0)
    .tp_name = "paper_1901_03771_amd._fastbind.ArrayBase",
    .tp_basicsize = sizeof(ArrayObject),
    .tp_dealloc = (destructor)array_dealloc,
    .tp_as_number = &array_as_number,
    .tp_as_mapping = &array_as_mapping,
    .tp_flags = Py_TPFLAGS_DEFAULT | Py_TPFLAGS_BASETYPE,
    .tp_doc = "Handle of one DAG node (fast paths of the recording calls).",
    .tp_methods = array_methods,
    .tp_members = array_members,
    .tp_getset = array_getset,
    .tp_init = (initproc)array_init,
    .tp_new = PyType_GenericNew,
};

/* ---- module ----------------------------------------------------------------------------- */

static PyObject* mod_unary(PyObject* m, PyObject* args) {
  int op;
  PyObject* a;
  if (!PyArg_ParseTuple(args, "iO", &op, &a)) return NULL;
  return do_unary(op, a);
}

static PyObject* mod_binary(PyObject* m, PyObject* args) {
  int op;
  PyObject *a, *b;
  if (!PyArg_ParseTuple(args, "iOO", &op, &a, &b)) return NULL;
  return do_binary(op, a, b);
}

static int take_address(PyObject* d, const char* name, void** out) {
  PyObject* v = PyDict_GetItemString(d, name);
  if (!v) { PyErr_Format(PyExc_KeyError, "bind: address of %s is missing", name); return 0; }
  *out = PyLong_AsVoidPtr(v);
  if (!*out) { if (!PyErr_Occurred()) PyErr_Format(PyExc_ValueError, "bind: %s is NULL", name); return 0; }
  return 1;
}

static PyObject* mod_bind(PyObject* m, PyObject* d) {
  if (!PyDict_Check(d)) { PyErr_SetString(PyExc_TypeError, "bind(dict of entry point addresses)"); return NULL; }
  if (!take_address(d, "gr_unary", (void**)&p_unary) || !take_address(d, "gr_binary", (void**)&p_binary) ||
      !take_address(d, "gr_binary_scalar", (void**)&p_binary_scalar) || !take_address(d, "gr_slice", (void**)&p_slice) ||
      !take_address(d, "gr_transpose", (void**)&p_transpose) || !take_address(d, "gr_dot", (void**)&p_dot) ||
      !take_address(d, "gr_assign", (void**)&p_assign) || !take_address(d, "gr_materialize", (void**)&p_materialize) ||
      !take_address(d, "gr_release", (void**)&p_release) || !take_address(d, "gr_reduce", (void**)&p_reduce) ||
      !take_address(d, "gr_ndim", (void**)&p_ndim) || !take_address(d, "gr_shape", (void**)&p_shape) ||
      !take_address(d, "gr_materialize_into", (void**)&p_materialize_into) ||
      !take_address(d, "gr_materialize_into_static", (void**)&p_materialize_into_static) ||
      !take_address(d, "gr_is_materialized", (void**)&p_is_materialized) ||
      !take_address(d, "gr_program_run", (void**)&p_program_run))
    return NULL;
  Py_RETURN_NONE;
}

static PyObject* mod_set_hooks(PyObject* m, PyObject* args) {
  PyObject *b, *g, *s, *p, *r;
  if (!PyArg_ParseTuple(args, "OOOOO", &b, &g, &s, &p, &r)) return NULL;
  Py_INCREF(r); Py_XSETREF(hook_reduce, r);
  Py_INCREF(b); Py_XSETREF(hook_binary, b);
  Py_INCREF(g); Py_XSETREF(hook_getitem, g);
  Py_INCREF(s); Py_XSETREF(hook_setitem, s);
  Py_INCREF(p); Py_XSETREF(hook_pow, p);
  Py_RETURN_NONE;
}

static PyMethodDef module_methods[] = {
    {"unary", mod_unary, METH_VARARGS, "unary(op, a): gr_unary"},
    {"binary", mod_binary, METH_VARARGS, "binary(op, a, b): gr_binary / gr_binary_scalar"},
    {"reduce", mod_reduce, METH_VARARGS, "reduce(op, a, axis, keepdims): gr_reduce"},
    {"program_run", mod_program_run, METH_VARARGS, "program_run(program, input addresses, output address) -> status: gr_program_run"},
    {"bind", mod_bind, METH_O, "bind({name: address}): entry points of the loaded library"},
    {"set_hooks", mod_set_hooks, METH_VARARGS, "set_hooks(binary, getitem, setitem, pow, reduce): Python fallbacks"},
    {NULL, NULL, 0, NULL}};

static struct PyModuleDef moduledef = {PyModuleDef_HEAD_INIT, "_fastbind", "Fast paths of the lazy-array binding.", -1, module_methods};

PyMODINIT_FUNC PyInit__fastbind(void) {
  if (PyType_Ready(&ArrayBase_Type) < 0) return NULL;
  PyObject* m = PyModule_Create(&moduledef);
  if (!m) return NULL;
  str_addr = PyUnicode_InternFromString("_addr");
  str_check = PyUnicode_InternFromString("check");
  Py_INCREF(&ArrayBase_Type);
  if (PyModule_AddObject(m, "ArrayBase", (PyObject*)&ArrayBase_Type) < 0) { Py_DECREF(&ArrayBase_Type); Py_DECREF(m); return NULL; }
  return m;
}
