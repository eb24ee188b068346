// ORACLE -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, eager CPU evaluator of NumPy-style array operations: every
// compute op materialises one fresh C-contiguous host array, exactly the
// execution model the paper sets out to replace (Section 1: each operation is
// executed eagerly and its result array is stored; Section 2: "the semantics
// of all operations match the semantics of the corresponding numpy
// operations", broadcasting included).  Fusion must reach the same values as
// this op-by-op evaluation, so this evaluator is the definition the GPU path
// is compared against.
//
// Only tests, the smoke check and the bench's cpu_baseline leg may use this
// file.  It shares no code with the GPU library and includes none of its
// headers.  All parity pins for the functions below live in tests/ (closed
// forms, brute force on tiny arrays, the paper's worked example of Listing 1,
// NumPy as a third opinion); no function here is "parity unpinned".
//
// Arithmetic rules (one per op, nothing reordered or fused):
//   * f32 + - * / neg abs sqrt square maximum minimum: one IEEE-754 binary32
//     round-to-nearest operation per op (square(x) = x*x).  Build with
//     -ffp-contract=off and without fast-math.
//   * f32 exp log tanh erf: evaluated in binary64 libm, rounded once to binary32.
//   * i32 + - * neg abs square: two's-complement wrap-around.
//   * maximum/minimum: NaN-propagating, as NumPy's.
//   * sum of f32 over axes: binary64 accumulator, elements taken in row-major
//     index order, rounded once to binary32.  sum of i32: exact in int64
//     (NumPy's default result type on Linux).  max/min: exact.
//   * dot: binary64 accumulator over k in index order, rounded once.
//   * cumulative sum / max / min along one axis (the map-scan primitive of
//     Section 3.2): f32 running sum kept in binary64, every prefix rounded
//     once to binary32; i32 running sum exact in int64; max/min exact.
//   * slice assignment dst[...] = value (Listing 6): the value is a finished
//     array (eager evaluation), then copied element by element into the view;
//     every view of the same buffer sees the new contents, as in NumPy.
//   * slice / transpose: views (offset + strides), no data touched
//     (Section 3.1: index translation for slicing and transpose (i,j)->(j,i)).
//   * reshape (Section 2 lists it with the n-D transpose): a fresh C-contiguous
//     array holding the operand's elements in row-major order under the new
//     shape; always a copy (NumPy returns a view where it can; the values
//     are the same, only writes through the result differ).
//   * a "weak" scalar (a Python number) takes the array operand's dtype:
//     rounded to binary32 first when it meets an f32 array.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <memory>
#include <string>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { DT_F32 = 0, DT_I32 = 1, DT_I64 = 2, DT_WEAK = 3 };
enum { U_NEG = 0, U_ABS, U_EXP, U_LOG, U_SQRT, U_SQUARE, U_TANH, U_ERF };
enum { B_ADD = 0, B_SUB, B_MUL, B_DIV, B_MAXIMUM, B_MINIMUM };
enum { R_SUM = 0, R_MAX, R_MIN };
const int MAXD = 8;

struct Arr {
  int dtype = DT_F32;
  int ndim = 0;
  int64_t shape[MAXD] = {0};
  int64_t strides[MAXD] = {0};  // in elements
  int64_t offset = 0;           // in elements
  std::shared_ptr<std::vector<unsigned char>> buf;
  // weak scalar payload (dtype == DT_WEAK)
  double weak_value = 0.0;
  int weak_is_int = 0;
};

thread_local std::string g_err;
int g_threads = 1;

int64_t itemsize(int dt) { return dt == DT_I64 ? 8 : 4; }

int64_t count(const Arr* a) {
  int64_t n = 1;
  for (int d = 0; d < a->ndim; ++d) n *= a->shape[d];
  return n;
}

Arr* fresh(int dtype, int ndim, const int64_t* shape) {
  Arr* r = new Arr();
  r->dtype = dtype;
  r->ndim = ndim;
  int64_t n = 1;
  for (int d = ndim - 1; d >= 0; --d) {
    r->shape[d] = shape[d];
    r->strides[d] = n;
    n *= shape[d];
  }
  r->buf = std::make_shared<std::vector<unsigned char>>((size_t)(n > 0 ? n : 1) * itemsize(dtype));
  return r;
}

template <class T>
T* base(const Arr* a) { return reinterpret_cast<T*>(a->buf->data()); }

// Row-major linear index -> multi-index of `shape`.
void unravel(int64_t lin, int ndim, const int64_t* shape, int64_t* idx) {
  for (int d = ndim - 1; d >= 0; --d) {
    int64_t s = shape[d];
    idx[d] = s ? lin % s : 0;
    lin = s ? lin / s : 0;
  }
}

// Element offset of operand `a` for output multi-index idx (rank ondim),
// under NumPy broadcasting: shapes right-aligned, a size-1 dim reads index 0.
int64_t bcast_offset(const Arr* a, int ondim, const int64_t* idx) {
  int64_t off = a->offset;
  int shift = ondim - a->ndim;
  for (int d = 0; d < a->ndim; ++d) {
    int64_t i = (a->shape[d] == 1) ? 0 : idx[d + shift];
    off += i * a->strides[d];
  }
  return off;
}

// NumPy broadcast of two shapes; false if incompatible.
bool broadcast_shapes(const Arr* a, const Arr* b, int* ondim, int64_t* oshape) {
  int n = a->ndim > b->ndim ? a->ndim : b->ndim;
  for (int d = 0; d < n; ++d) {
    int da = d - (n - a->ndim), db = d - (n - b->ndim);
    int64_t sa = da >= 0 ? a->shape[da] : 1;
    int64_t sb = db >= 0 ? b->shape[db] : 1;
    if (sa == sb) oshape[d] = sa;
    else if (sa == 1) oshape[d] = sb;
    else if (sb == 1) oshape[d] = sa;
    else return false;
  }
  *ondim = n;
  return true;
}

float f32_unary(int op, float x) {
  switch (op) {
    case U_NEG: return -x;
    case U_ABS: return std::fabs(x);
    case U_EXP: return (float)std::exp((double)x);
    case U_LOG: return (float)std::log((double)x);
    case U_SQRT: return std::sqrt(x);
    case U_SQUARE: return x * x;
    case U_TANH: return (float)std::tanh((double)x);
    case U_ERF: return (float)std::erf((double)x);
  }
  return 0.f;
}

int32_t i32_unary(int op, int32_t x, bool* ok) {
  uint32_t u = (uint32_t)x;
  switch (op) {
    case U_NEG: return (int32_t)(0u - u);
    case U_ABS: return x < 0 ? (int32_t)(0u - u) : x;
    case U_SQUARE: return (int32_t)(u * u);
  }
  *ok = false;
  return 0;
}

float f32_binary(int op, float a, float b) {
  switch (op) {
    case B_ADD: return a + b;
    case B_SUB: return a - b;
    case B_MUL: return a * b;
    case B_DIV: return a / b;
    case B_MAXIMUM: return (a >= b || a != a) ? a : b;
    case B_MINIMUM: return (a <= b || a != a) ? a : b;
  }
  return 0.f;
}

int32_t i32_binary(int op, int32_t a, int32_t b, bool* ok) {
  uint32_t ua = (uint32_t)a, ub = (uint32_t)b;
  switch (op) {
    case B_ADD: return (int32_t)(ua + ub);
    case B_SUB: return (int32_t)(ua - ub);
    case B_MUL: return (int32_t)(ua * ub);
    case B_MAXIMUM: return a >= b ? a : b;
    case B_MINIMUM: return a <= b ? a : b;
  }
  *ok = false;  // integer division is not part of the vocabulary
  return 0;
}

// A weak scalar becomes a rank-0 array of the partner's dtype.
Arr* harden(const Arr* w, int dtype) {
  if (dtype == DT_F32) {
    Arr* r = fresh(DT_F32, 0, nullptr);
    base<float>(r)[0] = (float)w->weak_value;
    return r;
  }
  if (dtype == DT_I32 && w->weak_is_int) {
    Arr* r = fresh(DT_I32, 0, nullptr);
    base<int32_t>(r)[0] = (int32_t)(int64_t)w->weak_value;
    return r;
  }
  return nullptr;
}

int normalize_axes(int ndim, const int* axes, int naxes, bool* red) {
  for (int d = 0; d < ndim; ++d) red[d] = (naxes == 0);
  for (int k = 0; k < naxes; ++k) {
    int ax = axes[k] < 0 ? axes[k] + ndim : axes[k];
    if (ax < 0 || ax >= ndim || red[ax]) return -1;
    red[ax] = true;
  }
  return 0;
}

}  // namespace

extern "C" {

const char* ora_last_error() { return g_err.c_str(); }

void ora_set_threads(int n) { g_threads = n > 0 ? n : 1; }
int ora_get_threads() {
#ifdef _OPENMP
  return g_threads;
#else
  return 1;
#endif
}

void ora_free(Arr* a) { delete a; }

// Copies `data` (C-contiguous, `shape`) into a new host array.
Arr* ora_from_host(const void* data, int dtype, int ndim, const int64_t* shape) {
  if (ndim < 0 || ndim > MAXD || dtype < DT_F32 || dtype > DT_I64) { g_err = "bad dtype/ndim"; return nullptr; }
  Arr* r = fresh(dtype, ndim, shape);
  int64_t n = count(r);
  if (n > 0) std::memcpy(r->buf->data(), data, (size_t)n * itemsize(dtype));
  return r;
}

Arr* ora_scalar(double value, int is_int) {
  Arr* r = new Arr();
  r->dtype = DT_WEAK;
  r->weak_value = value;
  r->weak_is_int = is_int;
  return r;
}

int ora_ndim(const Arr* a) { return a->ndim; }
int ora_dtype(const Arr* a) { return a->dtype; }
void ora_shape(const Arr* a, int64_t* shape) { for (int d = 0; d < a->ndim; ++d) shape[d] = a->shape[d]; }

// Writes the array's elements to dst in C order.
void ora_copy_out(const Arr* a, void* dst) {
  int64_t n = count(a);
  int64_t isz = itemsize(a->dtype);
  const unsigned char* src = a->buf->data();
  unsigned char* out = (unsigned char*)dst;
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[MAXD];
    unravel(lin, a->ndim, a->shape, idx);
    int64_t off = a->offset;
    for (int d = 0; d < a->ndim; ++d) off += idx[d] * a->strides[d];
    std::memcpy(out + lin * isz, src + off * isz, (size_t)isz);
  }
}

Arr* ora_unary(int op, const Arr* a) {
  if (a->dtype == DT_WEAK || a->dtype == DT_I64) { g_err = "unary: unsupported dtype"; return nullptr; }
  if (a->dtype == DT_I32 && !(op == U_NEG || op == U_ABS || op == U_SQUARE)) { g_err = "unary: float op on int array"; return nullptr; }
  Arr* r = fresh(a->dtype, a->ndim, a->shape);
  int64_t n = count(r);
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[MAXD];
    unravel(lin, r->ndim, r->shape, idx);
    int64_t off = bcast_offset(a, r->ndim, idx);
    if (a->dtype == DT_F32) base<float>(r)[lin] = f32_unary(op, base<float>(a)[off]);
    else { bool ok = true; base<int32_t>(r)[lin] = i32_unary(op, base<int32_t>(a)[off], &ok); }
  }
  return r;
}

Arr* ora_binary(int op, const Arr* a_in, const Arr* b_in) {
  std::unique_ptr<Arr> ha, hb;
  const Arr* a = a_in;
  const Arr* b = b_in;
  if (a->dtype == DT_WEAK && b->dtype == DT_WEAK) { g_err = "binary: two weak scalars"; return nullptr; }
  if (a->dtype == DT_WEAK) { ha.reset(harden(a, b->dtype)); if (!ha) { g_err = "binary: float scalar with int array"; return nullptr; } a = ha.get(); }
  if (b->dtype == DT_WEAK) { hb.reset(harden(b, a->dtype)); if (!hb) { g_err = "binary: float scalar with int array"; return nullptr; } b = hb.get(); }
  if (a->dtype != b->dtype || a->dtype == DT_I64) { g_err = "binary: dtype mix not supported"; return nullptr; }
  if (a->dtype == DT_I32 && op == B_DIV) { g_err = "binary: integer division not supported"; return nullptr; }
  int ondim; int64_t oshape[MAXD];
  if (!broadcast_shapes(a, b, &ondim, oshape)) { g_err = "binary: shapes do not broadcast"; return nullptr; }
  Arr* r = fresh(a->dtype, ondim, oshape);
  int64_t n = count(r);
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[MAXD];
    unravel(lin, ondim, oshape, idx);
    int64_t oa = bcast_offset(a, ondim, idx), ob = bcast_offset(b, ondim, idx);
    if (a->dtype == DT_F32) base<float>(r)[lin] = f32_binary(op, base<float>(a)[oa], base<float>(b)[ob]);
    else { bool ok = true; base<int32_t>(r)[lin] = i32_binary(op, base<int32_t>(a)[oa], base<int32_t>(b)[ob], &ok); }
  }
  return r;
}

// Python slicing rules per dimension (step >= 1): negative start/stop count
// from the end, both are clamped to [0, n], missing means 0 / n.  Dimensions
// beyond `nspec` are taken whole.  The result is a view.
Arr* ora_slice(const Arr* a, int nspec, const int64_t* start, const int64_t* stop, const int64_t* step,
               const unsigned char* has_start, const unsigned char* has_stop) {
  if (a->dtype == DT_WEAK || nspec > a->ndim) { g_err = "slice: too many indices"; return nullptr; }
  Arr* r = new Arr(*a);
  for (int d = 0; d < nspec; ++d) {
    int64_t n = a->shape[d], st = step[d];
    if (st < 1) { delete r; g_err = "slice: step must be >= 1"; return nullptr; }
    int64_t lo = has_start[d] ? start[d] : 0;
    int64_t hi = has_stop[d] ? stop[d] : n;
    if (lo < 0) lo += n;
    if (hi < 0) hi += n;
    if (lo < 0) lo = 0;
    if (lo > n) lo = n;
    if (hi < 0) hi = 0;
    if (hi > n) hi = n;
    int64_t len = hi > lo ? (hi - lo + st - 1) / st : 0;
    r->shape[d] = len;
    r->offset += lo * a->strides[d];
    r->strides[d] = a->strides[d] * st;
  }
  return r;
}

// perm == NULL reverses the axes.  A view: element (i0..) of the result is
// element (i_perm^-1..) of the operand, i.e. (i,j) -> (j,i) in 2-D.
Arr* ora_transpose(const Arr* a, const int* perm) {
  if (a->dtype == DT_WEAK) { g_err = "transpose: weak scalar"; return nullptr; }
  Arr* r = new Arr(*a);
  bool seen[MAXD] = {false};
  for (int d = 0; d < a->ndim; ++d) {
    int p = perm ? perm[d] : a->ndim - 1 - d;
    if (p < 0) p += a->ndim;
    if (p < 0 || p >= a->ndim || seen[p]) { delete r; g_err = "transpose: bad permutation"; return nullptr; }
    seen[p] = true;
    r->shape[d] = a->shape[p];
    r->strides[d] = a->strides[p];
  }
  return r;
}

// Elements of `a` in row-major order, laid out under `shape` (same count; one
// extent may be -1 and is then inferred).  Always a copy.
Arr* ora_reshape(const Arr* a, int ndim, const int64_t* shape) {
  if (a->dtype == DT_WEAK || ndim < 0 || ndim > MAXD) { g_err = "reshape: bad operand or rank"; return nullptr; }
  int64_t want[MAXD], known = 1, n = count(a);
  int infer = -1;
  for (int d = 0; d < ndim; ++d) {
    want[d] = shape[d];
    if (shape[d] == -1) { if (infer >= 0) { g_err = "reshape: more than one inferred extent"; return nullptr; } infer = d; }
    else if (shape[d] < 0) { g_err = "reshape: negative extent"; return nullptr; }
    else known *= shape[d];
  }
  if (infer >= 0) {
    if (known == 0 || n % known) { g_err = "reshape: cannot infer the extent"; return nullptr; }
    want[infer] = n / known;
    known *= want[infer];
  }
  if (known != n) { g_err = "reshape: element counts differ"; return nullptr; }
  Arr* r = fresh(a->dtype, ndim, want);
  const int64_t isz = itemsize(a->dtype);
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[MAXD], off = a->offset;
    unravel(lin, a->ndim, a->shape, idx);
    for (int d = 0; d < a->ndim; ++d) off += idx[d] * a->strides[d];
    std::memcpy(r->buf->data() + lin * isz, a->buf->data() + off * isz, (size_t)isz);
  }
  return r;
}

// Reduction over `axes` (naxes == 0: all axes).
Arr* ora_reduce(int op, const Arr* a, const int* axes, int naxes, int keepdims) {
  if (a->dtype != DT_F32 && a->dtype != DT_I32) { g_err = "reduce: unsupported dtype"; return nullptr; }
  bool red[MAXD];
  if (normalize_axes(a->ndim, axes, naxes, red) != 0) { g_err = "reduce: bad axis"; return nullptr; }
  // Output shape, and the shape of the reduced sub-space.
  int ondim = 0; int64_t oshape[MAXD];
  int rndim = 0; int64_t rshape[MAXD]; int raxis[MAXD];
  int kaxis[MAXD]; int kndim = 0;
  for (int d = 0; d < a->ndim; ++d) {
    if (red[d]) { rshape[rndim] = a->shape[d]; raxis[rndim++] = d; if (keepdims) oshape[ondim++] = 1; }
    else { kaxis[kndim++] = d; oshape[ondim++] = a->shape[d]; }
  }
  int64_t rcount = 1;
  for (int d = 0; d < rndim; ++d) rcount *= rshape[d];
  if (rcount == 0 && op != R_SUM) { g_err = "reduce: max/min of an empty range"; return nullptr; }
  int out_dt = (a->dtype == DT_I32 && op == R_SUM) ? DT_I64 : a->dtype;
  Arr* r = fresh(out_dt, ondim, oshape);
  int64_t kshape[MAXD];
  for (int d = 0; d < kndim; ++d) kshape[d] = a->shape[kaxis[d]];
  int64_t n = count(r);
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t kidx[MAXD], ridx[MAXD];
    unravel(lin, kndim, kshape, kidx);
    int64_t off0 = a->offset;
    for (int d = 0; d < kndim; ++d) off0 += kidx[d] * a->strides[kaxis[d]];
    double facc = 0.0; int64_t iacc = 0; float fext = 0.f; int32_t iext = 0;
    for (int64_t k = 0; k < rcount; ++k) {
      unravel(k, rndim, rshape, ridx);
      int64_t off = off0;
      for (int d = 0; d < rndim; ++d) off += ridx[d] * a->strides[raxis[d]];
      if (a->dtype == DT_F32) {
        float v = base<float>(a)[off];
        if (op == R_SUM) facc += (double)v;
        else if (k == 0) fext = v;
        else fext = f32_binary(op == R_MAX ? B_MAXIMUM : B_MINIMUM, fext, v);
      } else {
        int32_t v = base<int32_t>(a)[off];
        if (op == R_SUM) iacc += (int64_t)v;
        else if (k == 0) iext = v;
        else iext = (op == R_MAX) ? (iext >= v ? iext : v) : (iext <= v ? iext : v);
      }
    }
    if (a->dtype == DT_F32) base<float>(r)[lin] = (op == R_SUM) ? (float)facc : fext;
    else if (op == R_SUM) base<int64_t>(r)[lin] = iacc;
    else base<int32_t>(r)[lin] = iext;
  }
  return r;
}

// dst[...] = value for a view `dst`; value must have dst's shape and element type.
int ora_assign(Arr* dst, const Arr* value) {
  if (dst->dtype == DT_WEAK || value->dtype != dst->dtype || value->ndim != dst->ndim) { g_err = "assign: dtype or rank differs"; return 1; }
  for (int d = 0; d < dst->ndim; ++d) if (dst->shape[d] != value->shape[d]) { g_err = "assign: shape differs"; return 1; }
  // the value may be a view of the destination's own buffer: finish reading before writing
  int64_t n = count(dst), isz = itemsize(dst->dtype);
  std::vector<unsigned char> tmp((size_t)(n > 0 ? n : 1) * isz);
  ora_copy_out(value, tmp.data());
  unsigned char* out = dst->buf->data();
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t lin = 0; lin < n; ++lin) {
    int64_t idx[MAXD];
    unravel(lin, dst->ndim, dst->shape, idx);
    int64_t off = dst->offset;
    for (int d = 0; d < dst->ndim; ++d) off += idx[d] * dst->strides[d];
    std::memcpy(out + off * isz, tmp.data() + lin * isz, (size_t)isz);
  }
  return 0;
}

// Inclusive scan along `axis` (np.cumsum / np.maximum.accumulate / np.minimum.accumulate).
Arr* ora_scan(int op, const Arr* a, int axis) {
  if (a->dtype != DT_F32 && a->dtype != DT_I32) { g_err = "scan: unsupported dtype"; return nullptr; }
  if (a->ndim < 1) { g_err = "scan: rank-0 operand"; return nullptr; }
  if (axis < 0) axis += a->ndim;
  if (axis < 0 || axis >= a->ndim) { g_err = "scan: bad axis"; return nullptr; }
  int out_dt = (a->dtype == DT_I32 && op == R_SUM) ? DT_I64 : a->dtype;
  Arr* r = fresh(out_dt, a->ndim, a->shape);
  // the lines along `axis`: one per index of the other dimensions
  int kndim = 0; int64_t kshape[MAXD]; int kaxis[MAXD];
  for (int d = 0; d < a->ndim; ++d) if (d != axis) { kshape[kndim] = a->shape[d]; kaxis[kndim++] = d; }
  int64_t lines = 1;
  for (int d = 0; d < kndim; ++d) lines *= kshape[d];
  int64_t len = a->shape[axis];
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t ln = 0; ln < lines; ++ln) {
    int64_t kidx[MAXD];
    unravel(ln, kndim, kshape, kidx);
    int64_t ain = a->offset, rout = 0;
    for (int d = 0; d < kndim; ++d) { ain += kidx[d] * a->strides[kaxis[d]]; rout += kidx[d] * r->strides[kaxis[d]]; }
    double facc = 0.0; int64_t iacc = 0; float fext = 0.f; int32_t iext = 0;
    for (int64_t j = 0; j < len; ++j) {
      int64_t src = ain + j * a->strides[axis], dst = rout + j * r->strides[axis];
      if (a->dtype == DT_F32) {
        float v = base<float>(a)[src];
        if (op == R_SUM) { facc += (double)v; base<float>(r)[dst] = (float)facc; }
        else { fext = j == 0 ? v : f32_binary(op == R_MAX ? B_MAXIMUM : B_MINIMUM, fext, v); base<float>(r)[dst] = fext; }
      } else {
        int32_t v = base<int32_t>(a)[src];
        if (op == R_SUM) { iacc += (int64_t)v; base<int64_t>(r)[dst] = iacc; }
        else { iext = j == 0 ? v : (op == R_MAX ? (iext >= v ? iext : v) : (iext <= v ? iext : v)); base<int32_t>(r)[dst] = iext; }
      }
    }
  }
  return r;
}

// np.dot for f32: (M,K).(K,) -> (M,), (K,).(K,) -> (), (M,K).(K,N) -> (M,N).
Arr* ora_dot(const Arr* a, const Arr* b) {
  if (a->dtype != DT_F32 || b->dtype != DT_F32) { g_err = "dot: f32 only"; return nullptr; }
  if (a->ndim < 1 || a->ndim > 2 || b->ndim < 1 || b->ndim > 2 || (a->ndim == 1 && b->ndim == 2)) { g_err = "dot: unsupported ranks"; return nullptr; }
  int64_t K = a->shape[a->ndim - 1];
  if (b->shape[0] != K) { g_err = "dot: inner dimensions differ"; return nullptr; }
  int64_t M = a->ndim == 2 ? a->shape[0] : 1;
  int64_t N = b->ndim == 2 ? b->shape[1] : 1;
  int ondim = 0; int64_t oshape[2];
  if (a->ndim == 2) oshape[ondim++] = M;
  if (b->ndim == 2) oshape[ondim++] = N;
  Arr* r = fresh(DT_F32, ondim, oshape);
  int64_t sam = a->ndim == 2 ? a->strides[0] : 0, sak = a->strides[a->ndim - 1];
  int64_t sbk = b->strides[0], sbn = b->ndim == 2 ? b->strides[1] : 0;
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t mn = 0; mn < M * N; ++mn) {
    int64_t m = mn / N, nn = mn % N;
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k)
      acc += (double)base<float>(a)[a->offset + m * sam + k * sak] * (double)base<float>(b)[b->offset + k * sbk + nn * sbn];
    base<float>(r)[mn] = (float)acc;
  }
  return r;
}

}  // extern "C"
