// DAG recorder: every array operation appends a node with inferred shape and
// element type instead of executing (Section 1: deferred execution; Section 2:
// "the size of the tensor represented by each node, and the data type of the
// tensor elements are computed automatically while the DAG is built").
// Nothing in this file touches the device.
#include <algorithm>
#include <cmath>
#include <cstdio>

#include "ctx.h"

namespace gr {

static thread_local std::string g_create_err;

gr_status fail(gr_ctx* c, gr_status s, const std::string& msg) {
  if (c) c->err = msg; else g_create_err = msg;
  return s;
}

Node* lookup(gr_ctx* c, gr_array a) {
  auto it = c->nodes.find(a);
  if (it == c->nodes.end() || it->second->handle_refs <= 0) return nullptr;
  return it->second;
}

// Element counts and element offsets stay below 2^40 so that byte offsets and every product of two
// extents the planner forms fit int64 with room to spare (288 GB of HBM holds 2^36 f32 elements).
// Zero extents count as one: reducing an empty axis away leaves the other extents as the result.
constexpr int64_t MAX_COUNT = int64_t(1) << 40;

bool count_fits(const int64_t* shape, int ndim) {
  int64_t n = 1;
  for (int d = 0; d < ndim; ++d) {
    if (shape[d] <= 0) continue;
    if (shape[d] > MAX_COUNT || n > MAX_COUNT / shape[d]) return false;
    n *= shape[d];
  }
  return true;
}

Node* new_node(gr_ctx* c, Kind kind) {
  Node* n = new Node();
  n->id = c->next_id++;
  n->kind = kind;
  n->handle_refs = 1;
  c->nodes[n->id] = n;
  c->stats.nodes_recorded++;
  c->stats.nodes_alive++;
  return n;
}

static void add_input(Node* n, Node* in) {
  n->in.push_back(in);
  in->consumer_refs++;
}

static void forget_pending(gr_ctx* c, const Node* n) {
  auto range = c->pending_expensive.equal_range(n->shash);
  for (auto it = range.first; it != range.second; ++it)
    if (it->second == n->id) { c->pending_expensive.erase(it); return; }
}

// Frees every node that has lost its last reference, iteratively.
void node_maybe_free(gr_ctx* c, Node* n0) {
  std::vector<Node*> work{n0};
  while (!work.empty()) {
    Node* n = work.back();
    work.pop_back();
    if (n->handle_refs > 0 || n->consumer_refs > 0) continue;
    for (Node* p : n->in) {
      // a predecessor is queued exactly once: when it loses its last reference
      if (--p->consumer_refs == 0 && p->handle_refs == 0) work.push_back(p);
    }
    n->in.clear();
    if (n->owns_data && n->data) {
      // a value that was assigned directly into this array's storage may outlive the array: the
      // buffer then passes to it instead of being freed
      Node* heir = nullptr;
      if (c->any_storage_alias)
        for (auto& kv : c->nodes) {
          Node* m = kv.second;
          if (m != n && m->materialized && m->cow_alias && m->data == n->data) { heir = m; break; }
        }
      if (heir) { heir->owns_data = true; heir->alloc_bytes = n->alloc_bytes; heir->cow_alias = false; }
      else ctx_free(c, n->data, n->alloc_bytes);
    }
    if (n->shadow && n->shadow != n->lent) ctx_free(c, n->shadow, n->alloc_bytes);
    if (n->kind == Kind::REDUCE || n->kind == Kind::DOT || n->kind == Kind::SCAN) forget_pending(c, n);
    c->nodes.erase(n->id);
    c->stats.nodes_alive--;
    delete n;
  }
}

// A materialised node no longer needs its predecessors (Section 2: later
// requests read its data instead of recomputing it).
void drop_inputs(gr_ctx* c, Node* n) {
  std::vector<Node*> ins;
  ins.swap(n->in);
  for (Node* p : ins)
    if (--p->consumer_refs == 0 && p->handle_refs == 0) node_maybe_free(c, p);
}

static void contiguous_strides(Node* n) {
  int64_t s = 1;
  for (int d = n->ndim - 1; d >= 0; --d) {
    n->strides[d] = s;
    s *= n->shape[d];
  }
}

// ---- merging of equal pending expressions at record time -----------------------
// The DAG makes common subexpressions visible (Section 5 names their elimination as
// something the representation enables).  Cheap pointwise duplicates are merged later,
// inside a sub-graph, by value numbering of the point program: merging them here would
// hand one node to several sub-graphs and the multiple-use rule of Algorithm 1 would then
// store it, which costs more than recomputing it.  Reductions, scans and contractions are
// sub-graph roots anyway and expensive, so an operation of those kinds whose whole pending
// expression equals that of a node still waiting to be evaluated returns that node.
// Materialised nodes never match anything but themselves: their storage may have been
// written (slice assignment, or the caller's own code on a wrapped buffer) since.

static inline uint64_t mix(uint64_t h, uint64_t v) {
  h ^= v + 0x9e3779b97f4a7c15ull + (h << 6) + (h >> 2);
  return h * 0xff51afd7ed558ccdull;
}

static void set_shash(Node* n) {
  if (n->materialized || n->kind == Kind::LEAF) { n->shash = mix(0x4c454146, n->id); return; }
  uint64_t h = mix((uint64_t)n->kind, (uint64_t)n->op * 16 + (uint64_t)n->dtype);
  h = mix(h, (uint64_t)n->ndim);
  for (int d = 0; d < n->ndim; ++d) h = mix(h, (uint64_t)n->shape[d]);
  if (n->kind == Kind::CONST || n->kind == Kind::SCALAR) {
    uint64_t bits;
    std::memcpy(&bits, &n->value, 8);
    h = mix(h, bits * 2 + (n->is_int ? 1 : 0));
  }
  for (const Node* p : n->in) {
    h = mix(h, p->shash);
    if (n->kind == Kind::SLICE) for (int d = 0; d < p->ndim; ++d) h = mix(mix(h, (uint64_t)n->start[d]), (uint64_t)n->step[d]);
    if (n->kind == Kind::TRANSPOSE) for (int d = 0; d < p->ndim; ++d) h = mix(h, (uint64_t)n->perm[d]);
    if (n->kind == Kind::REDUCE || n->kind == Kind::SCAN) {
      for (int d = 0; d < p->ndim; ++d) h = mix(h, n->red_axis[d] ? 2 : 1);
      h = mix(h, n->keepdims ? 2 : 1);
    }
  }
  n->shash = h;
}

static bool same_expr(const Node* a, const Node* b, std::set<std::pair<uint64_t, uint64_t>>& assumed) {
  if (a == b) return true;
  if (a->materialized || b->materialized || a->kind == Kind::LEAF || b->kind == Kind::LEAF) return false;
  if (a->shash != b->shash || a->kind != b->kind || a->op != b->op || a->dtype != b->dtype || a->ndim != b->ndim ||
      a->in.size() != b->in.size())
    return false;
  for (int d = 0; d < a->ndim; ++d) if (a->shape[d] != b->shape[d]) return false;
  if (a->kind == Kind::CONST || a->kind == Kind::SCALAR) return std::memcmp(&a->value, &b->value, 8) == 0 && a->is_int == b->is_int;
  if (!assumed.insert({a->id, b->id}).second) return true;  // already compared (or being compared) on another path
  if (!a->in.empty()) {
    const Node* p = a->in[0];
    if (a->kind == Kind::SLICE) for (int d = 0; d < p->ndim; ++d) if (a->start[d] != b->start[d] || a->step[d] != b->step[d]) return false;
    if (a->kind == Kind::TRANSPOSE) for (int d = 0; d < p->ndim; ++d) if (a->perm[d] != b->perm[d]) return false;
    if (a->kind == Kind::REDUCE || a->kind == Kind::SCAN) {
      if (a->keepdims != b->keepdims || p->ndim != b->in[0]->ndim) return false;
      for (int d = 0; d < p->ndim; ++d) if (a->red_axis[d] != b->red_axis[d]) return false;
    }
  }
  for (size_t i = 0; i < a->in.size(); ++i) if (!same_expr(a->in[i], b->in[i], assumed)) return false;
  return true;
}

// Finishes the recording of `n`: returns the handle to give out, which is an equal pending
// node's if there is one (`n` is then dropped again).
static gr_array finish(gr_ctx* c, Node* n) {
  set_shash(n);
  if (!(n->kind == Kind::REDUCE || n->kind == Kind::DOT || n->kind == Kind::SCAN)) return n->id;
  if (c->opt_merge) {
    auto range = c->pending_expensive.equal_range(n->shash);
    for (auto it = range.first; it != range.second; ++it) {
      auto f = c->nodes.find(it->second);
      if (f == c->nodes.end() || f->second->materialized || f->second->planned) continue;
      std::set<std::pair<uint64_t, uint64_t>> assumed;
      if (!same_expr(f->second, n, assumed)) continue;
      Node* e = f->second;
      e->handle_refs++;
      n->handle_refs = 0;
      node_maybe_free(c, n);
      c->stats.nodes_merged++;
      return e->id;
    }
  }
  c->pending_expensive.emplace(n->shash, n->id);
  return n->id;
}

static bool is_unary(int op) { return op >= GR_NEG && op <= GR_ERF; }
static bool is_binary(int op) { return op >= GR_ADD && op <= GR_MINIMUM; }
static bool is_reduce(int op) { return op >= GR_SUM && op <= GR_MIN; }

// The integer a caller passed where the C ABI takes an enumeration.  Any int may arrive through the ABI, and reading
// an enumeration object that holds a value outside its range is undefined behaviour in C++: the bits are copied out
// and checked as an int before the argument is used with its own type.
template <class E>
static int enum_arg(const E& e) {
  int v;
  static_assert(sizeof(E) == sizeof(int), "enumerations of the ABI are int-sized");
  std::memcpy(&v, &e, sizeof v);
  return v;
}

}  // namespace gr

using namespace gr;

extern "C" {

const char* gr_last_error(gr_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

gr_status gr_ctx_set_option(gr_ctx* ctx, const char* key, int64_t value) {
  if (!ctx || !key) return GR_ERR_ARG;
  std::string k(key);
  ctx->options_epoch++;
  if (k == "fusion") ctx->opt_fusion = value;
  else if (k == "rowred_max_cols") ctx->opt_rowred_max_cols = value;
  else if (k == "map_rows") ctx->opt_map_rows = value;
  else if (k == "map_chunks") ctx->opt_map_chunks = value;
  else if (k == "profile") ctx->opt_profile = value;
  else if (k == "nontemporal") ctx->opt_nontemporal = value;
  else if (k == "map_bx") ctx->opt_map_bx = value;
  else if (k == "rowred_threads") ctx->opt_rowred_threads = value;
  else if (k == "rowred_rows") ctx->opt_rowred_rows = value;
  else if (k == "gemm_bn") ctx->opt_gemm_bn = value;
  else if (k == "gemm_kstep") ctx->opt_gemm_kstep = value;
  else if (k == "gemm_split") ctx->opt_gemm_split = value;
  else if (k == "gemm_big") ctx->opt_gemm_big = value;
  else if (k == "map_phase") ctx->opt_map_phase = value;
  else if (k == "pool_limit") ctx->opt_pool_limit = value;
  else if (k == "stage_rows") ctx->opt_stage_rows = value;
  else if (k == "stage_diag") ctx->opt_stage_diag = value;
  else if (k == "gemv_slabs") ctx->opt_gemv_slabs = value;
  else if (k == "gemv_unroll") ctx->opt_gemv_unroll = value;
  else if (k == "gemv_pair") ctx->opt_gemv_pair = value;
  else if (k == "async_compile") ctx->opt_async_compile = value;
  else if (k == "disk_cache") ctx->opt_disk_cache = value;
  else if (k == "merge") ctx->opt_merge = value;
  else if (k == "interp") ctx->opt_interp = value;
  else if (k == "assign_swap") ctx->opt_assign_swap = value;
  else if (k == "dry_run") ctx->opt_dry_run = value;
  else if (k == "stage_transposed") ctx->opt_stage = value;
  else if (k == "plan_cache") ctx->opt_plan_cache = value;
  else if (k == "scan_threads") ctx->opt_scan_threads = value;
  else if (k == "scan_min_threads") ctx->opt_scan_min_threads = value;
  else if (k == "scan_one_pass") ctx->opt_scan_one_pass = value;
  else if (k == "scan_polls") { if (value < 0 || value > ((int64_t)1 << 24)) return fail(ctx, GR_ERR_ARG, "scan_polls: 0 to 2^24"); ctx->opt_scan_polls = value; }
  else return fail(ctx, GR_ERR_ARG, "unknown option '" + k + "'");
  return GR_OK;
}

gr_status gr_ctx_set_allocator(gr_ctx* ctx, void* (*alloc)(size_t, void*), void (*free_)(void*, void*), void* user) {
  if (!ctx) return GR_ERR_ARG;
  if ((alloc == nullptr) != (free_ == nullptr)) return fail(ctx, GR_ERR_ARG, "alloc and free must be given together");
  ctx->alloc_fn = alloc;
  ctx->free_fn = free_;
  ctx->alloc_user = user;
  return GR_OK;
}

gr_status gr_array_from_device(gr_ctx* ctx, void* dptr, gr_dtype dtype, int ndim, const int64_t* shape,
                               const int64_t* strides_elems, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  if (ndim < 0 || ndim > MAXD || (ndim > 0 && !shape)) return fail(ctx, GR_ERR_ARG, "from_device: bad rank or NULL shape");
  { const int dt = enum_arg(dtype); if (dt != GR_F32 && dt != GR_I32 && dt != GR_I64) return fail(ctx, GR_ERR_ARG, "from_device: bad dtype"); }
  int64_t n = 1;
  for (int d = 0; d < ndim; ++d)
    if (shape[d] < 0) return fail(ctx, GR_ERR_ARG, "from_device: negative extent");
  if (!count_fits(shape, ndim)) return fail(ctx, GR_ERR_ARG, "from_device: more than 2^40 elements");
  for (int d = 0; d < ndim; ++d) n *= shape[d];
  if (strides_elems) {
    int64_t span = 0;  // largest |element offset| any index reaches
    for (int d = 0; d < ndim; ++d) {
      if (shape[d] <= 1) continue;
      if (strides_elems[d] < -MAX_COUNT || strides_elems[d] > MAX_COUNT)
        return fail(ctx, GR_ERR_ARG, "from_device: strides reach beyond 2^40 elements");
      int64_t st = strides_elems[d] < 0 ? -strides_elems[d] : strides_elems[d];
      if (st > (MAX_COUNT - span) / (shape[d] - 1))
        return fail(ctx, GR_ERR_ARG, "from_device: strides reach beyond 2^40 elements");
      span += st * (shape[d] - 1);
    }
  }
  if (n > 0 && !dptr) return fail(ctx, GR_ERR_ARG, "from_device: NULL device pointer");
  if (((uintptr_t)dptr) % itemsize(dtype)) return fail(ctx, GR_ERR_ARG, "from_device: pointer not aligned to the element size");
  Node* nd = new_node(ctx, Kind::LEAF);
  nd->dtype = dtype;
  nd->ndim = ndim;
  for (int d = 0; d < ndim; ++d) nd->shape[d] = shape[d];
  if (strides_elems) for (int d = 0; d < ndim; ++d) nd->strides[d] = strides_elems[d];
  else contiguous_strides(nd);
  nd->materialized = true;
  nd->data = dptr;
  nd->offset = 0;
  set_shash(nd);
  *out = nd->id;
  return GR_OK;
}

gr_status gr_scalar(gr_ctx* ctx, double value, int is_integer, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  if (is_integer && value != std::floor(value)) return fail(ctx, GR_ERR_ARG, "scalar: is_integer set on a fractional value");
  Node* nd = new_node(ctx, Kind::SCALAR);
  nd->value = value;
  nd->is_int = is_integer != 0;
  nd->ndim = 0;
  set_shash(nd);
  *out = nd->id;
  return GR_OK;
}

gr_status gr_unary(gr_ctx* ctx, gr_op op, gr_array a, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  if (!is_unary(enum_arg(op))) return fail(ctx, GR_ERR_ARG, "unary: not a unary op");
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "unary: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "unary: operand is a bare scalar");
  if (x->dtype == GR_I64) return fail(ctx, GR_ERR_UNSUPPORTED, "unary: i64 arithmetic is not supported");
  if (x->dtype == GR_I32 && !(op == GR_NEG || op == GR_ABS || op == GR_SQUARE))
    return fail(ctx, GR_ERR_DTYPE, "unary: float function of an i32 array would promote to f64");
  Node* n = new_node(ctx, Kind::UNARY);
  n->op = op;
  n->dtype = x->dtype;
  n->ndim = x->ndim;
  for (int d = 0; d < x->ndim; ++d) n->shape[d] = x->shape[d];
  add_input(n, x);
  *out = finish(ctx, n);
  return GR_OK;
}

gr_status gr_binary(gr_ctx* ctx, gr_op op, gr_array a, gr_array b, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  if (enum_arg(op) == GR_POW_INT) {
    // x ** 2 with an integer scalar 2 is recorded as square(x), NumPy's own fast path; no other power
    // is in the vocabulary
    const Node* x = lookup(ctx, a);
    const Node* e = lookup(ctx, b);
    if (!x || !e) return fail(ctx, GR_ERR_HANDLE, "binary: bad handle");
    if (e->kind != Kind::SCALAR || !e->is_int || e->value != 2.0 || x->kind == Kind::SCALAR)
      return fail(ctx, GR_ERR_UNSUPPORTED, "binary: the only power recorded is array ** 2 with an integer scalar");
    return gr_unary(ctx, GR_SQUARE, a, out);
  }
  if (!is_binary(enum_arg(op))) return fail(ctx, GR_ERR_ARG, "binary: not a binary op");
  Node* x = lookup(ctx, a);
  Node* y = lookup(ctx, b);
  if (!x || !y) return fail(ctx, GR_ERR_HANDLE, "binary: bad handle");
  bool wx = x->kind == Kind::SCALAR, wy = y->kind == Kind::SCALAR;
  if (wx && wy) return fail(ctx, GR_ERR_UNSUPPORTED, "binary: two bare scalars");
  gr_dtype dt = wx ? y->dtype : x->dtype;
  if (!wx && !wy && x->dtype != y->dtype) return fail(ctx, GR_ERR_DTYPE, "binary: mixed element types would promote to f64");
  if (dt == GR_I64) return fail(ctx, GR_ERR_UNSUPPORTED, "binary: i64 arithmetic is not supported");
  if (dt == GR_I32 && op == GR_DIV) return fail(ctx, GR_ERR_UNSUPPORTED, "binary: integer division is not supported");
  const Node* w = wx ? x : (wy ? y : nullptr);
  if (w && dt == GR_I32) {
    if (!w->is_int) return fail(ctx, GR_ERR_DTYPE, "binary: float scalar with an i32 array would promote to f64");
    if (w->value < -2147483648.0 || w->value > 2147483647.0) return fail(ctx, GR_ERR_DTYPE, "binary: integer scalar does not fit i32");
  }
  // NumPy broadcast: right-align, each pair equal or one of them 1.
  const Node* ax = wx ? nullptr : x;
  const Node* ay = wy ? nullptr : y;
  int nx = ax ? ax->ndim : 0, ny = ay ? ay->ndim : 0;
  int n = std::max(nx, ny);
  int64_t shape[MAXD];
  for (int d = 0; d < n; ++d) {
    int dx = d - (n - nx), dy = d - (n - ny);
    int64_t sx = (ax && dx >= 0) ? ax->shape[dx] : 1;
    int64_t sy = (ay && dy >= 0) ? ay->shape[dy] : 1;
    if (sx == sy) shape[d] = sx;
    else if (sx == 1) shape[d] = sy;
    else if (sy == 1) shape[d] = sx;
    else return fail(ctx, GR_ERR_SHAPE, "binary: shapes do not broadcast");
  }
  if (!count_fits(shape, n)) return fail(ctx, GR_ERR_SHAPE, "binary: the broadcast result has more than 2^40 elements");
  Node* r = new_node(ctx, Kind::BINARY);
  r->op = op;
  r->dtype = dt;
  r->ndim = n;
  for (int d = 0; d < n; ++d) r->shape[d] = shape[d];
  auto operand = [&](Node* o) -> Node* {
    if (o->kind != Kind::SCALAR) return o;
    Node* k = new_node(ctx, Kind::CONST);  // the scalar hardened to this op's element type
    k->handle_refs = 0;
    k->dtype = dt;
    k->ndim = 0;
    k->is_int = o->is_int;
    k->value = dt == GR_F32 ? (double)(float)o->value : o->value;
    set_shash(k);
    return k;
  };
  add_input(r, operand(x));
  add_input(r, operand(y));
  *out = finish(ctx, r);
  return GR_OK;
}

gr_status gr_binary_scalar(gr_ctx* ctx, gr_op op, gr_array a, double value, int is_integer, int scalar_on_left,
                           gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  if (!is_binary(enum_arg(op)) && enum_arg(op) != GR_POW_INT) return fail(ctx, GR_ERR_ARG, "binary: not a binary op");
  gr_array s = 0;
  gr_status st = gr_scalar(ctx, value, is_integer, &s);
  if (st != GR_OK) return st;
  st = scalar_on_left ? gr_binary(ctx, op, s, a, out) : gr_binary(ctx, op, a, s, out);
  gr_release(ctx, s);
  return st;
}

gr_status gr_slice(gr_ctx* ctx, gr_array a, int nspec, const int64_t* start, const int64_t* stop,
                   const int64_t* step, const uint8_t* has_start, const uint8_t* has_stop, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "slice: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "slice: operand is a bare scalar");
  if (nspec < 0 || nspec > x->ndim) return fail(ctx, GR_ERR_SHAPE, "slice: too many indices");
  if (nspec > 0 && (!start || !stop || !step || !has_start || !has_stop)) return fail(ctx, GR_ERR_ARG, "slice: NULL argument");
  int64_t lo[MAXD], st[MAXD], len[MAXD];
  for (int d = 0; d < x->ndim; ++d) {
    int64_t n = x->shape[d];
    if (d >= nspec) { lo[d] = 0; st[d] = 1; len[d] = n; continue; }
    if (step[d] < 1) return fail(ctx, GR_ERR_UNSUPPORTED, "slice: step must be >= 1");
    int64_t l = has_start[d] ? start[d] : 0, h = has_stop[d] ? stop[d] : n;
    if (l < 0) l += n;
    if (h < 0) h += n;
    l = std::min(std::max<int64_t>(l, 0), n);
    h = std::min(std::max<int64_t>(h, 0), n);
    lo[d] = l;
    st[d] = step[d];
    len[d] = h > l ? (h - l + step[d] - 1) / step[d] : 0;
  }
  Node* r = new_node(ctx, Kind::SLICE);
  r->dtype = x->dtype;
  r->ndim = x->ndim;
  for (int d = 0; d < x->ndim; ++d) { r->shape[d] = len[d]; r->start[d] = lo[d]; r->step[d] = st[d]; }
  add_input(r, x);
  *out = finish(ctx, r);
  return GR_OK;
}

gr_status gr_transpose(gr_ctx* ctx, gr_array a, const int* perm, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "transpose: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "transpose: operand is a bare scalar");
  int p[MAXD];
  bool seen[MAXD] = {false};
  for (int d = 0; d < x->ndim; ++d) {
    int v = perm ? perm[d] : x->ndim - 1 - d;
    if (v < 0) v += x->ndim;
    if (v < 0 || v >= x->ndim || seen[v]) return fail(ctx, GR_ERR_AXIS, "transpose: not a permutation");
    seen[v] = true;
    p[d] = v;
  }
  Node* r = new_node(ctx, Kind::TRANSPOSE);
  r->dtype = x->dtype;
  r->ndim = x->ndim;
  for (int d = 0; d < x->ndim; ++d) { r->shape[d] = x->shape[p[d]]; r->perm[d] = p[d]; }
  add_input(r, x);
  *out = finish(ctx, r);
  return GR_OK;
}

gr_status gr_reshape(gr_ctx* ctx, gr_array a, int ndim, const int64_t* shape, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "reshape: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "reshape: operand is a bare scalar");
  if (ndim < 0 || ndim > MAXD || (ndim > 0 && !shape)) return fail(ctx, GR_ERR_ARG, "reshape: bad rank or NULL shape");
  if (!count_fits(shape, ndim)) return fail(ctx, GR_ERR_SHAPE, "reshape: element counts differ");
  int64_t want[MAXD], known = 1;
  const int64_t n = x->count();
  int infer = -1;
  for (int d = 0; d < ndim; ++d) {
    want[d] = shape[d];
    if (shape[d] == -1) { if (infer >= 0) return fail(ctx, GR_ERR_SHAPE, "reshape: more than one inferred extent"); infer = d; }
    else if (shape[d] < 0) return fail(ctx, GR_ERR_SHAPE, "reshape: negative extent");
    else known *= shape[d];
  }
  if (infer >= 0) {
    if (known == 0 || n % known) return fail(ctx, GR_ERR_SHAPE, "reshape: cannot infer the extent");
    want[infer] = n / known;
    known *= want[infer];
  }
  if (known != n) return fail(ctx, GR_ERR_SHAPE, "reshape: element counts differ");
  Node* r = new_node(ctx, Kind::RESHAPE);
  r->dtype = x->dtype;
  r->ndim = ndim;
  for (int d = 0; d < ndim; ++d) r->shape[d] = want[d];
  add_input(r, x);
  *out = finish(ctx, r);
  return GR_OK;
}

gr_status gr_reduce(gr_ctx* ctx, gr_op op, gr_array a, const int* axes, int naxes, int keepdims, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  if (!is_reduce(enum_arg(op))) return fail(ctx, GR_ERR_ARG, "reduce: not a reduction op");
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "reduce: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "reduce: operand is a bare scalar");
  if (x->dtype == GR_I64) return fail(ctx, GR_ERR_UNSUPPORTED, "reduce: i64 operands are not supported");
  if (naxes < 0 || naxes > x->ndim || (naxes > 0 && !axes)) return fail(ctx, GR_ERR_AXIS, "reduce: bad axis list");
  bool red[MAXD];
  for (int d = 0; d < x->ndim; ++d) red[d] = (naxes == 0);
  for (int k = 0; k < naxes; ++k) {
    int ax = axes[k] < 0 ? axes[k] + x->ndim : axes[k];
    if (ax < 0 || ax >= x->ndim) return fail(ctx, GR_ERR_AXIS, "reduce: axis out of range");
    if (red[ax]) return fail(ctx, GR_ERR_AXIS, "reduce: repeated axis");
    red[ax] = true;
  }
  int64_t rcount = 1;
  for (int d = 0; d < x->ndim; ++d) if (red[d]) rcount *= x->shape[d];
  if (rcount == 0 && op != GR_SUM) return fail(ctx, GR_ERR_SHAPE, "reduce: max/min over an empty range");
  Node* r = new_node(ctx, Kind::REDUCE);
  r->op = op;
  r->dtype = (x->dtype == GR_I32 && op == GR_SUM) ? GR_I64 : x->dtype;
  r->keepdims = keepdims != 0;
  int nd = 0;
  for (int d = 0; d < x->ndim; ++d) {
    r->red_axis[d] = red[d];
    if (red[d]) { if (keepdims) r->shape[nd++] = 1; }
    else r->shape[nd++] = x->shape[d];
  }
  r->ndim = nd;
  add_input(r, x);
  *out = finish(ctx, r);
  return GR_OK;
}

gr_status gr_scan(gr_ctx* ctx, gr_op op, gr_array a, int axis, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  if (!is_reduce(enum_arg(op))) return fail(ctx, GR_ERR_ARG, "scan: not a scan op");
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "scan: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "scan: operand is a bare scalar");
  if (x->dtype == GR_I64) return fail(ctx, GR_ERR_UNSUPPORTED, "scan: i64 operands are not supported");
  if (x->ndim < 1) return fail(ctx, GR_ERR_AXIS, "scan: rank-0 operand has no axis");
  int ax = axis < 0 ? axis + x->ndim : axis;
  if (ax < 0 || ax >= x->ndim) return fail(ctx, GR_ERR_AXIS, "scan: axis out of range");
  Node* r = new_node(ctx, Kind::SCAN);
  r->op = op;
  r->dtype = (x->dtype == GR_I32 && op == GR_SUM) ? GR_I64 : x->dtype;
  r->ndim = x->ndim;
  for (int d = 0; d < x->ndim; ++d) { r->shape[d] = x->shape[d]; r->red_axis[d] = d == ax; }
  add_input(r, x);
  *out = finish(ctx, r);
  return GR_OK;
}

gr_status gr_dot(gr_ctx* ctx, gr_array a, gr_array b, gr_array* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  Node* y = lookup(ctx, b);
  if (!x || !y) return fail(ctx, GR_ERR_HANDLE, "dot: bad handle");
  if (x->kind == Kind::SCALAR || y->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "dot: scalar operand");
  if (x->dtype != GR_F32 || y->dtype != GR_F32) return fail(ctx, GR_ERR_DTYPE, "dot: f32 operands only");
  if (y->ndim == 2 && x->ndim == 1) return fail(ctx, GR_ERR_UNSUPPORTED, "dot: vector-matrix product is not supported (transpose both sides)");
  if (y->ndim < 1 || y->ndim > 2 || x->ndim < 1 || x->ndim > 2) return fail(ctx, GR_ERR_UNSUPPORTED, "dot: supported ranks are (M,K).(K,N), (M,K).(K,) and (K,).(K,)");
  if (x->shape[x->ndim - 1] != y->shape[0]) return fail(ctx, GR_ERR_SHAPE, "dot: inner dimensions differ");
  {
    const int64_t mn[2] = {x->ndim == 2 ? x->shape[0] : 1, y->ndim == 2 ? y->shape[1] : 1};
    if (!count_fits(mn, 2)) return fail(ctx, GR_ERR_SHAPE, "dot: the result has more than 2^40 elements");
  }
  Node* r = new_node(ctx, Kind::DOT);
  r->dtype = GR_F32;
  r->ndim = x->ndim - 1 + y->ndim - 1;
  if (x->ndim == 2) r->shape[0] = x->shape[0];
  if (y->ndim == 2) r->shape[r->ndim - 1] = y->shape[1];
  add_input(r, x);
  add_input(r, y);
  *out = finish(ctx, r);
  return GR_OK;
}

gr_status gr_ndim(gr_ctx* ctx, gr_array a, int* ndim) {
  if (!ctx || !ndim) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "ndim: bad handle");
  *ndim = x->ndim;
  return GR_OK;
}

gr_status gr_shape(gr_ctx* ctx, gr_array a, int64_t* shape) {
  if (!ctx || !shape) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "shape: bad handle");
  for (int d = 0; d < x->ndim; ++d) shape[d] = x->shape[d];
  return GR_OK;
}

gr_status gr_dtype_of(gr_ctx* ctx, gr_array a, gr_dtype* dtype) {
  if (!ctx || !dtype) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "dtype_of: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "dtype_of: a bare scalar has no element type");
  *dtype = x->dtype;
  return GR_OK;
}

// Resolves a chain of views down to a materialised node, composing offset and
// strides.  Returns false if the chain ends at a lazy node.
static bool resolve_view(const Node* n, void** data, int64_t* offset, int64_t* strides) {
  if (n->materialized) {
    *data = n->data;
    *offset = n->offset;
    for (int d = 0; d < n->ndim; ++d) strides[d] = n->strides[d];
    return true;
  }
  if (!n->is_view()) return false;
  int64_t st[MAXD];
  if (!resolve_view(n->in[0], data, offset, st)) return false;
  if (n->kind == Kind::SLICE) {
    for (int d = 0; d < n->ndim; ++d) { *offset += n->start[d] * st[d]; strides[d] = st[d] * n->step[d]; }
  } else {
    for (int d = 0; d < n->ndim; ++d) strides[d] = st[n->perm[d]];
  }
  return true;
}

gr_status gr_is_materialized(gr_ctx* ctx, gr_array a, int* flag) {
  if (!ctx || !flag) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "is_materialized: bad handle");
  void* p; int64_t off, st[MAXD];
  *flag = (x->kind != Kind::SCALAR && resolve_view(x, &p, &off, st)) ? 1 : 0;
  return GR_OK;
}

gr_status gr_data_ptr(gr_ctx* ctx, gr_array a, void** dptr, int64_t* strides) {
  if (!ctx || !dptr) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "data_ptr: bad handle");
  void* p; int64_t off, st[MAXD];
  if (x->kind == Kind::SCALAR || !resolve_view(x, &p, &off, st)) return fail(ctx, GR_ERR_UNSUPPORTED, "data_ptr: array is not materialised");
  *dptr = (char*)p + off * (int64_t)itemsize(x->dtype);
  if (strides) for (int d = 0; d < x->ndim; ++d) strides[d] = st[d];
  return GR_OK;
}

gr_status gr_retain(gr_ctx* ctx, gr_array a) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "retain: bad handle");
  x->handle_refs++;
  return GR_OK;
}

gr_status gr_release(gr_ctx* ctx, gr_array a) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "release: bad handle");
  x->handle_refs--;
  node_maybe_free(ctx, x);
  return GR_OK;
}

gr_status gr_stats(gr_ctx* ctx, gr_stats_t* out) {
  if (!ctx || !out) return GR_ERR_ARG;
  *out = ctx->stats;
  out->pool_bytes = ctx->pool_bytes;
  return GR_OK;
}

}  // extern "C"
