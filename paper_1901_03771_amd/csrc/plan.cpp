// Materialiser and fusion partitioner.
//
// Section 2 of the paper: on a request the DAG is walked back from the
// requested node to materialised nodes; Algorithm 1 (create_subgraph) splits
// the visited sub-DAG into an ordered list of sub-graphs, cutting at nodes that
// must be materialised (materialize_node: library-grade contractions and
// reductions), at operands of such library operations
// (materialize_pred_of_node, with a transposed operand folded into the call),
// and at nodes that a second sub-graph would otherwise recompute (the
// multiple-use rule: such a node is materialised once and is a leaf of every
// user).  This file implements that rule set in closed form:
//
//   cut(n) :=  n is the requested root
//           |  n is a dot node whose consumers cannot run as its epilogue
//           |  n is the (view-stripped) lazy operand of a dot node
//           |  n is a reduction that cannot stay resident in registers
//           |  n is reached from two different cut nodes
//
// and every cut node becomes the root of one sub-graph; ascending node ids are
// a topological order, so the list is in execution order.  Two relaxations of
// the paper's rules are deliberate: a reduction over the innermost axis whose
// row fits in registers stays fused with producers and consumers, and
// pointwise consumers of a dot run as the contraction kernel's epilogue.
//
// For each sub-graph the point function of Section 3.1 is built as a flat SSA
// program: output indices are translated back to leaf indices through
// broadcast, slice and transpose nodes by composing affine per-dimension maps.
#include <algorithm>
#include <cstdio>
#include <functional>
#include <sstream>

#include "ctx.h"

namespace gr {

namespace {

int64_t floordiv(int64_t a, int64_t b) { int64_t q = a / b; return (a % b != 0 && ((a < 0) != (b < 0))) ? q - 1 : q; }
int64_t floormod(int64_t a, int64_t b) { return a - floordiv(a, b) * b; }

const char* op_name(int op) {
  switch (op) {
    case GR_NEG: return "neg"; case GR_ABS: return "abs"; case GR_EXP: return "exp"; case GR_LOG: return "log";
    case GR_SQRT: return "sqrt"; case GR_SQUARE: return "square"; case GR_TANH: return "tanh"; case GR_ERF: return "erf";
    case GR_ADD: return "add"; case GR_SUB: return "sub"; case GR_MUL: return "mul"; case GR_DIV: return "div";
    case GR_MAXIMUM: return "maximum"; case GR_MINIMUM: return "minimum";
    case GR_SUM: return "sum"; case GR_MAX: return "max"; case GR_MIN: return "min";
  }
  return "?";
}

std::string node_label(const Node* n) {
  switch (n->kind) {
    case Kind::LEAF: return "leaf";
    case Kind::SCALAR: return "scalar";
    case Kind::CONST: return "const";
    case Kind::UNARY: case Kind::BINARY: case Kind::REDUCE: return op_name(n->op);
    case Kind::SLICE: return "slice";
    case Kind::TRANSPOSE: return "transpose";
    case Kind::RESHAPE: return "reshape";
    case Kind::DOT: return "dot";
    case Kind::SCAN: return std::string("cum") + op_name(n->op);
  }
  return "?";
}

struct Invalid {
  const Node* node;
  std::string why;
};

// A contraction over at most eight terms (points times a 3 x 3 matrix, a handful of weights) is
// written out as products and sums inside the point function: it fuses with producers and
// consumers like any pointwise op instead of becoming a library-style kernel of its own.
bool small_dot(const Node* n) {
  return n->kind == Kind::DOT && n->ndim >= 1 && n->in[1]->shape[0] <= 8;
}

// Builds the SSA program of one sub-graph.
struct Builder {
  GroupPlan* g;
  const NodeSet* owned;  // lazy nodes this sub-graph computes
  int rank = 0;                        // iteration rank (original dims)
  const int64_t* dims = nullptr;
  std::vector<Instr>* prog = nullptr;

  std::map<std::pair<uint64_t, std::vector<int64_t>>, int> memo;
  std::map<std::vector<int64_t>, int> load_ids;   // (group, delta...) -> instr
  std::map<std::vector<int64_t>, int> value_ids;  // (kind, op, dtype, a, b) -> instr
  std::map<const Node*, int, NodeIdLess> phase_of;
  const Node* dot_core = nullptr;
  std::vector<Invalid> invalid;
  NodeSet leaves_seen, members_seen;

  static std::vector<int64_t> flatten(const IndexMap& m) {
    std::vector<int64_t> v;
    v.reserve(m.size() * 3);
    for (const DimMap& d : m) { v.push_back(d.src); v.push_back(d.scale); v.push_back(d.off); }
    return v;
  }

  void canonicalize(const Node* n, IndexMap& m) const {
    for (int d = 0; d < n->ndim; ++d) {
      DimMap& e = m[d];
      if (n->shape[d] == 1) { e = DimMap{-1, 0, 0}; continue; }
      if (e.src >= 0 && (e.scale == 0 || dims[e.src] == 1)) e = DimMap{-1, 0, e.off};
    }
  }

  int push(const Instr& in) {
    prog->push_back(in);
    return (int)prog->size() - 1;
  }

  int value_number(Instr in) {
    std::vector<int64_t> key{(int64_t)in.kind, in.op, (int64_t)in.dtype, in.a, in.b, in.cslot, in.phase};
    auto it = value_ids.find(key);
    if (it != value_ids.end()) return it->second;
    int id = push(in);
    value_ids[key] = id;
    return id;
  }

  int constant(gr_dtype dt, double v) {
    int slot = -1;
    for (size_t i = 0; i < g->consts.size(); ++i)
      if (g->consts[i].dtype == dt && std::memcmp(&g->consts[i].value, &v, sizeof(double)) == 0) slot = (int)i;
    if (slot < 0) { g->consts.push_back(ConstSlot{dt, v}); slot = (int)g->consts.size() - 1; }
    Instr in;
    in.kind = IKind::CONST; in.dtype = dt; in.cslot = slot; in.uniform = true;
    return value_number(in);
  }

  int load(const Node* leaf, const IndexMap& m) {
    leaves_seen.insert(leaf);
    std::vector<int64_t> ident{(int64_t)leaf->id};
    int64_t delta[MAXD] = {0};
    for (int d = 0; d < leaf->ndim; ++d) {
      const DimMap& e = m[d];
      ident.push_back(e.src);
      ident.push_back(e.scale);
      if (e.src < 0) ident.push_back(e.off);
      else { ident.push_back(floormod(e.off, e.scale)); delta[e.src] += floordiv(e.off, e.scale); }
    }
    int gid = -1;
    for (size_t i = 0; i < g->groups.size(); ++i) if (g->groups[i].ident == ident) gid = (int)i;
    if (gid < 0) {
      AccessGroup ag;
      ag.leaf = leaf; ag.dtype = leaf->dtype; ag.ident = ident;
      ag.base = leaf->offset;
      for (int k = 0; k < MAXD; ++k) ag.structural_zero[k] = true;
      for (int d = 0; d < leaf->ndim; ++d) {
        const DimMap& e = m[d];
        if (e.src < 0) ag.base += leaf->strides[d] * e.off;
        else {
          ag.base += leaf->strides[d] * floormod(e.off, e.scale);
          ag.coef[e.src] += leaf->strides[d] * e.scale;
          ag.structural_zero[e.src] = false;
        }
      }
      g->groups.push_back(ag);
      gid = (int)g->groups.size() - 1;
    }
    std::vector<int64_t> dv(delta, delta + rank);
    g->groups[gid].deltas.insert(dv);
    std::vector<int64_t> key{gid};
    key.insert(key.end(), dv.begin(), dv.end());
    auto it = load_ids.find(key);
    if (it != load_ids.end()) return it->second;
    Instr in;
    in.kind = IKind::LOAD; in.dtype = leaf->dtype; in.group = gid;
    for (int k = 0; k < rank; ++k) in.delta[k] = delta[k];
    in.uniform = g->groups[gid].structural_zero[rank - 1];
    int id = push(in);
    load_ids[key] = id;
    return id;
  }

  static bool is_identity_on(const IndexMap& m, int d, int src, int64_t extent) {
    if (extent == 1) return true;  // canonicalised to a constant 0
    return m[d].src == src && m[d].scale == 1 && m[d].off == 0;
  }

  int eval(const Node* n, IndexMap m) {
    canonicalize(n, m);
    auto key = std::make_pair(n->id, flatten(m));
    auto it = memo.find(key);
    if (it != memo.end()) return it->second;
    int id = -1;
    if (n->kind == Kind::CONST) {
      id = constant(n->dtype, n->value);
    } else if (n->has_data()) {
      id = load(n, m);
    } else {
      members_seen.insert(n);
      switch (n->kind) {
        case Kind::UNARY: {
          Instr in;
          in.kind = IKind::UNARY; in.op = n->op; in.dtype = n->dtype;
          in.a = eval(n->in[0], m);
          in.uniform = (*prog)[in.a].uniform;
          id = value_number(in);
          break;
        }
        case Kind::BINARY: {
          int ops[2];
          for (int s = 0; s < 2; ++s) {
            const Node* o = n->in[s];
            IndexMap om(o->ndim);
            for (int d = 0; d < o->ndim; ++d) om[d] = m[d + (n->ndim - o->ndim)];
            ops[s] = eval(o, om);  // canonicalize() zeroes broadcast (extent-1) dims
          }
          Instr in;
          in.kind = IKind::BINARY; in.op = n->op; in.dtype = n->dtype; in.a = ops[0]; in.b = ops[1];
          in.uniform = (*prog)[in.a].uniform && (*prog)[in.b].uniform;
          id = value_number(in);
          break;
        }
        case Kind::SLICE: {
          IndexMap om(n->ndim);
          for (int d = 0; d < n->ndim; ++d)
            om[d] = DimMap{m[d].src, m[d].scale * n->step[d], n->start[d] + n->step[d] * m[d].off};
          id = eval(n->in[0], om);
          break;
        }
        case Kind::TRANSPOSE: {
          IndexMap om(n->ndim);
          for (int d = 0; d < n->ndim; ++d) om[n->perm[d]] = m[d];
          id = eval(n->in[0], om);
          break;
        }
        case Kind::REDUCE: {
          id = reduce_result(n, m);
          break;
        }
        case Kind::DOT: {
          if (small_dot(n)) {
            const Node* A = n->in[0];
            const Node* B = n->in[1];
            const int64_t K = B->shape[0];
            // the sum starts from +0 like the accumulator of a contraction kernel (and of the eager
            // evaluation): products that are all -0 add up to +0
            id = constant(n->dtype, 0.0);
            for (int64_t k = 0; k < K; ++k) {
              IndexMap am(A->ndim), bm(B->ndim);
              if (A->ndim == 2) am[0] = m[0];
              am[A->ndim - 1] = DimMap{-1, 0, k};
              bm[0] = DimMap{-1, 0, k};
              if (B->ndim == 2) bm[1] = m[n->ndim - 1];
              Instr mul;
              mul.kind = IKind::BINARY; mul.op = GR_MUL; mul.dtype = n->dtype;
              mul.a = eval(A, am); mul.b = eval(B, bm);
              mul.uniform = (*prog)[mul.a].uniform && (*prog)[mul.b].uniform;
              int p = value_number(mul);
              Instr add;
              add.kind = IKind::BINARY; add.op = GR_ADD; add.dtype = n->dtype; add.a = id; add.b = p;
              add.uniform = (*prog)[id].uniform && (*prog)[p].uniform;
              id = value_number(add);
            }
            break;  // (an empty contraction is the constant 0)
          }
          bool ok = (g->kind == GroupKind::GEMV || g->kind == GroupKind::GEMM) && (dot_core == nullptr || dot_core == n);
          for (int d = 0; ok && d < n->ndim; ++d) ok = is_identity_on(m, d, d, n->shape[d]);
          if (!ok) { invalid.push_back({n, "dot result not usable as an epilogue input"}); id = constant(GR_F32, 0.0); break; }
          dot_core = n;
          Instr in;
          in.kind = IKind::ACC; in.dtype = GR_F32;
          id = value_number(in);
          break;
        }
        case Kind::SCAN:
          invalid.push_back({n, "a scan is always materialised"});
          id = constant(n->dtype, 0.0);
          break;
        default:
          invalid.push_back({n, "unexpected lazy node kind (" + node_label(n) + " #" + std::to_string(n->id) + ")"});
          id = constant(GR_F32, 0.0);
      }
    }
    memo[key] = id;
    return id;
  }

  // A reduction met inside a row-resident sub-graph: its value for the current
  // row is the result of one reduction phase over the row.
  int reduce_result(const Node* r, const IndexMap& m) {
    const Node* x = r->in[0];
    bool ok = g->kind == GroupKind::ROWRED && x->ndim == rank && x->ndim >= 1;
    if (ok) for (int d = 0; d < x->ndim; ++d) {
      if (r->red_axis[d] != (d == x->ndim - 1)) ok = false;
      if (x->shape[d] != dims[d]) ok = false;
    }
    if (ok) {
      int kept = x->ndim - 1;
      if ((int)m.size() != (r->keepdims ? x->ndim : kept)) ok = false;
      for (int d = 0; ok && d < kept; ++d) if (!is_identity_on(m, d, d, x->shape[d])) ok = false;
    }
    if (!ok) {
      invalid.push_back({r, "reduction cannot stay row-resident in this sub-graph"});
      return constant(r->dtype, 0.0);
    }
    auto it = phase_of.find(r);
    int ph;
    if (it != phase_of.end()) ph = it->second;
    else {
      IndexMap full(x->ndim);
      for (int d = 0; d < x->ndim; ++d) full[d] = DimMap{d, 1, 0};
      int v = eval(x, full);
      Phase p;
      p.op = r->op; p.in_dtype = x->dtype; p.out_dtype = r->dtype; p.value = v; p.node = r;
      g->phases.push_back(p);
      ph = (int)g->phases.size() - 1;
      phase_of[r] = ph;
    }
    Instr in;
    in.kind = IKind::RED; in.dtype = r->dtype; in.phase = ph; in.uniform = true;
    return value_number(in);
  }
};

// Follows views from `n` down to a node with data, composing the index map.
bool resolve_to_leaf(const Node* n, IndexMap m, const Node** leaf, IndexMap* lm) {
  while (!n->has_data()) {
    if (n->kind == Kind::SLICE) {
      IndexMap om(n->ndim);
      for (int d = 0; d < n->ndim; ++d) om[d] = DimMap{m[d].src, m[d].scale * n->step[d], n->start[d] + n->step[d] * m[d].off};
      m = om;
    } else if (n->kind == Kind::TRANSPOSE) {
      IndexMap om(n->ndim);
      for (int d = 0; d < n->ndim; ++d) om[n->perm[d]] = m[d];
      m = om;
    } else return false;
    n = n->in[0];
  }
  *leaf = n;
  *lm = m;
  return true;
}

// A contraction with one output row or very few, over a long k: too little parallelism for the
// row-per-lane-group kernel.  It is planned as the map-reduce it is (Listing 5 of the paper writes
// the inner product exactly so): value a[m,k] * v[k], reduced over k in two stages.
// Element strides an array will have when it is read: those of its storage if it has one, of a
// C-contiguous result if it is still to be computed, transformed by the views in between.
static void strides_when_read(const Node* n, int64_t* st) {
  if (n->materialized) { for (int d = 0; d < n->ndim; ++d) st[d] = n->strides[d]; return; }
  if (!n->is_view()) {
    int64_t s = 1;
    for (int d = n->ndim - 1; d >= 0; --d) { st[d] = s; s *= n->shape[d]; }
    return;
  }
  int64_t in[MAXD];
  strides_when_read(n->in[0], in);
  if (n->kind == Kind::SLICE) for (int d = 0; d < n->ndim; ++d) st[d] = in[d] * n->step[d];
  else for (int d = 0; d < n->ndim; ++d) st[d] = in[n->perm[d]];
}

bool dot_as_reduce(const Node* n) {
  if (n->kind != Kind::DOT) return false;
  const Node* A = n->in[0];
  const Node* v = n->in[1];
  if (v->ndim != 1) return false;
  const int64_t K = v->shape[0], M = A->ndim == 2 ? A->shape[0] : 1;
  if (!(K >= 8192 && M * 64 <= K && M <= 2048)) return false;
  // rows that are contiguous along k only: a transposed matrix has the column-accumulate kernel
  int64_t st[MAXD];
  strides_when_read(A, st);
  return st[A->ndim - 1] == 1 || st[A->ndim - 1] == 2 || A->ndim == 1;
}

// The node whose index space a map sub-graph rooted at `r` iterates over: the operand of a reshape
// that is still to be evaluated, `r` itself otherwise.
const Node* map_source(const Node* r) {
  return (r->kind == Kind::RESHAPE && !r->materialized && !r->in.empty()) ? r->in[0] : r;
}

const Node* strip_views(const Node* n) {
  while (n->is_view() && !n->has_data()) n = n->in[0];
  return n;
}

int next_pow2(int64_t v) { int p = 1; while (p < v && p < (1 << 30)) p <<= 1; return p; }  // saturates at 2^30

void normalize_deltas(GroupPlan* g, std::vector<Instr>* progs[], int nprogs, int rank) {
  for (size_t gi = 0; gi < g->groups.size(); ++gi) {
    AccessGroup& ag = g->groups[gi];
    if (ag.deltas.empty()) continue;
    std::vector<int64_t> mn(rank, INT64_MAX);
    for (const auto& d : ag.deltas) for (int k = 0; k < rank; ++k) mn[k] = std::min(mn[k], d[k]);
    std::set<std::vector<int64_t>> nd;
    for (auto d : ag.deltas) { for (int k = 0; k < rank; ++k) d[k] -= mn[k]; nd.insert(d); }
    ag.deltas.swap(nd);
    for (int k = 0; k < rank; ++k) ag.base += ag.coef[k] * mn[k];
    for (int p = 0; p < nprogs; ++p)
      for (Instr& in : *progs[p])
        if (in.kind == IKind::LOAD && in.group == (int)gi) for (int k = 0; k < rank; ++k) in.delta[k] -= mn[k];
  }
}

// Merges adjacent iteration dimensions that every access (and the contiguous
// output) walks as one linear run.  `barrier[k]` forbids merging dim k with k+1.
void collapse_dims(GroupPlan* g, const bool* barrier, std::vector<Instr>* progs[], int nprogs) {
  int n = g->orig_rank;
  // runs of original dims, extent-1 dims dropped
  std::vector<std::vector<int>> runs;
  for (int k = 0; k < n; ++k) {
    if (g->orig_dims[k] == 1) continue;
    bool merged = false;
    if (!runs.empty()) {
      int prev = runs.back().back();
      bool blocked = false;
      for (int j = prev; j < k; ++j) if (barrier[j]) blocked = true;
      if (!blocked) {
        // prev (outer) merges with k (inner) if coef[prev] == coef[k] * dims[k] everywhere,
        // and no access is shifted in the outer dim
        bool ok = true;
        for (const AccessGroup& ag : g->groups) {
          if (ag.coef[prev] != ag.coef[k] * g->orig_dims[k]) ok = false;
          for (const auto& d : ag.deltas) if (d[prev] != 0) ok = false;
        }
        if (ok) { runs.back().push_back(k); merged = true; }
      }
    }
    if (!merged) runs.push_back({k});
  }
  if (runs.empty()) runs.push_back({n - 1});
  // a run (outer..inner) was built by appending inner dims; verify pairwise chain (outer vs next) held
  g->rank = (int)runs.size();
  for (int k = 0; k < MAXD; ++k) g->collapse_to[k] = -1;
  for (int r = 0; r < g->rank; ++r) {
    int64_t e = 1;
    for (int k : runs[r]) { e *= g->orig_dims[k]; g->collapse_to[k] = r; }
    g->dims[r] = e;
  }
  for (AccessGroup& ag : g->groups) {
    int64_t nc[MAXD] = {0};
    bool nz[MAXD];
    for (int r = 0; r < g->rank; ++r) { nc[r] = ag.coef[runs[r].back()]; nz[r] = ag.structural_zero[runs[r].back()]; }
    std::set<std::vector<int64_t>> nd;
    for (const auto& d : ag.deltas) {
      std::vector<int64_t> v(g->rank);
      for (int r = 0; r < g->rank; ++r) v[r] = d[runs[r].back()];
      nd.insert(v);
    }
    ag.deltas.swap(nd);
    for (int r = 0; r < MAXD; ++r) { ag.coef[r] = r < g->rank ? nc[r] : 0; ag.structural_zero[r] = r < g->rank ? nz[r] : true; }
  }
  for (int p = 0; p < nprogs; ++p)
    for (Instr& in : *progs[p])
      if (in.kind == IKind::LOAD) {
        int64_t v[MAXD] = {0};
        for (int r = 0; r < g->rank; ++r) v[r] = in.delta[runs[r].back()];
        for (int r = 0; r < MAXD; ++r) in.delta[r] = v[r];
      }
}

void put(std::string& s, int64_t v) { s.append(reinterpret_cast<const char*>(&v), sizeof(v)); }

void dump_prog(std::string& s, const std::vector<Instr>& prog, int rank) {
  for (const Instr& in : prog) {
    put(s, ((int64_t)in.kind << 48) | ((int64_t)in.op << 32) | ((int64_t)in.dtype << 16) | (int64_t)in.uniform);
    put(s, ((int64_t)(in.a + 1) << 32) | (int64_t)(in.b + 1));
    put(s, ((int64_t)(in.group + 1) << 40) | ((int64_t)(in.cslot + 1) << 20) | (int64_t)(in.phase + 1));
    if (in.kind == IKind::LOAD) for (int k = 0; k < rank; ++k) put(s, in.delta[k]);
  }
}

// Cache key: everything the generated source depends on, and nothing else (extents,
// strides, base offsets and constants are kernel arguments).
void make_signature(GroupPlan* g) {
  std::string s;
  s.reserve(256 + 32 * (g->prog.size() + g->prog1.size()));
  for (int64_t v : {(int64_t)g->kind, (int64_t)g->rank, (int64_t)g->out_dtype, (int64_t)g->out_per_row, (int64_t)g->BX, (int64_t)g->BY,
                    (int64_t)g->VR + (g->kind == GroupKind::GEMM && g->VR == 2 && g->slabs > 1 ? 1024 : 0) /* (the direct-to-LDS product kernels compile the split of K in or out) */, (int64_t)g->UC, (int64_t)g->NP, (int64_t)g->row_threads + 1024 * (int64_t)g->row_iters, (int64_t)g->xcd_remap + 2 * (int64_t)g->stage_mask + (((int64_t)g->tail) << 40) + (((int64_t)g->diag) << 44) + (((int64_t)g->cphase) << 48), (int64_t)g->red_mode + 16 * (int64_t)g->red_vec,
                    (int64_t)g->red_kept_rank, (int64_t)g->gemv_mode, (int64_t)g->LPR, (int64_t)g->KV, (int64_t)g->mat_group,
                    (int64_t)g->vec_group, (int64_t)g->nt, (int64_t)g->unroll, (int64_t)g->scan_mode + 16 * (int64_t)g->scan_vec + (g->scan_mode >= 2 ? 256 * g->scan_chunk : 0) /* (a one-pass scan's tile size is compiled in) */, (int64_t)g->out_unit, (int64_t)g->groups.size()})
    put(s, v);
  for (const AccessGroup& ag : g->groups) {
    int64_t cls = (int64_t)ag.dtype;
    bool core = g->kind == GroupKind::GEMV;
    int nd = core ? 2 : g->rank;
    for (int k = 0; k < nd; ++k) cls = cls * 4 + (ag.structural_zero[k] ? 0 : (ag.coef[k] == 1 ? 1 : 2));
    put(s, cls);
  }
  put(s, (int64_t)g->consts.size());
  for (const ConstSlot& c : g->consts) put(s, (int64_t)c.dtype);
  put(s, (int64_t)g->phases.size());
  for (const Phase& p : g->phases) put(s, ((int64_t)p.op << 40) | ((int64_t)p.in_dtype << 32) | ((int64_t)p.out_dtype << 24) | (int64_t)p.value);
  put(s, (int64_t)g->results.size());
  if (g->kind != GroupKind::MAP) { for (int r : g->results) put(s, r); dump_prog(s, g->prog, g->rank); }
  put(s, g->result1);
  dump_prog(s, g->prog1, g->rank);
  if (g->pair) { s.append("|pair|"); s.append(g->pair->signature); }
  g->signature.swap(s);
}

// The output takes part in dimension collapsing as one more access (its strides need not be
// those of a C-contiguous array when the root is written through a slice assignment).
void push_output_group(GroupPlan* g, int n) {
  AccessGroup og;
  og.leaf = nullptr;
  og.dtype = g->out_dtype;
  for (int k = 0; k < MAXD; ++k) og.structural_zero[k] = true;
  for (int k = 0; k < n; ++k) { og.coef[k] = g->out_orig_coef[k]; og.structural_zero[k] = g->orig_dims[k] == 1; }
  og.deltas.insert(std::vector<int64_t>(n, 0));
  g->groups.push_back(og);
}

void pop_output_group(GroupPlan* g) {
  for (int k = 0; k < g->rank; ++k) g->out_coef[k] = g->groups.back().coef[k];
  g->groups.pop_back();
  g->out_unit = g->out_coef[g->rank - 1] == 1 || g->dims[g->rank - 1] == 1;
}

struct Planner {
  gr_ctx* c;
  Node* root;
  const OutSpec* out = nullptr;
  std::vector<Node*> sub;                 // lazy nodes of the visited sub-DAG, ascending id
  NodeSet cuts;
  std::map<const Node*, const Node*, NodeIdLess> owner;

  void collect() {
    std::set<Node*> seen;
    std::vector<Node*> work{root};
    while (!work.empty()) {
      Node* n = work.back();
      work.pop_back();
      if (n->materialized || seen.count(n)) continue;  // a materialised node ends the walk (Section 2)
      seen.insert(n);
      for (Node* p : n->in) work.push_back(p);
    }
    sub.assign(seen.begin(), seen.end());
    std::sort(sub.begin(), sub.end(), [](Node* a, Node* b) { return a->id < b->id; });
  }

  void initial_cuts() {
    cuts.insert(root);
    for (Node* n : sub) {
      if (!c->opt_fusion && n->is_compute()) cuts.insert(n);
      if (n->kind == Kind::DOT && !small_dot(n)) {
        // operands of a contraction are materialised first; views (a transposed
        // matrix in particular) are folded into the contraction kernel instead
        for (Node* o : n->in) {
          const Node* b = strip_views(o);
          if (!b->materialized) cuts.insert(b);
        }
      }
      if (dot_as_reduce(n)) cuts.insert(n);       // evaluated as a two-stage reduction: consumers read its result
      if (n->kind == Kind::SCAN) cuts.insert(n);  // a scan is materialised (materialize_node, Section 2)
      if (n->kind == Kind::RESHAPE) cuts.insert(n);  // a reshape is a stored copy: its consumers index it under the new shape
      if (n->kind == Kind::REDUCE) {
        const Node* x = n->in[0];
        bool last_only = x->ndim >= 1;
        for (int d = 0; d < x->ndim; ++d) if (n->red_axis[d] != (d == x->ndim - 1)) last_only = false;
        if (!last_only || x->shape[x->ndim - 1] > std::min<int64_t>(c->opt_rowred_max_cols, 16384)) cuts.insert(n);
      }
    }
  }

  // Returns false (after adding a cut) if some node is reached from two roots.
  bool assign_owners() {
    owner.clear();
    for (Node* r : sub) {
      if (!cuts.count(r)) continue;
      std::vector<const Node*> work;
      NodeSet seen;
      for (Node* p : r->in) work.push_back(p);
      owner[r] = r;
      while (!work.empty()) {
        const Node* n = work.back();
        work.pop_back();
        if (n->materialized || cuts.count(n) || seen.count(n)) continue;
        seen.insert(n);
        if (n->is_compute()) {
          auto it = owner.find(n);
          if (it != owner.end() && it->second != r) { cuts.insert(n); return false; }  // multiple-use rule
          owner[n] = r;
        }
        for (Node* p : n->in) work.push_back(p);
      }
    }
    return true;
  }

  NodeSet owned_by(const Node* r) const {
    NodeSet s;
    for (const auto& kv : owner) if (kv.second == r) s.insert(kv.first);
    return s;
  }
};

void choose_map_schedule(gr_ctx* c, GroupPlan* g) {
  int64_t C = g->dims[g->rank - 1];
  int64_t R = g->rank >= 2 ? g->dims[g->rank - 2] : 1;
  int64_t outer = 1;
  for (int k = 0; k + 2 < g->rank; ++k) outer *= g->dims[k];
  g->BX = std::min(256, std::max(1, next_pow2((C + 3) / 4)));
  if (c->opt_map_bx > 0 && c->opt_map_bx <= 256 && (c->opt_map_bx & (c->opt_map_bx - 1)) == 0) g->BX = std::min<int>(g->BX, (int)c->opt_map_bx);
  bool shifted_rows = false;
  for (const AccessGroup& ag : g->groups)
    for (const auto& d : ag.deltas) if (g->rank >= 2 && d[g->rank - 2] != 0) shifted_rows = true;
  // Programs without row-shifted views (pointwise and broadcast): a wave per 256 columns and the
  // four waves of a workgroup on neighbouring row pairs, two rows per lane (measured on MI355X,
  // normalize 8192^2: 83.0 us against 85.3 with 1024 columns by four rows per workgroup; stencils
  // keep the wide tile, 96 us against 97-113)
  // Only where every row piece of 256 columns is a run of whole 256-byte blocks in every array
  // (rows of 1024 columns or more in multiples of 256, no views shifted along the columns, row
  // strides in multiples of 64 elements): a narrow tile leaves the ends of unaligned pieces to
  // other workgroups, and their partial lines cost more than the tile shape gains (x*row on
  // 8192 x 8190: 113 us narrow, 95 us wide).
  bool aligned = C >= 1024 && C % 256 == 0;
  for (const AccessGroup& ag : g->groups) {
    if (ag.structural_zero[g->rank - 1]) continue;
    if (ag.deltas.size() != 1 || ag.coef[g->rank - 1] != 1 || ag.base % 64 != 0) aligned = false;
    for (const auto& d : ag.deltas) if (d[g->rank - 1] != 0) aligned = false;
    for (int k = 0; k + 1 < g->rank; ++k) if (!ag.structural_zero[k] && ag.coef[k] % 64 != 0) aligned = false;
  }
  for (int k = 0; k + 1 < g->rank; ++k) if (g->out_coef[k] % 64 != 0) aligned = false;
  if (g->out_base % 64 != 0) aligned = false;
  const bool narrow_tile = g->rank >= 2 && R > 1 && !shifted_rows && aligned && c->opt_map_bx == 0 && g->BX > 64;
  if (narrow_tile) g->BX = 64;
  // Views shifted by at most one row up and down (a five-point sweep): 512 columns by four rows per workgroup, two
  // rows per lane (measured on MI355X against 1024 columns by four rows with four rows per lane, right-hand side of a
  // Jacobi sweep: 8192^2 92.5 against 97.6 us, 16384 x 4096 93.5 against 104.2, 4096 x 16384 92.6 against 96.8,
  // 4096^2 30.4 against 31.2, 8190^2 90.9 against 91.7; taller stencils keep the wide tile, within 1-3 % either way)
  int64_t row_lo = 0, row_hi = 0;
  for (const AccessGroup& ag : g->groups)
    for (const auto& d : ag.deltas) if (g->rank >= 2) { row_lo = std::min(row_lo, d[g->rank - 2]); row_hi = std::max(row_hi, d[g->rank - 2]); }
  const bool low_stencil = shifted_rows && row_hi - row_lo <= 2 && c->opt_map_bx == 0 && g->BX == 256;
  if (low_stencil) g->BX = 128;
  g->BY = 256 / g->BX;
  auto tiles = [&](int vr, int uc) {
    int64_t tc = (int64_t)g->BX * 4 * uc, tr = (int64_t)g->BY * vr;
    return outer * ((C + tc - 1) / tc) * ((R + tr - 1) / tr);
  };
  g->VR = 1; g->UC = 1;
  if (g->rank == 1 || R == 1) {
    for (int uc : {4, 2}) if (tiles(1, uc) >= 2048) { g->UC = uc; break; }
  } else {
    int want = narrow_tile || low_stencil ? 2 : 4;  // measured on MI355X: 4 rows per lane is the best patch for tall stencil programs and for broadcast programs on wide tiles
    // (lanes whose patch sticks out of the array take the guarded point-by-point path: with few
    // rows the patch height has to divide them)
    for (int vr = want; vr >= 2; vr >>= 1)
      if ((R % vr == 0 || R >= 16 * vr) && (tiles(vr, 1) >= 1024 || (shifted_rows && tiles(vr, 1) >= 256))) { g->VR = vr; break; }
  }
  // Operands whose contiguous dimension is the row dimension of the iteration space (transposed
  // views): lanes along the columns would read them with a stride.  A tile (64 columns by 64 or 128 rows) of such an
  // operand is loaded along its own contiguous dimension into LDS and read from there transposed.
  g->stage_mask = 0;
  g->diag = 0;
  if (g->rank >= 2 && R >= 64 && C >= 64 && c->opt_map_rows == 0 && c->opt_map_chunks == 0 && c->opt_map_bx == 0 && c->opt_stage) {
    int staged = 0;
    for (size_t gi = 0; gi < g->groups.size() && gi < 24; ++gi) {
      const AccessGroup& ag = g->groups[gi];
      if (ag.dtype == GR_I64 || ag.deltas.size() != 1) continue;
      if (ag.structural_zero[g->rank - 1] || ag.structural_zero[g->rank - 2]) continue;
      if (ag.coef[g->rank - 1] != 1 && ag.coef[g->rank - 2] == 1 && staged < 2) { g->stage_mask |= 1 << gi; ++staged; }
    }
    // (64 columns by 64 or 128 rows: the taller tile reads 512-byte runs of the operand)
    if (g->stage_mask) { g->BX = 16; g->BY = 16; g->VR = (R >= 128 && c->opt_stage_rows != 64) ? 8 : 4; g->UC = 1; g->diag = c->opt_stage_diag != 0; }
    // Such a tile writes 256-byte pieces of output rows.  Where rows do not start on 64-byte
    // boundaries the pieces of neighbouring tiles share cache lines, which only plain stores let
    // the L2 merge (measured, 8191^2 transposed: 144 us plain, 177 us with hinted stores).
    if (g->stage_mask && (g->nt & 8) && c->opt_nontemporal == 1 && (C % 16 != 0 || g->out_coef[g->rank - 2] % 16 != 0)) g->nt &= ~8;
  }
  if (c->opt_map_rows > 0 && g->rank >= 2) g->VR = (int)std::min<int64_t>(c->opt_map_rows, 16);
  if (c->opt_map_chunks > 0) g->UC = (int)std::min<int64_t>(c->opt_map_chunks, 8);
  g->xcd_remap = shifted_rows;
  // A strided destination (the box of a slice assignment, a stencil sweep writing the interior of a
  // grid) may start off a 16-byte boundary while its rows are 16-byte multiples apart: lanes then own
  // the column groups that are aligned in the OUTPUT (the first and the last group of a row are
  // partial and take the guarded path), so that a wave's vector stores cover whole cache lines.
  g->cphase = 0;
  if (g->rank >= 2 && C >= 256 && g->out_unit && g->out_dtype != GR_I64 && !g->stage_mask && g->UC == 1 && c->opt_map_phase) {
    bool rows_aligned = true;
    for (int k = 0; k + 1 < g->rank; ++k) if (g->out_coef[k] % 4 != 0) rows_aligned = false;
    if (rows_aligned) g->cphase = (int)(((g->out_base % 4) + 4) % 4);
  }
  // Narrow arrays (points, pixels: a few columns): the lanes that own the last, incomplete group
  // of four columns are a large share of all lanes (all of them below four columns).  The kernel
  // is specialised on columns mod 4 and gives those lanes straight-line code as well.
  g->tail = (g->rank >= 2 && C < 64 && (C & 3) && g->UC == 1 && !g->stage_mask) ? (int)(C & 3) : 0;
}

}  // namespace

// ---------------------------------------------------------------------------

// Operand of a contraction as an access group of its own.  The contraction kernels address it as
// base + i * coef[0] + j * coef[1]; the static shift that `load` keeps apart (a slice that starts
// at or beyond its step) is folded into the base here, and the group is never shared with another
// access: the other operand or an epilogue load may read the same array with the same map, but
// with coefficient slots that mean other dimensions or with another shift.
static int add_core_group(GroupPlan* g, const Builder& like, const Node* leaf, const IndexMap& lm) {
  GroupPlan tmp;
  std::vector<Instr> prog;
  Builder cb;
  cb.g = &tmp; cb.owned = like.owned; cb.rank = 2; cb.dims = like.dims; cb.prog = &prog;
  cb.load(leaf, lm);
  AccessGroup ag = tmp.groups[0];
  const Instr& ld = prog.back();
  for (int k = 0; k < 2; ++k) if (!ag.structural_zero[k]) ag.base += ag.coef[k] * ld.delta[k];
  ag.deltas.clear();
  ag.deltas.insert(std::vector<int64_t>(2, 0));
  g->groups.push_back(ag);
  return (int)g->groups.size() - 1;
}

static gr_status build_group(gr_ctx* c, Planner& pl, Node* r, GroupPlan* g, std::vector<Invalid>* invalid, bool force_generic = false) {
  NodeSet owned = pl.owned_by(r);
  g->root = r;
  g->out_dtype = r->dtype;
  g->nt = (int)c->opt_nontemporal;
  // An output of at least three quarters of the memory-side cache (256 MiB) is streamed out: its vector
  // stores carry the non-temporal hint as well (measured on MI355X: normalize 8192^2 93.9 ->
  // 86.7 us).  Smaller outputs stay cacheable for the sub-graph that reads them next (a 64 MiB
  // result that is consumed, or whose buffer is reused, within a few launches is 7-15 % slower
  // with hinted stores).
  // Only the value the request asked for: an intermediate result is read by the next sub-graph
  // of the same request at once.
  if (g->nt == 1 && r == pl.root && r->count() * (r->dtype == GR_I64 ? 8 : 4) >= (192ll << 20)) g->nt |= 8;

  // A root that already has data (the plain copy of an array into another buffer or through a
  // strided destination) is a map that loads it, whatever operation once produced it.
  if (r->materialized) owned.clear();

  // classify
  const Node* dot = nullptr;
  std::vector<const Node*> reds;
  for (const Node* n : owned) {
    if (n->kind == Kind::DOT && !small_dot(n)) { if (dot) { invalid->push_back({n, "second dot in one sub-graph"}); return GR_OK; } dot = n; }
    if (n->kind == Kind::REDUCE) reds.push_back(n);
  }
  if (dot && !reds.empty()) { invalid->push_back({dot, "dot mixed with a reduction"}); return GR_OK; }
  if (r->kind == Kind::RESHAPE && !r->materialized && (dot || !reds.empty())) {
    // a reshape is a row-major copy fused with pointwise producers only: reductions and contractions
    // below it are evaluated first and read as stored arrays
    if (dot) invalid->push_back({dot, "dot under a reshape"});
    for (const Node* n : reds) invalid->push_back({n, "reduction under a reshape"});
    return GR_OK;
  }

  Builder b;
  b.g = g;
  b.owned = &owned;

  if (r->kind == Kind::SCAN && !r->materialized) {
    // ---- map-scan: the operand expression is the map, the scan runs along one axis --------
    g->kind = GroupKind::SCAN;
    b.g->kind = GroupKind::SCAN;
    for (const Node* n : owned) if (n != r && (n->kind == Kind::REDUCE || (n->kind == Kind::DOT && !small_dot(n)) || n->kind == Kind::SCAN))
      invalid->push_back({n, "reduction, scan or dot under a scan"});
    if (!invalid->empty()) return GR_OK;
    const Node* x = r->in[0];
    int axis = 0;
    for (int d = 0; d < x->ndim; ++d) if (r->red_axis[d]) axis = d;
    // iteration space: the other dimensions in order, the scanned axis last
    int pos[MAXD], nk = 0;
    for (int d = 0; d < x->ndim; ++d) if (d != axis) { pos[d] = nk; g->orig_dims[nk++] = x->shape[d]; }
    pos[axis] = nk;
    g->orig_dims[nk] = x->shape[axis];
    const int n = nk + 1;
    g->orig_rank = n;
    b.rank = n; b.dims = g->orig_dims; b.prog = &g->prog;
    IndexMap xm(x->ndim);
    for (int d = 0; d < x->ndim; ++d) xm[d] = DimMap{pos[d], 1, 0};
    int v = b.eval(x, xm);
    if (!b.invalid.empty()) { *invalid = b.invalid; return GR_OK; }
    b.members_seen.insert(r);
    Phase p;
    p.op = r->op; p.in_dtype = x->dtype; p.out_dtype = r->dtype; p.value = v; p.node = r;
    g->phases.push_back(p);
    // the C-contiguous output takes part in dimension collapsing as one more access
    AccessGroup og;
    og.leaf = nullptr; og.dtype = r->dtype;
    for (int k = 0; k < MAXD; ++k) og.structural_zero[k] = true;
    { int64_t st = 1; for (int d = x->ndim - 1; d >= 0; --d) { og.coef[pos[d]] = st; og.structural_zero[pos[d]] = false; st *= x->shape[d]; } }
    og.deltas.insert(std::vector<int64_t>(n, 0));
    g->groups.push_back(og);
    std::vector<Instr>* ps[1] = {&g->prog};
    normalize_deltas(g, ps, 1, n);
    bool barrier[MAXD] = {false};
    if (nk > 0) barrier[nk - 1] = true;
    collapse_dims(g, barrier, ps, 1);
    if (g->orig_dims[n - 1] == 1 || g->collapse_to[n - 1] != g->rank - 1 || nk == 0) {
      // the scanned axis must remain the last collapsed dim even if its extent is 1
      if (g->orig_dims[n - 1] == 1) {
        bool only = true;
        for (int k = 0; k < nk; ++k) if (g->orig_dims[k] != 1) only = false;
        if (!only) { g->dims[g->rank] = 1; g->collapse_to[n - 1] = g->rank; g->rank++; }
      }
    }
    for (int k = 0; k < g->rank; ++k) g->out_coef[k] = g->groups.back().coef[k];
    g->groups.pop_back();
    const int sd = g->rank - 1;
    int64_t L = g->dims[sd], lines = 1;
    for (int k = 0; k < sd; ++k) lines *= g->dims[k];
    bool unit = g->out_coef[sd] == 1 || L == 1;
    for (const AccessGroup& ag : g->groups) if (!ag.structural_zero[sd] && ag.coef[sd] != 1) unit = false;
    g->scan_mode = unit ? 0 : 1;
    g->scan_nchunk = 1;
    g->scan_chunk = ((L + 1023) / 1024) * 1024;
    if (g->scan_mode == 0 && lines < 512 && L > 32768) {
      // long lines and few of them: reduce-then-scan over chunks (Section 3.2 refers to the
      // work-efficient scan: chunk sums, a scan of the sums, then the chunks with their offsets)
      int64_t want = std::max<int64_t>(1, 2048 / std::max<int64_t>(lines, 1));
      int64_t chunk = std::max<int64_t>(8192, (L + want - 1) / want);
      chunk = ((chunk + 1023) / 1024) * 1024;
      int64_t nch = (L + chunk - 1) / chunk;
      if (nch > 4096) { chunk = (((L + 4095) / 4096 + 1023) / 1024) * 1024; nch = (L + chunk - 1) / chunk; }
      g->scan_chunk = chunk;
      g->scan_nchunk = (int)nch;
      // 4-byte running values: one pass over the input with chained tiles of 8192 elements
      // (option "scan_one_pass" = 0 keeps the three kernels, which read the input twice)
      // tiles of 8192 elements, 20480 for lines of 2^25 elements and more (measured: 2^27 elements 200 us with 12288, 192-195 with 16384, 188 with 20480, 207 with 24576; option values from 2 to 24: 1024-element blocks per tile)
      const int64_t tile = 1024 * (c->opt_scan_one_pass >= 2 ? c->opt_scan_one_pass : (L >= ((int64_t)1 << 25) ? 20 : 8));
      if (c->opt_scan_one_pass && p.out_dtype != GR_I64 && tile <= 24576 && (L + tile - 1) / tile <= (int64_t)1 << 24) {
        g->scan_mode = 2;
        g->scan_chunk = tile;
        g->scan_nchunk = (int)((L + tile - 1) / tile);
      }
    }
    // four neighbouring lines per thread where the innermost line dimension is contiguous in every
    // array read and in the output, holds a multiple of four, and all values are 32 bits wide
    g->scan_vec = 0;
    if (g->scan_mode == 1 && sd >= 1 && g->dims[sd - 1] % 4 == 0 && g->out_coef[sd - 1] == 1 && p.in_dtype != GR_I64) {
      bool ok = true;
      for (const AccessGroup& ag : g->groups)
        if (ag.dtype == GR_I64 || (!ag.structural_zero[sd - 1] && ag.coef[sd - 1] != 1)) ok = false;
      for (const Instr& in : g->prog) if (in.dtype == GR_I64) ok = false;
      g->scan_vec = ok ? 1 : 0;
    }
    if (g->scan_vec) lines /= 4;   // threads per chunk
    // A thread walks its line eight steps at a time (eight loads in flight).  One pass over the
    // lines reads the input once and is kept down to scan_min threads (measured: 2^14 threads with
    // dwordx4 loads still beat the chunked form); below that the lines are cut into chunks so that
    // about scan_threads threads run.
    const int64_t scan_threads = c->opt_scan_threads > 0 ? c->opt_scan_threads : (g->scan_vec ? 65536 : 131072);
    const int64_t scan_min = c->opt_scan_min_threads > 0 ? c->opt_scan_min_threads : (g->scan_vec ? 16384 : 32768);
    int n_loads = 0;
    for (const Instr& in : g->prog) if (in.kind == IKind::LOAD) ++n_loads;
    if (g->scan_mode == 1 && g->scan_vec && lines > 0 && L >= 128 && c->opt_scan_one_pass && p.out_dtype != GR_I64 && n_loads <= 8) {
      // Lines of 128 positions or more, four of them per lane, 4-byte running values: ONE pass over
      // the input.  A workgroup keeps a tile of R positions along the scanned axis by W neighbouring
      // lines in registers (BX lanes across the lines, 256/BX lane groups along the axis, RPL
      // positions per lane), publishes the tile's totals and collects its offsets from the tiles
      // before it.  (Measured against a thread per four lines at every line count from 64 to 2^20:
      // the tiles win everywhere, by 5 % at 2^18 lines of 512 and by 2x at 2^16 lines of 1024.)
      const int64_t D = g->dims[sd - 1];
      int bx = 64;
      while (bx > 4 && (int64_t)bx * 4 > D) bx /= 2;   // W = 4*BX lines: at most D where D allows, at least 16
      const int ly = 256 / bx;
      const int64_t chains = (lines * 4 / D) * ((D + 4 * bx - 1) / (4 * bx));
      int rpl = n_loads <= 1 ? 32 : (n_loads <= 2 ? 16 : 8);
      while (rpl > 4 && chains * ((L + (int64_t)rpl * ly - 1) / ((int64_t)rpl * ly)) < 1024) rpl /= 2;
      const int64_t R = (int64_t)rpl * ly;
      const int64_t nch = (L + R - 1) / R;
      if (nch <= ((int64_t)1 << 20) && chains * nch <= ((int64_t)1 << 30)) {
        g->scan_mode = 3;
        g->BX = bx;
        g->scan_chunk = R;
        g->scan_nchunk = (int)nch;
        int grp = 4;
        while (grp < 64 && (int64_t)grp * grp < nch) grp *= 2;
        g->slabs = grp;   // tiles per group of the offset collection
      }
    }
    if (g->scan_mode == 1 && lines < scan_min && L >= 128) {
      // fewer lines than that: cut the lines into chunks (chunk totals, scan of the totals, chunks
      // with offsets, as above), which costs a second read of the input
      int64_t want = std::max<int64_t>(1, scan_threads / std::max<int64_t>(lines, 1));
      int64_t chunk = std::max<int64_t>(32, (L + want - 1) / want);
      int64_t nch = (L + chunk - 1) / chunk;
      if (nch > 4096) { chunk = (L + 4095) / 4096; nch = (L + chunk - 1) / chunk; }
      g->scan_chunk = chunk;
      g->scan_nchunk = (int)nch;
    }
    g->red_out = g->scan_vec ? lines * 4 : lines;
    g->red_len = L;
  } else if (dot && dot->ndim == 2) {
    // ---- matrix-matrix product on the matrix cores, with pointwise epilogue -----------------
    g->kind = GroupKind::GEMM;
    b.g->kind = GroupKind::GEMM;
    const Node* A = dot->in[0];
    const Node* B = dot->in[1];
    g->M = A->shape[0]; g->K = A->shape[1]; g->N = B->shape[1];
    if (r->ndim != 2 || r->shape[0] != g->M || r->shape[1] != g->N) { invalid->push_back({dot, "epilogue changes the shape"}); return GR_OK; }
    g->orig_rank = 2;
    g->orig_dims[0] = g->M; g->orig_dims[1] = g->N;
    b.rank = 2; b.dims = g->orig_dims; b.prog = &g->prog;
    IndexMap im(2);
    im[0] = DimMap{0, 1, 0}; im[1] = DimMap{1, 1, 0};
    int res = b.eval(r, im);
    if (!b.invalid.empty()) { *invalid = b.invalid; return GR_OK; }
    g->results.push_back(res);
    std::vector<Instr>* eps[1] = {&g->prog};
    normalize_deltas(g, eps, 1, 2);
    // operands: left in the space (m,k), right in the space (k,n); resolved through views only
    for (int side = 0; side < 2; ++side) {
      const Node* X = side == 0 ? A : B;
      int64_t cd[2] = {side == 0 ? g->M : g->K, side == 0 ? g->K : g->N};
      Builder cb;
      std::vector<Instr> scratch;
      cb.g = g; cb.owned = &owned; cb.rank = 2; cb.dims = cd; cb.prog = &scratch;
      IndexMap xm(2);
      xm[0] = DimMap{0, 1, 0}; xm[1] = DimMap{1, 1, 0};
      cb.canonicalize(X, xm);
      const Node* leaf; IndexMap lm;
      if (!resolve_to_leaf(X, xm, &leaf, &lm)) return fail(c, GR_ERR_UNSUPPORTED, "dot: operand is not materialised");
      // a private group per operand (an epilogue access or the other operand may read the same leaf
      // with the same map, but their coefficient slots mean different dimensions)
      (side == 0 ? g->mat_group : g->vec_group) = add_core_group(g, cb, leaf, lm);
      b.leaves_seen.insert(leaf);
    }
    b.members_seen.insert(dot);
    g->rank = 2;
    g->dims[0] = g->M; g->dims[1] = g->N;
    g->collapse_to[0] = 0; g->collapse_to[1] = 1;
    // few output tiles and a long contraction: split K over workgroups (about 512 of them, at
    // least 128 k per split); the partial tiles are combined by a second kernel
    g->slabs = 1;
    // columns of the output tile of one workgroup: 128, or 32 for narrow results and where the last
    // 128-wide tile would be more than half empty (measured, 65536 x 64 x 64: 14.5 us against 21.8 us;
    // 8192 x 512 x 520: 67 against 94 us; a full 128-wide tile costs about 0.3 of four 32-wide ones less)
    // (only where those empty columns are more than an eighth of the padded width: 4000 columns keep 128-wide tiles)
    {
      const int64_t padded = ((g->N + 127) / 128) * 128, pad = padded - g->N;
      g->BX = (g->N <= 96 || (pad >= 64 && pad * 8 > padded)) ? 32 : 128;
    }
    if (c->opt_gemm_bn == 32 || c->opt_gemm_bn == 128) g->BX = (int)c->opt_gemm_bn;
    // k extent of one step of the main loop (one barrier per step): 16, or 32 on request
    g->UC = (g->BX == 128 && c->opt_gemm_kstep == 32) ? 2 : 1;
    {
      const int64_t tiles = ((g->M + 127) / 128) * ((g->N + g->BX - 1) / g->BX);
      if (tiles > 0 && tiles < 192 && g->K >= 256) {
        int64_t ks = std::min<int64_t>(512 / tiles, g->K / 128);
        if (ks >= 2) g->slabs = (int)std::min<int64_t>(ks, 256);
      }
      if (c->opt_gemm_split >= 1) g->slabs = (int)std::min<int64_t>(std::min<int64_t>(c->opt_gemm_split, 256), std::max<int64_t>(1, g->K / 32));
    }
    // Large products of operands that are contiguous along one of their two dimensions: 256 x 256 tiles, one
    // workgroup per compute unit, tiles loaded straight into LDS (BX = 256 selects that kernel).  It needs
    // whole steps of 16 values of k, a result that fills most of its rounds over the 256 compute units, and lane offsets
    // of 32 bits: an operand contiguous along k is loaded in rows of its
    // other dimension (row stride below 2^21 elements), one contiguous along its other dimension in rows of k
    // (stride below 2^24).
    {
      const AccessGroup& ag = g->groups[g->mat_group];
      const AccessGroup& bg = g->groups[g->vec_group];
      const int64_t tiles = ((g->M + 255) / 256) * ((g->N + 255) / 256), rounds = (tiles + 255) / 256;
      // other: the extent of the operand's dimension that is not k (a multiple of four where that dimension is the
      // contiguous one: its elements are loaded in groups of four)
      auto fits = [](const AccessGroup& x, int kdim, int64_t other) {   // kdim: which of the operand's two dimensions is k
        if (x.structural_zero[0] || x.structural_zero[1]) return false;
        const int64_t sk = x.coef[kdim], so = x.coef[1 - kdim];
        if (sk == 1 && so != 1) return so >= 16 && so < ((int64_t)1 << 21);
        if (so == 1 && sk != 1) return sk >= 128 && sk < ((int64_t)1 << 24) && other % 4 == 0;
        return false;
      };
      // Edge tiles are whole tiles of work: the result must fill 85 % of its rounds over the 256 compute units, 65 %
      // where M or N is not a multiple of 128 (the 128-wide kernel's guarded edge tiles make it slower there; measured
      // on 4000^3: 136 against 97 TFLOP/s, 8000^3: 144 against 114, 10000 x 4096 x 10000, seven rounds 85 % full: 126 against 117).
      const int64_t need = (g->M % 128 == 0 && g->N % 128 == 0) ? 17 : 13;
      const bool direct = c->opt_gemm_big && c->opt_gemm_bn == 0 && g->K % 16 == 0 && g->K >= 32 && fits(ag, 1, g->M) && fits(bg, 0, g->N);
      // (with K split over workgroups every split has to hold whole steps of k and at least two of them: the last one is the shortest)
      const bool split_ok = g->slabs == 1 || g->K - (g->slabs - 1) * gemm_split_extent(g->K, g->slabs) >= 32;
      if (direct && g->slabs == 1 && g->M >= 256 && g->N >= 256 && g->M * g->N * 20 >= rounds * 256 * 65536 * need) {
        g->BX = 256;
        g->VR = 2;   // (marks the kernels whose tiles go straight into LDS)
        g->UC = 1;
      } else if (direct && g->BX == 128 && g->M >= 128 && g->N >= 128 && c->opt_gemm_split == 0) {
        // The same kernel with 128 x 128 tiles, up to three workgroups per compute unit, and K divided over `slabs`
        // workgroups per tile where that fills the compute units more evenly or at all.  The count is the one with the
        // lowest cost in a model fitted to measurements (microseconds): rounds of 256 workgroups times the steps of one
        // workgroup at 0.95 per step (1.1 where compute units hold a single workgroup, which has nobody to overlap its
        // barriers with), plus, for a split product, 6 for the second launch and the traffic of the partial tiles at
        // 5 TB/s.  A larger count has to beat a smaller one by 3 %.  Every split holds at least 128 values of k, the last
        // one at least two steps; the partial tiles stay below 1 GiB (within the static scratch array for a request that must not
        // allocate).
        // (measured, split chosen / one workgroup per tile / the kernel that stages through registers with its own
        // split: 1024^3 30 / 68 / 38 us, 1536^3 77 / 98 / 90, 3072^3 442 / 525 / 598, 8192 x 256 x 8192 273 / 499 / 306,
        // 1024 x 1024 x 8192 139 / 493 / 159, 512 x 512 x 16384 80 / 976 / 89)
        const int64_t tiles128 = ((g->M + 127) / 128) * ((g->N + 127) / 128);
        const int64_t room = c->plan_static ? (int64_t)(c->static_cap / sizeof(float)) : (int64_t)1 << 28;   // floats of partial tiles
        double best = 0;
        int best_ks = 0;
        for (int ks = 1; ks <= 64; ++ks) {
          const int64_t kch = gemm_split_extent(g->K, ks);
          if (ks > 1 && (kch < 128 || g->K - (ks - 1) * kch < 32 || (int64_t)ks * g->M * g->N > room)) continue;
          const int64_t wgs = tiles128 * ks, rnd = (wgs + 255) / 256, steps = (kch + 15) / 16;
          const double cost = (double)rnd * (double)steps * (wgs <= 256 ? 1.1 : 0.95) + (ks > 1 ? 6.0 + (double)ks * (double)g->M * (double)g->N * 8.0 / 5e6 : 0.0);
          if (best_ks == 0 || cost < best * 0.97) { best = cost; best_ks = ks; }
        }
        g->slabs = best_ks;
        g->VR = 2;
        g->UC = 1;
      } else if (direct && split_ok && g->BX == 128 && g->M >= 128 && g->N >= 128) {
        // (a number of workgroups per tile set by option "gemm_split")
        g->VR = 2;
        g->UC = 1;
      }
    }
  } else if (dot && !(dot == r && dot_as_reduce(dot) && c->opt_fusion)) {
    // ---- contraction with pointwise epilogue ------------------------------
    g->kind = GroupKind::GEMV;
    const Node* A = dot->in[0];
    const Node* v = dot->in[1];
    g->K = v->shape[0];
    g->M = A->ndim == 2 ? A->shape[0] : 1;
    if (r->ndim != dot->ndim || (dot->ndim == 1 && r->shape[0] != dot->shape[0])) { invalid->push_back({dot, "epilogue changes the shape"}); return GR_OK; }
    g->orig_rank = 1;
    g->orig_dims[0] = g->M;
    b.rank = 1;
    b.dims = g->orig_dims;
    b.prog = &g->prog;
    IndexMap im(r->ndim);
    for (int d = 0; d < r->ndim; ++d) im[d] = DimMap{d, 1, 0};
    int res = b.eval(r, im);
    if (!b.invalid.empty()) { *invalid = b.invalid; return GR_OK; }
    g->results.push_back(res);
    // core operands, in the 2-D space (m, k); resolved through views only
    int64_t core_dims[2] = {g->M, g->K};
    Builder cb;
    cb.g = g; cb.owned = &owned; cb.rank = 2; cb.dims = core_dims;
    std::vector<Instr> scratch;
    cb.prog = &scratch;
    const Node* leaf; IndexMap lm;
    IndexMap am(A->ndim);
    if (A->ndim == 2) { am[0] = DimMap{0, 1, 0}; am[1] = DimMap{1, 1, 0}; } else am[0] = DimMap{1, 1, 0};
    cb.canonicalize(A, am);
    if (!resolve_to_leaf(A, am, &leaf, &lm)) return fail(c, GR_ERR_UNSUPPORTED, "dot: matrix operand is not materialised");
    // the epilogue's groups use 1-D coefficients; core groups are appended with (m,k) coefficients
    g->mat_group = add_core_group(g, cb, leaf, lm);
    b.leaves_seen.insert(leaf);
    IndexMap vm(1);
    vm[0] = DimMap{1, 1, 0};
    cb.canonicalize(v, vm);
    if (!resolve_to_leaf(v, vm, &leaf, &lm)) return fail(c, GR_ERR_UNSUPPORTED, "dot: vector operand is not materialised");
    g->vec_group = add_core_group(g, cb, leaf, lm);
    b.leaves_seen.insert(leaf);
    b.members_seen.insert(dot);
    g->rank = 1;
    g->dims[0] = g->M;
    g->collapse_to[0] = 0;
    const AccessGroup& mg = g->groups[g->mat_group];
    if (mg.coef[1] == 1 || g->K == 1) g->gemv_mode = 0;
    else if (mg.coef[0] == 1) g->gemv_mode = 1;
    else g->gemv_mode = 0;  // strided both ways: row-dot with scalar loads
    if (g->gemv_mode == 0) {
      g->LPR = g->K >= 2048 ? 64 : 16;
      int64_t per = (g->K + (int64_t)g->LPR * 4 - 1) / ((int64_t)g->LPR * 4);
      g->KV = (int)std::min<int64_t>(std::max<int64_t>(per, 1), 8);
    } else {
      g->BX = std::min(256, std::max(16, next_pow2((g->M + 3) / 4)));  // lanes across the output index
      g->BY = 256 / g->BX;
      int64_t colblocks = std::max<int64_t>(1, (g->M + (int64_t)g->BX * 4 - 1) / ((int64_t)g->BX * 4));
      // about one workgroup per CU measured best on MI355X (256 slabs: 78 us for 512 MiB, 1024: 85 us),
      // and fewer partial vectors make the second stage cheaper
      int64_t rows_per_slab = std::max<int64_t>((int64_t)g->BY * 8, (g->K + 255) / 256);
      int64_t slabs = std::max<int64_t>(1, (g->K + rows_per_slab - 1) / rows_per_slab);
      slabs = std::min<int64_t>(slabs, std::max<int64_t>(1, 256 / colblocks));
      if (c->opt_gemv_slabs > 0) slabs = std::min<int64_t>(c->opt_gemv_slabs, std::max<int64_t>(1, g->K));
      g->slabs = (int)slabs;
      g->unroll = c->opt_gemv_unroll == 16 ? 16 : (c->opt_gemv_unroll == 4 ? 4 : 8);
    }
    std::vector<Instr>* ps[1] = {&g->prog};
    // epilogue groups only: core groups carry no deltas
    normalize_deltas(g, ps, 1, 1);
  } else if (!reds.empty() || dot) {
    // Decide between row-resident and generic reduction.
    bool generic = dot != nullptr || force_generic;   // (a contraction planned as a reduction, see dot_as_reduce)
    if (r->kind == Kind::REDUCE) {
      const Node* x = r->in[0];
      bool last_only = x->ndim >= 1;
      for (int d = 0; d < x->ndim; ++d) if (r->red_axis[d] != (d == x->ndim - 1)) last_only = false;
      if (!last_only || x->shape[x->ndim - 1] > std::min<int64_t>(c->opt_rowred_max_cols, 16384)) generic = true;
    }
    if (generic) {
      // ---- generic reduction root: kept dims first, reduced dims last -----
      g->kind = GroupKind::REDUCE;
      for (const Node* n : reds) if (n != r) { invalid->push_back({n, "nested reduction under a generic reduction"}); }
      if (!invalid->empty()) return GR_OK;
      const Node* x = r->in[0];
      int pos[MAXD];
      int nk = 0;
      int v = -1;
      if (dot) {
        // iteration space (m, k) or (k): value A[m,k] * v[k], summed over k
        const Node* A = dot->in[0];
        const Node* vec = dot->in[1];
        if (A->ndim == 2) g->orig_dims[nk++] = A->shape[0];
        g->red_kept_rank = nk;
        g->orig_dims[nk] = vec->shape[0];
        g->orig_rank = nk + 1;
        b.rank = g->orig_rank; b.dims = g->orig_dims; b.prog = &g->prog;
        b.g->kind = GroupKind::REDUCE;
        int ids[2];
        for (int side = 0; side < 2; ++side) {
          const Node* X = side == 0 ? A : vec;
          IndexMap xm(X->ndim);
          if (X->ndim == 2) { xm[0] = DimMap{0, 1, 0}; xm[1] = DimMap{1, 1, 0}; } else xm[0] = DimMap{nk, 1, 0};
          b.canonicalize(X, xm);
          const Node* leaf; IndexMap lm;
          if (!resolve_to_leaf(X, xm, &leaf, &lm)) return fail(c, GR_ERR_UNSUPPORTED, "dot: operand is not materialised");
          ids[side] = b.load(leaf, lm);
        }
        Instr mul;
        mul.kind = IKind::BINARY; mul.op = GR_MUL; mul.dtype = GR_F32; mul.a = ids[0]; mul.b = ids[1];
        v = b.value_number(mul);
      } else {
      for (int d = 0; d < x->ndim; ++d) if (!r->red_axis[d]) { pos[d] = nk; g->orig_dims[nk++] = x->shape[d]; }
      g->red_kept_rank = nk;
      int nr = nk;
      for (int d = 0; d < x->ndim; ++d) if (r->red_axis[d]) { pos[d] = nr; g->orig_dims[nr++] = x->shape[d]; }
      g->orig_rank = nr;
      if (nr == 0) { g->orig_rank = 1; g->orig_dims[0] = 1; }
      b.rank = g->orig_rank; b.dims = g->orig_dims; b.prog = &g->prog;
      IndexMap xm(x->ndim);
      for (int d = 0; d < x->ndim; ++d) xm[d] = DimMap{pos[d], 1, 0};
      b.g->kind = GroupKind::REDUCE;
      v = b.eval(x, xm);
      }
      if (!b.invalid.empty()) { *invalid = b.invalid; return GR_OK; }
      b.members_seen.insert(r);
      Phase p;
      p.op = dot ? (int)GR_SUM : r->op; p.in_dtype = x->dtype; p.out_dtype = r->dtype; p.value = v; p.node = r;
      g->phases.push_back(p);
      std::vector<Instr>* ps[1] = {&g->prog};
      normalize_deltas(g, ps, 1, g->orig_rank);
      bool barrier[MAXD] = {false};
      if (nk > 0 && nk < g->orig_rank) barrier[nk - 1] = true;
      // kept/reduced boundary must survive extent-1 drops: recompute kept rank after collapsing
      collapse_dims(g, barrier, ps, 1);
      int kept_rank = 0;
      for (int k = 0; k < nk; ++k) if (g->collapse_to[k] >= 0) kept_rank = std::max(kept_rank, g->collapse_to[k] + 1);
      g->red_kept_rank = kept_rank;
      g->red_out = 1; g->red_len = 1;
      for (int k = 0; k < g->rank; ++k) (k < kept_rank ? g->red_out : g->red_len) *= g->dims[k];
      if (nk == g->orig_rank || (kept_rank == g->rank)) {
        // nothing left to reduce after dropping extent-1 dims: treat the single point as the reduced range
        g->red_len = 1;
      }
      // mode 0 (a thread per output) when consecutive outputs are consecutive in memory, mode 1
      // (a workgroup per output, lanes along the reduced range) when the reduced range is
      bool kept_unit = false, red_unit = false;
      for (const AccessGroup& ag : g->groups) {
        if (kept_rank > 0 && ag.coef[kept_rank - 1] == 1) kept_unit = true;
        if (g->rank > kept_rank && ag.coef[g->rank - 1] == 1) red_unit = true;
      }
      g->red_mode = (kept_unit && !red_unit) ? 0 : ((red_unit && !kept_unit) ? 1 : (g->red_out >= 4096 ? 0 : 1));
      // a handful of outputs (column sums of an array of points): a thread per output would leave
      // most lanes idle, so the lanes go along the reduced range even though it is strided
      if (g->red_mode == 0 && g->red_out < 64 && g->red_len >= 4096) g->red_mode = 1;
      // split the reduced range so that about 2048 workgroups run (two-stage reduction, Section 3.2)
      // mode 0 with four consecutive outputs per thread: the innermost kept dimension is contiguous
      // (or absent) in every array read, holds a multiple of four, and all values are 32 bits wide
      g->red_vec = 0;
      if (g->red_mode == 0 && kept_rank >= 1 && g->dims[kept_rank - 1] % 4 == 0 && p.in_dtype != GR_I64) {
        bool ok = true;
        for (const AccessGroup& ag : g->groups)
          if (ag.dtype == GR_I64 || (!ag.structural_zero[kept_rank - 1] && ag.coef[kept_rank - 1] != 1)) ok = false;
        for (const Instr& in : g->prog) if (in.dtype == GR_I64) ok = false;
        g->red_vec = ok ? 1 : 0;
      }
      // mode 1 over several reduced dimensions: four consecutive elements per lane as long as they
      // cannot straddle the innermost one
      if (g->red_mode == 1 && g->rank > kept_rank + 1 && g->dims[g->rank - 1] % 4 == 0) g->red_vec = 1;
      int64_t units = g->red_mode == 0 ? ((g->red_vec ? g->red_out / 4 : g->red_out) + 255) / 256 : g->red_out;
      // measured on MI355X (column sums of 8192^2): fewer, longer chunks win once a thread streams
      // dwordx4 rows (32 splits: 53 us, 128 splits: 61 us, 512 splits: 72 us)
      int64_t min_chunk = g->red_mode == 0 ? (g->red_vec ? 256 : 128) : 256 * 16;
      const int64_t target = 2048;
      int64_t nsplit = std::min<int64_t>(std::max<int64_t>(1, target / std::max<int64_t>(units, 1)), std::max<int64_t>(1, g->red_len / min_chunk));
      g->slabs = (int)std::min<int64_t>(nsplit, 4096);
    } else {
      // ---- row-resident reductions fused with producers and consumers -----
      g->kind = GroupKind::ROWRED;
      // the reduction recorded last (nearest to the root, possibly the root itself) fixes the row
      // space; reductions over any other space become sub-graphs of their own
      const Node* x = reds.back()->in[0];
      for (const Node* n : reds) {
        const Node* xo = n->in[0];
        bool same = xo->ndim == x->ndim;
        for (int d = 0; same && d < x->ndim; ++d) if (xo->shape[d] != x->shape[d]) same = false;
        if (!same) invalid->push_back({n, "reductions over different row spaces"});
      }
      if (!invalid->empty()) return GR_OK;
      int n = x->ndim;
      g->orig_rank = n;
      for (int d = 0; d < n; ++d) g->orig_dims[d] = x->shape[d];
      // root shape must be the row space, or one value per row
      bool full = r->ndim == n, per_row_keep = r->ndim == n, per_row_drop = r->ndim == n - 1;
      for (int d = 0; d < n; ++d) {
        if (full && r->shape[d] != x->shape[d]) full = false;
        if (per_row_keep && r->shape[d] != (d == n - 1 ? 1 : x->shape[d])) per_row_keep = false;
        if (per_row_drop && d < n - 1 && r->shape[d] != x->shape[d]) per_row_drop = false;
      }
      if (x->shape[n - 1] == 1) per_row_keep = false;  // degenerate: full covers it
      if (!full && !per_row_keep && !per_row_drop) {
        for (const Node* q : reds) invalid->push_back({q, "consumer shape differs from the row space"});
        return GR_OK;
      }
      g->out_per_row = !full;
      b.rank = n; b.dims = g->orig_dims; b.prog = &g->prog;
      IndexMap im(r->ndim);
      for (int d = 0; d < r->ndim; ++d) im[d] = DimMap{d, 1, 0};
      int res = b.eval(r, im);
      if (!b.invalid.empty()) { *invalid = b.invalid; return GR_OK; }
      g->results.push_back(res);
      std::vector<Instr>* ps[1] = {&g->prog};
      normalize_deltas(g, ps, 1, n);
      bool barrier[MAXD] = {false};
      if (n >= 2) barrier[n - 2] = true;  // never merge rows into the reduced axis
      collapse_dims(g, barrier, ps, 1);
      // the reduced axis must remain the last collapsed dim even if its extent is 1
      if (g->orig_dims[n - 1] == 1) {
        g->dims[g->rank] = 1;
        g->collapse_to[n - 1] = g->rank;
        g->rank++;
        if (g->rank == 2 && g->dims[0] == 1 && g->collapse_to[0] < 0 && n == 1) {}
      }
      int64_t C = g->dims[g->rank - 1];
      // few vec4 positions per lane keep the register count low and the occupancy high
      // (measured on MI355X for 4096-float rows: 256 lanes 93 us, 128 lanes 96 us, 64 lanes 104 us)
      // lanes per row: enough for one to four dwordx4 positions per lane; very short rows share a
      // wave between many rows instead of leaving most of 16 lanes idle
      g->row_threads = C <= 4 ? 1 : (C <= 8 ? 2 : (C <= 16 ? 4 : (C <= 32 ? 8 : (C <= 256 ? 16 : (C <= 1024 ? 64 : (C <= 2048 ? 128 : 256))))));
      if (c->opt_rowred_threads == 16 || c->opt_rowred_threads == 64 || c->opt_rowred_threads == 128 || c->opt_rowred_threads == 256)
        if (C <= c->opt_rowred_threads * 64) g->row_threads = (int)c->opt_rowred_threads;  // at most 16 positions per lane
      g->NP = (int)std::max<int64_t>(1, (C + (int64_t)g->row_threads * 4 - 1) / ((int64_t)g->row_threads * 4));
      // Rows that run along a strided axis of every array read while another axis is the contiguous
      // one (an array stored transposed): lanes along such a row would each touch another cache
      // line.  The reductions are evaluated by the generic kernel instead, which gives a thread
      // to each output and walks the lanes along the contiguous axis.
      if (g->row_threads > 1) {
        const int cd = g->rank - 1;
        bool inner_unit = false, outer_unit = false;
        for (const AccessGroup& ag : g->groups) {
          if (!ag.structural_zero[cd] && ag.coef[cd] == 1) inner_unit = true;
          for (int k = 0; k < cd; ++k) if (!ag.structural_zero[k] && ag.coef[k] == 1 && g->dims[k] > 1) outer_unit = true;
        }
        if (!inner_unit && outer_unit) {
          if (reds.size() == 1 && reds[0] == r) {
            *g = GroupPlan();
            return build_group(c, pl, r, g, invalid, true);
          }
          for (const Node* n : reds) if (n != r) invalid->push_back({n, "reduction along a strided axis"});
          if (!invalid->empty()) return GR_OK;
        }
      }
      // Short rows (up to 64 elements) reduced to one value each: a wave that owns only 4 to 64 rows lives about as long as
      // its loads take, and the waves a SIMD can hold then bound the rate.  Each lane group takes four
      // rows, the loads of all four in flight together, the four results stored at the end.
      int64_t rows = 1;
      for (int k = 0; k + 1 < g->rank; ++k) rows *= g->dims[k];
      g->row_iters = (g->out_per_row && C <= 64 && rows >= (int64_t)1 << 18 && c->opt_rowred_rows != 1) ? 4 : 1;  // (measured: 2 and 8 rows are no better, 256-element rows lose)
      if (c->opt_rowred_rows > 1 && g->out_per_row && g->row_threads <= 64) g->row_iters = (int)std::min<int64_t>(c->opt_rowred_rows, 8);
    }
  } else {
    // ---- map ----------------------------------------------------------------
    g->kind = GroupKind::MAP;
    for (const Node* n : reds) invalid->push_back({n, "reduction inside a map sub-graph"});
    if (!invalid->empty()) return GR_OK;
    // A reshape root is the row-major copy of its operand: the sub-graph iterates over the operand's
    // index space and writes a C-contiguous buffer, which is the result under either shape.
    const Node* src = map_source(r);
    int n = std::max(src->ndim, 1);
    g->orig_rank = n;
    if (src->ndim == 0) g->orig_dims[0] = 1;
    for (int d = 0; d < src->ndim; ++d) g->orig_dims[d] = src->shape[d];
    IndexMap im(src->ndim);
    for (int d = 0; d < src->ndim; ++d) im[d] = DimMap{d, 1, 0};
    // Single-point program: enough to learn the accesses, fix the schedule and key the
    // kernel cache.  The per-lane patch program is a function of exactly these and is only
    // built when the cache misses (expand_patch).
    b.rank = n; b.dims = g->orig_dims; b.prog = &g->prog1;
    g->result1 = b.eval(src, im);
    if (src != r) b.members_seen.insert(r);
    if (!b.invalid.empty()) { *invalid = b.invalid; return GR_OK; }
    // where the elements go: a C-contiguous buffer, or the strided destination of a slice assignment
    // (whose strides are given in the root's own shape: not for a reshape root)
    if (r == pl.root && pl.out && r->ndim > 0 && src == r) {
      g->out_base = pl.out->base;
      for (int d = 0; d < r->ndim; ++d) g->out_orig_coef[d] = pl.out->strides[d];
    } else {
      int64_t st = 1;
      for (int d = n - 1; d >= 0; --d) { g->out_orig_coef[d] = st; st *= g->orig_dims[d]; }
    }
    push_output_group(g, n);
    std::vector<Instr>* ps[1] = {&g->prog1};
    normalize_deltas(g, ps, 1, n);
    bool barrier[MAXD] = {false};
    collapse_dims(g, barrier, ps, 1);
    pop_output_group(g);
    choose_map_schedule(c, g);
    g->owned = owned;
  }

  for (const Node* n : b.members_seen) g->members.push_back(n);
  std::sort(g->members.begin(), g->members.end(), [](const Node* a, const Node* b2) { return a->id < b2->id; });
  for (const Node* n : b.leaves_seen) g->leaves.push_back(n);
  std::sort(g->leaves.begin(), g->leaves.end(), [](const Node* a, const Node* b2) { return a->id < b2->id; });
  make_signature(g);
  return GR_OK;
}

// Builds the patch program of a MAP sub-graph: the point function evaluated at every
// point of the per-lane patch (VR rows x UC chunks of 4 columns), with values shared
// between points (broadcast operands, overlapping slice views) computed once.
gr_status expand_patch(gr_ctx* c, GroupPlan* g) {
  if (g->kind != GroupKind::MAP || !g->prog.empty()) return GR_OK;
  Node* r = g->root;
  const int n = g->orig_rank;
  // innermost original dims of the last two collapsed dims carry the patch shifts
  int col_dim = -1, row_dim = -1;
  for (int k = 0; k < n; ++k) {
    if (g->collapse_to[k] == g->rank - 1) col_dim = k;
    if (g->rank >= 2 && g->collapse_to[k] == g->rank - 2) row_dim = k;
  }
  if (col_dim < 0) col_dim = n - 1;
  GroupPlan tmp;
  tmp.kind = GroupKind::MAP;
  tmp.root = r;
  tmp.orig_rank = n;
  for (int k = 0; k < n; ++k) tmp.orig_dims[k] = g->orig_dims[k];
  tmp.consts = g->consts;
  Builder b;
  b.g = &tmp; b.owned = &g->owned; b.rank = n; b.dims = tmp.orig_dims; b.prog = &tmp.prog;
  const Node* src = map_source(r);
  IndexMap im(src->ndim);
  for (int d = 0; d < src->ndim; ++d) im[d] = DimMap{d, 1, 0};
  const bool was_planned = r->planned;  // the root is computed here, not read
  r->planned = false;
  for (int v = 0; v < g->VR; ++v)
    for (int u = 0; u < g->UC; ++u)
      for (int j = 0; j < 4; ++j) {
        IndexMap pm = im;
        for (int d = 0; d < src->ndim; ++d) {
          if (d == col_dim) pm[d].off += (int64_t)u * g->BX * 4 + j;
          if (d == row_dim) pm[d].off += v;
        }
        // shifted points are evaluated as if the root were larger; the root's own extent-1
        // dims stay canonicalised to index 0, which is right: such dims carry no shift
        tmp.results.push_back(b.eval(src, pm));
      }
  r->planned = was_planned;
  if (!b.invalid.empty()) return fail(c, GR_ERR_UNSUPPORTED, "map: patch expansion met an unexpected node");
  tmp.out_dtype = g->out_dtype;
  for (int k = 0; k < n; ++k) tmp.out_orig_coef[k] = g->out_orig_coef[k];
  push_output_group(&tmp, n);
  std::vector<Instr>* ps[1] = {&tmp.prog};
  normalize_deltas(&tmp, ps, 1, n);
  bool barrier[MAXD] = {false};
  // the patch shifts touch only dims that are innermost in their runs, so the collapse
  // decision of the single-point program is reproduced
  collapse_dims(&tmp, barrier, ps, 1);
  pop_output_group(&tmp);
  bool same = tmp.rank == g->rank && tmp.groups.size() == g->groups.size() && tmp.consts.size() == g->consts.size();
  for (size_t i = 0; same && i < tmp.groups.size(); ++i)
    if (tmp.groups[i].ident != g->groups[i].ident || tmp.groups[i].base != g->groups[i].base) same = false;
  if (!same) {
    std::ostringstream m;
    m << "map: patch expansion disagrees with the single-point program (rank " << tmp.rank << "/" << g->rank << ", groups "
      << tmp.groups.size() << "/" << g->groups.size() << ", consts " << tmp.consts.size() << "/" << g->consts.size() << ")";
    return fail(c, GR_ERR_UNSUPPORTED, m.str());
  }
  g->prog.swap(tmp.prog);
  g->results.swap(tmp.results);
  return GR_OK;
}

// A row-dot contraction z = A.v whose (epilogue) result r is the vector operand of the
// column-accumulate contraction A^T.r over the same matrix needs the matrix only once: the
// two sub-graphs become one kernel pass (the row stays in registers between the two
// contractions).  This goes one step further than the paper, which runs every contraction
// as its own library call; the sub-graph list, the materialised nodes and the values are
// the same.
static void fuse_gemv_pairs(gr_ctx* c, Plan* plan) {
  if (!c->opt_gemv_pair || !c->opt_fusion) return;
  for (size_t i = 0; i + 1 < plan->groups.size(); ++i) {
    GroupPlan& A = *plan->groups[i];
    GroupPlan& B = *plan->groups[i + 1];
    if (A.kind != GroupKind::GEMV || B.kind != GroupKind::GEMV || A.gemv_mode != 0 || B.gemv_mode != 1) continue;
    const AccessGroup& ma = A.groups[A.mat_group];
    const AccessGroup& mb = B.groups[B.mat_group];
    const AccessGroup& vb = B.groups[B.vec_group];
    bool same_matrix = ma.leaf == mb.leaf && ma.base == mb.base && ma.coef[1] == 1 && mb.coef[0] == 1 && ma.coef[0] == mb.coef[1] &&
                       A.M == B.K && A.K == B.M;
    bool feeds = vb.leaf == A.root && vb.base == 0 && vb.coef[1] == 1;
    if (!same_matrix || !feeds || A.K > 2048 || A.M < 1) continue;
    A.LPR = A.K <= 512 ? 16 : 64;
    A.KV = (int)std::max<int64_t>(1, (A.K + (int64_t)A.LPR * 4 - 1) / ((int64_t)A.LPR * 4));
    int rpb = 256 / A.LPR;
    int64_t slabs = std::min<int64_t>(512, (A.M + rpb - 1) / rpb);  // measured: 256 -> 115 us, 512 -> 94 us, 1024 -> 96 us, 4096 -> 109 us
    if (c->opt_gemv_slabs > 0) slabs = std::min<int64_t>(c->opt_gemv_slabs, (A.M + rpb - 1) / rpb);
    A.slabs = (int)std::max<int64_t>(1, slabs);
    B.slabs = A.slabs;
    A.gemv_mode = 2;
    A.pair = std::move(plan->groups[i + 1]);
    plan->groups.erase(plan->groups.begin() + i + 1);
    make_signature(&A);
  }
}

gr_status make_plan_uncached(gr_ctx* c, Node* root, Plan* plan) {
  if (root->kind == Kind::SCALAR) return fail(c, GR_ERR_UNSUPPORTED, "a bare scalar cannot be materialised");
  Planner pl;
  pl.c = c;
  pl.root = root;
  pl.out = plan->out;
  pl.collect();
  pl.initial_cuts();
  for (int iter = 0; iter < 10000; ++iter) {
    if (!pl.assign_owners()) continue;
    clear_planned(plan);
    plan->groups.clear();
    std::vector<Invalid> invalid;
    bool restart = false;
    std::vector<Node*> order;
    for (Node* n : pl.sub) if (pl.cuts.count(n)) order.push_back(n);
    if (!pl.cuts.count(root) || root->materialized) order.push_back(root);  // root with data: a plain copy
    std::sort(order.begin(), order.end(), [](Node* a, Node* b) { return a->id < b->id; });
    order.erase(std::unique(order.begin(), order.end()), order.end());
    for (Node* r : order) {
      std::unique_ptr<GroupPlan> g(new GroupPlan());
      gr_status st = build_group(c, pl, r, g.get(), &invalid);
      if (st != GR_OK) { clear_planned(plan); plan->groups.clear(); return st; }
      if (!invalid.empty()) {
        bool added = false;
        for (const Invalid& iv : invalid) if (pl.cuts.insert(iv.node).second) added = true;
        if (!added) { clear_planned(plan); plan->groups.clear(); return fail(c, GR_ERR_UNSUPPORTED, "cannot plan: " + invalid[0].why); }
        restart = true;
        break;
      }
      plan->groups.push_back(std::move(g));
      if (!r->materialized) {
        // later sub-graphs read this node as a C-contiguous leaf
        r->planned = true;
        int64_t s = 1;
        for (int d = r->ndim - 1; d >= 0; --d) { r->strides[d] = s; s *= r->shape[d]; }
        r->offset = 0;
        plan->planned_nodes.push_back(r);
      }
    }
    if (!restart) {
      plan->out_honoured = !plan->out || (!plan->groups.empty() && plan->groups.back()->root == root && plan->groups.back()->kind == GroupKind::MAP &&
                                          map_source(root) == root);
      fuse_gemv_pairs(c, plan);
      return GR_OK;
    }
  }
  clear_planned(plan);
  plan->groups.clear();
  return fail(c, GR_ERR_UNSUPPORTED, "planner did not converge");
}

void clear_planned(Plan* plan) {
  for (Node* n : plan->planned_nodes) n->planned = false;
  plan->planned_nodes.clear();
}

std::string describe_plan(const Plan& plan) {
  std::ostringstream s;
  int i = 0;
  for (const auto& gp : plan.groups) {
    const GroupPlan& g = *gp;
    const char* kn = g.kind == GroupKind::MAP ? "MAP" : g.kind == GroupKind::ROWRED ? "ROWRED" : g.kind == GroupKind::REDUCE ? "REDUCE" : g.kind == GroupKind::SCAN ? "SCAN" : g.kind == GroupKind::GEMM ? "GEMM" : "GEMV";
    s << '#' << i++ << ' ' << kn << " root=" << g.root->id << " shape=(";
    for (int d = 0; d < g.root->ndim; ++d) s << (d ? "," : "") << g.root->shape[d];
    s << ") iter=(";
    for (int d = 0; d < g.rank; ++d) s << (d ? "," : "") << g.dims[d];
    s << ") members=[";
    bool first = true;
    for (const Node* n : g.members) {
      if (n->is_view()) continue;
      s << (first ? "" : ",") << n->id << ':' << node_label(n);
      first = false;
    }
    s << "] leaves=[";
    first = true;
    for (const Node* n : g.leaves) { s << (first ? "" : ",") << n->id; first = false; }
    s << "] loads=" << [&] { int k = 0; for (const Instr& in : (g.kind == GroupKind::MAP ? g.prog1 : g.prog)) if (in.kind == IKind::LOAD) ++k; return k; }();
    if (g.kind == GroupKind::GEMM) s << " M=" << g.M << " N=" << g.N << " K=" << g.K << " tile=" << (g.BX == 256 ? 256 : 128) << "x" << g.BX << (g.VR == 2 ? " direct" : "");
    if (g.kind == GroupKind::GEMM && g.slabs > 1) s << " split=" << g.slabs;
    if (g.kind == GroupKind::GEMV) s << " mode=" << (g.gemv_mode == 2 ? "row-dot+column-accumulate" : (g.gemv_mode ? "column-accumulate" : "row-dot")) << " M=" << g.M << " K=" << g.K;
    if (g.pair) {
      s << " fused-with=[root=" << g.pair->root->id << " members=[";
      bool f2 = true;
      for (const Node* n : g.pair->members) { if (n->is_view()) continue; s << (f2 ? "" : ",") << n->id << ':' << node_label(n); f2 = false; }
      s << "]]";
    }
    if (g.kind == GroupKind::ROWRED) s << " phases=" << g.phases.size() << " row_threads=" << g.row_threads << " NP=" << g.NP << (g.row_iters > 1 ? " rows_per_group=" + std::to_string(g.row_iters) : std::string());
    if (g.kind == GroupKind::SCAN) s << " mode=" << (g.scan_mode == 3 ? "one-pass-line-tiles" : (g.scan_mode == 2 ? "one-pass-tiles" : (g.scan_mode ? "thread-per-line" : "lanes-along-axis"))) << " lines=" << g.red_out << " length=" << g.red_len << " chunks=" << g.scan_nchunk;
    if (g.kind == GroupKind::MAP) s << " tile=" << g.BY * g.VR << "x" << g.BX * 4 * g.UC << " patch=" << g.VR << "x" << g.UC * 4;
    s << '\n';
  }
  return s.str();
}

}  // namespace gr
