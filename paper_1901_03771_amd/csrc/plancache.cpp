// Plan cache: a request whose sub-DAG looks exactly like one planned before reuses that plan.
//
// Section 2 of the paper evaluates on demand, so an iterative program (a solver sweep, a
// training step) hands the library the same expression again and again, each time over new
// nodes.  Partitioning (Algorithm 1), index-map composition and signature building depend only
// on the structure of the requested sub-DAG, never on the identity of its nodes or on device
// addresses, so their result is remembered under a fingerprint of that structure:
//
//   * the nodes reachable from the root, stopping at nodes that have data, numbered in
//     depth-first order; per node its kind, element type, shape, operation payload (slice
//     bounds, permutation, reduced axes, scalar value) and the numbers of its inputs, so shared
//     sub-expressions and repeated operands are part of the fingerprint;
//   * for nodes with data: strides and offset (they enter access-group bases and coefficients);
//   * the order of the node ids (the planner orders sub-graphs and access groups by id);
//   * the destination of a slice assignment, and a counter bumped by every option change.
//
// A remembered plan holds node pointers (roots, leaves, members, access-group buffers).  Each
// such pointer slot is stored with the number of its node, and a later request with an equal
// fingerprint points the slots at its own nodes and replays the marks the planner leaves on
// the roots of earlier sub-graphs (planned, C-contiguous strides).  Option "plan_cache" = 2
// plans afresh on every hit as well and fails the request if the two plans differ.
#include <algorithm>
#include <sstream>

#include "ctx.h"

namespace gr {

namespace {

constexpr size_t MAX_ENTRIES = 512;
constexpr size_t MAX_NODES = 4096;  // larger requests are planned afresh (the walk itself would dominate)

struct Walk {
  std::vector<Node*> nodes;
  std::vector<int64_t> key;
  uint64_t hash = 0;
};

int64_t bits_of(double v) {
  int64_t b;
  std::memcpy(&b, &v, sizeof b);
  return b;
}

// Numbers the sub-DAG below `root` and writes its fingerprint.  False: too large to be worth it.
bool fingerprint(gr_ctx* c, Node* root, const OutSpec* out, Walk* w) {
  const uint64_t epoch = ++c->walk_epoch;
  std::vector<Node*>& nodes = w->nodes;
  std::vector<Node*> stack{root};
  while (!stack.empty()) {
    Node* n = stack.back();
    stack.pop_back();
    if (n->walk_epoch == epoch) continue;
    n->walk_epoch = epoch;
    n->walk_idx = (int)nodes.size();
    nodes.push_back(n);
    if (nodes.size() > MAX_NODES) return false;
    if (n->has_data()) continue;
    for (size_t i = n->in.size(); i-- > 0;) stack.push_back(n->in[i]);
  }
  std::vector<int64_t>& k = w->key;
  k.reserve(nodes.size() * 12 + 32);
  k.push_back((int64_t)c->options_epoch);
  k.push_back((int64_t)c->plan_static);
  k.push_back((int64_t)nodes.size());
  if (out) {
    k.push_back(1);
    k.push_back(out->base);
    for (int d = 0; d < root->ndim; ++d) k.push_back(out->strides[d]);
  } else k.push_back(0);
  for (Node* n : nodes) {
    k.push_back((int64_t)n->kind | ((int64_t)n->dtype << 8) | ((int64_t)n->ndim << 16) | ((int64_t)n->materialized << 24) |
                ((int64_t)n->planned << 25) | ((int64_t)n->is_int << 26) | ((int64_t)n->keepdims << 27));
    for (int d = 0; d < n->ndim; ++d) k.push_back(n->shape[d]);
    if (n->has_data()) {
      for (int d = 0; d < n->ndim; ++d) k.push_back(n->strides[d]);
      k.push_back(n->offset);
      continue;
    }
    k.push_back(n->op);
    switch (n->kind) {
      case Kind::SCALAR: case Kind::CONST: k.push_back(bits_of(n->value)); break;
      case Kind::SLICE: for (int d = 0; d < n->ndim; ++d) { k.push_back(n->start[d]); k.push_back(n->step[d]); } break;
      case Kind::TRANSPOSE: for (int d = 0; d < n->ndim; ++d) k.push_back(n->perm[d]); break;
      case Kind::REDUCE: case Kind::SCAN: {
        int64_t m = 0;
        for (int d = 0; d < MAXD; ++d) m |= (int64_t)n->red_axis[d] << d;
        k.push_back(m);
        break;
      }
      default: break;
    }
    k.push_back((int64_t)n->in.size());
    for (Node* p : n->in) k.push_back(p->walk_idx);
  }
  // order of the node ids
  std::vector<int> by_id(nodes.size());
  for (size_t i = 0; i < nodes.size(); ++i) by_id[i] = (int)i;
  std::sort(by_id.begin(), by_id.end(), [&](int a, int b) { return nodes[a]->id < nodes[b]->id; });
  for (int i : by_id) k.push_back(i);
  uint64_t h = 1469598103934665603ull;
  for (int64_t v : k) { h ^= (uint64_t)v; h *= 1099511628211ull; h ^= h >> 29; }
  w->hash = h;
  return true;
}

// Visits every node pointer slot of a sub-graph list in a fixed order.  `owned` is a set ordered by
// node id and is handled by the callers (read_owned / the rebinding below).
template <class F>
void for_each_slot(std::vector<std::unique_ptr<GroupPlan>>& groups, F&& f) {
  for (auto& up : groups)
    for (GroupPlan* g : {up.get(), up->pair.get()}) {
      if (!g) continue;
      { const Node* r = g->root; f(r); g->root = const_cast<Node*>(r); }
      for (const Node*& m : g->members) f(m);
      for (const Node*& l : g->leaves) f(l);
      for (AccessGroup& ag : g->groups) f(ag.leaf);
      for (Phase& p : g->phases) f(p.node);
    }
}

std::string dump(const std::vector<std::unique_ptr<GroupPlan>>& groups) {
  std::ostringstream o;
  for (auto& up : groups)
    for (const GroupPlan* g : {(const GroupPlan*)up.get(), (const GroupPlan*)up->pair.get()}) {
      if (!g) continue;
      o << "G kind=" << (int)g->kind << " root=" << g->root->id << " rank=" << g->rank << "/" << g->orig_rank << " sig=" << std::hash<std::string>()(g->signature) << "/" << g->signature.size() << "\n";
      for (int d = 0; d < MAXD; ++d) o << g->dims[d] << "," << g->orig_dims[d] << "," << g->collapse_to[d] << "," << g->out_orig_coef[d] << "," << g->out_coef[d] << ";";
      o << "\n m:";
      for (const Node* m : g->members) o << m->id << ",";
      o << " l:";
      for (const Node* l : g->leaves) o << l->id << ",";
      o << " o:";
      for (const Node* m : g->owned) o << m->id << ",";
      o << "\n";
      for (const AccessGroup& ag : g->groups) {
        o << " ag leaf=" << (ag.leaf ? ag.leaf->id : 0) << " dt=" << (int)ag.dtype << " base=" << ag.base << " coef=";
        for (int d = 0; d < MAXD; ++d) o << ag.coef[d] << (ag.structural_zero[d] ? "z" : "") << ",";
        o << " ident=";
        for (int64_t v : ag.ident) o << v << ",";
        o << " deltas=";
        for (auto& dl : ag.deltas) { for (int64_t v : dl) o << v << ","; o << "|"; }
        o << "\n";
      }
      for (const ConstSlot& cs : g->consts) o << " c" << (int)cs.dtype << ":" << bits_of(cs.value);
      for (const Phase& p : g->phases) o << " ph" << p.op << "," << (int)p.in_dtype << "," << (int)p.out_dtype << "," << p.value << "," << (p.node ? p.node->id : 0);
      o << "\n out_base=" << g->out_base << " unit=" << g->out_unit << " dt=" << (int)g->out_dtype << " per_row=" << g->out_per_row << " sched=" << g->BX << ","
        << g->BY << "," << g->VR << "," << g->UC << "," << g->NP << "," << g->row_threads << "," << g->row_iters << "," << g->xcd_remap << "," << g->cphase << "," << g->stage_mask << "," << g->tail << "," << g->nt << ","
        << g->red_mode << "," << g->red_vec << "," << g->red_out << "," << g->red_len << "," << g->red_kept_rank << "," << g->scan_mode << "," << g->scan_vec << ","
        << g->scan_chunk << "," << g->scan_nchunk << "," << g->gemv_mode << "," << g->M << "," << g->K << "," << g->N << "," << g->mat_group << ","
        << g->vec_group << "," << g->LPR << "," << g->KV << "," << g->slabs << "," << g->unroll << " result1=" << g->result1 << " prog1=" << g->prog1.size() << "\n";  // (prog / results of a map sub-graph are expanded on demand)
    }
  return o.str();
}

void evict_if_full(gr_ctx* c) {
  if (c->plan_cache.size() < MAX_ENTRIES) return;
  // drop the older half (entries on loan stay)
  std::vector<uint64_t> ages;
  for (auto& kv : c->plan_cache) ages.push_back(kv.second->last_use);
  std::nth_element(ages.begin(), ages.begin() + ages.size() / 2, ages.end());
  const uint64_t cut = ages[ages.size() / 2];
  for (auto it = c->plan_cache.begin(); it != c->plan_cache.end();)
    if (!it->second->on_loan && it->second->last_use < cut) it = c->plan_cache.erase(it);
    else ++it;
}

}  // namespace

Plan::~Plan() {
  if (!entry) return;
  // the sub-graph list goes back to the cache; its node pointers are stale from here on and are
  // rewritten before the next use
  entry->groups = std::move(groups);
  entry->on_loan = false;
}

gr_status make_plan(gr_ctx* c, Node* root, Plan* plan) {
  if (!c->opt_plan_cache || root->kind == Kind::SCALAR) return make_plan_uncached(c, root, plan);
  Walk w;
  if (!fingerprint(c, root, plan->out, &w)) return make_plan_uncached(c, root, plan);
  PlanEntry* hit = nullptr;
  auto range = c->plan_cache.equal_range(w.hash);
  for (auto it = range.first; it != range.second; ++it)
    if (it->second->key == w.key) { hit = it->second.get(); break; }
  if (hit && hit->on_loan) return make_plan_uncached(c, root, plan);  // the same request nested in itself
  if (hit) {
    size_t si = 0;
    for_each_slot(hit->groups, [&](const Node*& p) { int i = hit->slots[si++]; p = i >= 0 ? w.nodes[i] : nullptr; });
    // the sets of owned nodes are ordered by id: emptied (no node is looked at) and filled again
    for (auto& up : hit->groups)
      for (GroupPlan* g : {up.get(), up->pair.get()}) {
        if (!g) continue;
        // the numeric identity of an access group starts with the id of the buffer it reads
        for (AccessGroup& ag : g->groups) if (ag.leaf && !ag.ident.empty()) ag.ident[0] = (int64_t)ag.leaf->id;
        g->owned.clear();
        const size_t n = (size_t)hit->slots[si++];
        for (size_t j = 0; j < n; ++j) g->owned.insert(w.nodes[hit->slots[si++]]);
      }
    if (c->opt_plan_cache >= 2) {
      Plan fresh;
      fresh.out = plan->out;
      gr_status st = make_plan_uncached(c, root, &fresh);
      if (st != GR_OK) return st;
      std::string a = dump(hit->groups), b = dump(fresh.groups);
      bool same = a == b && fresh.out_honoured == hit->out_honoured && fresh.planned_nodes.size() == hit->planned.size();
      for (size_t i = 0; same && i < hit->planned.size(); ++i) same = fresh.planned_nodes[i] == w.nodes[hit->planned[i]];
      clear_planned(&fresh);
      if (!same) return fail(c, GR_ERR_UNSUPPORTED, "plan cache: the remembered plan differs from a fresh one\n--- remembered\n" + a + "--- fresh\n" + b);
    }
    for (int i : hit->planned) {
      Node* r = w.nodes[i];
      r->planned = true;
      int64_t s = 1;
      for (int d = r->ndim - 1; d >= 0; --d) { r->strides[d] = s; s *= r->shape[d]; }
      r->offset = 0;
      plan->planned_nodes.push_back(r);
    }
    plan->groups = std::move(hit->groups);
    plan->out_honoured = hit->out_honoured;
    plan->entry = hit;
    hit->on_loan = true;
    hit->last_use = ++c->plan_clock;
    c->stats.plan_hits++;
    return GR_OK;
  }
  gr_status st = make_plan_uncached(c, root, plan);
  if (st != GR_OK) return st;
  // remember it, unless it names a node the walk did not number
  std::unique_ptr<PlanEntry> e(new PlanEntry());
  const uint64_t epoch = c->walk_epoch;
  bool ok = true;
  auto number_of = [&](const Node* p) -> int {
    if (!p) return -1;
    if (p->walk_epoch != epoch) { ok = false; return -1; }
    return p->walk_idx;
  };
  for_each_slot(plan->groups, [&](const Node*& p) { e->slots.push_back(number_of(p)); });
  for (auto& up : plan->groups)
    for (GroupPlan* g : {up.get(), up->pair.get()}) {
      if (!g) continue;
      e->slots.push_back((int)g->owned.size());
      for (const Node* m : g->owned) { int i = number_of(m); if (i < 0) ok = false; e->slots.push_back(i); }
    }
  for (Node* r : plan->planned_nodes) { int i = number_of(r); if (i < 0) ok = false; e->planned.push_back(i); }
  if (!ok) return GR_OK;
  evict_if_full(c);
  e->key = std::move(w.key);
  e->out_honoured = plan->out_honoured;
  e->on_loan = true;
  e->last_use = ++c->plan_clock;
  plan->entry = e.get();
  c->plan_cache.emplace(w.hash, std::move(e));
  return GR_OK;
}

}  // namespace gr
