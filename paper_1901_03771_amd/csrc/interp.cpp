// Host side of the point-program interpreter: encodes the single-point program
// of a map sub-graph, or the phases and the final map of a row-resident
// reduction sub-graph, as byte code with LDS slots assigned by a linear scan
// over the values' live ranges, and launches the precompiled kernels.
#include <algorithm>

#include "ctx.h"
#include "interp.h"

extern "C" int gr_launch_interp_map(void* stream, const GrInterpArgs* args, unsigned grid);
extern "C" int gr_launch_interp_rowred(void* stream, const GrInterpRowArgs* args, unsigned grid);
extern "C" int gr_launch_interp_gen(void* stream, const GrInterpGenArgs* args, unsigned grid);

namespace gr {

static int opcode(const Instr& in) {
  const bool f = in.dtype == GR_F32;
  if (in.kind == IKind::UNARY) switch (in.op) {
    case GR_NEG: return f ? GI_FNEG : GI_INEG;
    case GR_ABS: return f ? GI_FABS : GI_IABS;
    case GR_SQUARE: return f ? GI_FSQUARE : GI_ISQUARE;
    case GR_EXP: return f ? GI_FEXP : -1;
    case GR_LOG: return f ? GI_FLOG : -1;
    case GR_SQRT: return f ? GI_FSQRT : -1;
    case GR_TANH: return f ? GI_FTANH : -1;
    case GR_ERF: return f ? GI_FERF : -1;
  }
  if (in.kind == IKind::BINARY) switch (in.op) {
    case GR_ADD: return f ? GI_FADD : GI_IADD;
    case GR_SUB: return f ? GI_FSUB : GI_ISUB;
    case GR_MUL: return f ? GI_FMUL : GI_IMUL;
    case GR_DIV: return f ? GI_FDIV : -1;
    case GR_MAXIMUM: return f ? GI_FMAX : GI_IMAX;
    case GR_MINIMUM: return f ? GI_FMIN : GI_IMIN;
  }
  return -1;
}

// Fills `A` and `grid` for sub-graph `g` writing to `out_ptr`; false if the sub-graph is outside
// what the interpreter covers (then the caller waits for the compiler as usual).
bool interp_encode(const GroupPlan& g, void* out_ptr, GrInterpArgs* A, unsigned* grid) {
  if (g.kind != GroupKind::MAP || g.rank < 1 || g.rank > GR_INTERP_RANK || g.out_dtype == GR_I64 || g.result1 < 0) return false;
  if (g.groups.size() > GR_INTERP_GROUPS || g.consts.size() > GR_INTERP_CONSTS) return false;
  const std::vector<Instr>& p = g.prog1;
  const int n = (int)p.size();
  // instructions the result depends on, and the last reader of each value
  std::vector<int> last(n, -1);
  std::vector<char> need(n, 0);
  need[g.result1] = 1;
  for (int i = n - 1; i >= 0; --i) {
    if (!need[i]) continue;
    for (int o : {p[i].a, p[i].b}) {
      if (o < 0) continue;
      if (o >= i) return false;  // not in evaluation order
      need[o] = 1;
      last[o] = std::max(last[o], i);
    }
  }
  last[g.result1] = n;
  const int pad = GR_INTERP_RANK - g.rank;
  std::memset(A, 0, sizeof *A);
  int64_t total = 1;
  for (int k = 0; k < GR_INTERP_RANK; ++k) A->dims[k] = 1;
  for (int k = 0; k < g.rank; ++k) { A->dims[k + pad] = g.dims[k]; total *= g.dims[k]; }
  if (total <= 0) return false;
  int64_t blocks = (g.dims[g.rank - 1] + 255) / 256;
  for (int k = 0; k + 1 < g.rank; ++k) {
    blocks *= g.dims[k];
    if (blocks > 0x7fffffffLL) return false;
  }
  *grid = (unsigned)blocks;
  for (size_t gi = 0; gi < g.groups.size(); ++gi) {
    const AccessGroup& ag = g.groups[gi];
    if (ag.dtype == GR_I64 || !ag.leaf || !ag.leaf->data) return false;
    A->gptr[gi] = (unsigned long long)(uintptr_t)ag.leaf->data + 4ull * (unsigned long long)ag.base;
    for (int k = 0; k < g.rank; ++k) A->gcoef[gi][k + pad] = ag.structural_zero[k] ? 0 : ag.coef[k];
  }
  A->out = (unsigned long long)(uintptr_t)out_ptr + 4ull * (unsigned long long)g.out_base;
  for (int k = 0; k < g.rank; ++k) A->ocoef[k + pad] = g.out_coef[k];
  if (g.out_unit) A->ocoef[GR_INTERP_RANK - 1] = 1;
  for (size_t i = 0; i < g.consts.size(); ++i) {
    const ConstSlot& cs = g.consts[i];
    if (cs.dtype == GR_F32) { float f = (float)cs.value; std::memcpy(&A->consts[i], &f, 4); }
    else if (cs.dtype == GR_I32) A->consts[i] = (unsigned)(int32_t)(int64_t)cs.value;
    else return false;
  }
  // linear scan: a value's slot is free again after its last reader
  std::vector<int> slot(n, -1), free_slots;
  for (int s = GR_INTERP_SLOTS - 1; s >= 0; --s) free_slots.push_back(s);
  int ni = 0, nl = 0;
  for (int i = 0; i < n; ++i) {
    if (!need[i]) continue;
    const Instr& in = p[i];
    if (in.dtype == GR_I64 || ni >= GR_INTERP_INSTR) return false;
    unsigned op, xa = 0, xb = 0;
    if (in.kind == IKind::LOAD) {
      if (nl >= GR_INTERP_LOADS || in.group < 0 || in.group >= (int)g.groups.size()) return false;
      const AccessGroup& ag = g.groups[in.group];
      int64_t off = 0;
      for (int k = 0; k < g.rank; ++k) if (!ag.structural_zero[k]) off += in.delta[k] * ag.coef[k];
      A->ldoff[nl] = off;
      op = GI_LOAD; xa = (unsigned)in.group; xb = (unsigned)nl++;
    } else if (in.kind == IKind::CONST) {
      if (in.cslot < 0 || in.cslot >= (int)g.consts.size()) return false;
      op = GI_CONST; xa = (unsigned)in.cslot;
    } else {
      int oc = opcode(in);
      if (oc < 0 || in.a < 0 || slot[in.a] < 0) return false;
      op = (unsigned)oc;
      xa = (unsigned)slot[in.a];
      xb = xa;
      if (in.kind == IKind::BINARY) {
        if (in.b < 0 || slot[in.b] < 0) return false;
        xb = (unsigned)slot[in.b];
      }
      // operands are read before the result is written: a dying operand's slot can be reused at once
      for (int o : {in.a, in.kind == IKind::BINARY ? in.b : -1})
        if (o >= 0 && last[o] == i && slot[o] >= 0) { free_slots.push_back(slot[o]); slot[o] = -2 - slot[o]; }
    }
    if (free_slots.empty()) return false;
    int dst = free_slots.back();
    free_slots.pop_back();
    slot[i] = dst;
    A->code[ni++] = op | ((unsigned)dst << 8) | (xa << 16) | (xb << 24);
  }
  A->n_instr = ni;
  A->result_slot = slot[g.result1];
  return A->result_slot >= 0;
}

// Operand patterns, constants and extents of a sub-graph: what map and row-resident sub-graphs share.
static bool encode_operands(const GroupPlan& g, GrInterpArgs* A, const Node* fresh = nullptr, void* fresh_ptr = nullptr) {
  if (g.rank < 1 || g.rank > GR_INTERP_RANK || g.groups.size() > GR_INTERP_GROUPS || g.consts.size() > GR_INTERP_CONSTS) return false;
  const int pad = GR_INTERP_RANK - g.rank;
  for (int k = 0; k < GR_INTERP_RANK; ++k) A->dims[k] = 1;
  for (int k = 0; k < g.rank; ++k) A->dims[k + pad] = g.dims[k];
  for (size_t gi = 0; gi < g.groups.size(); ++gi) {
    const AccessGroup& ag = g.groups[gi];
    void* const data = ag.leaf == fresh && fresh ? fresh_ptr : (ag.leaf ? ag.leaf->data : nullptr);
    if (ag.dtype == GR_I64 || !data) return false;
    A->gptr[gi] = (unsigned long long)(uintptr_t)data + 4ull * (unsigned long long)ag.base;
    for (int k = 0; k < g.rank; ++k) A->gcoef[gi][k + pad] = ag.structural_zero[k] ? 0 : ag.coef[k];
  }
  for (size_t i = 0; i < g.consts.size(); ++i) {
    const ConstSlot& cs = g.consts[i];
    if (cs.dtype == GR_F32) { float f = (float)cs.value; std::memcpy(&A->consts[i], &f, 4); }
    else if (cs.dtype == GR_I32) A->consts[i] = (unsigned)(int32_t)(int64_t)cs.value;
    else return false;
  }
  return true;
}

// Appends to A->code the instructions of `p` that `want` depends on (slots by a linear scan of the
// live ranges); returns the slot of `want`, -1 if the program is outside what the interpreter covers.
static int encode_segment(const GroupPlan& g, const std::vector<Instr>& p, int want, GrInterpArgs* A, int* ni, int* nl) {
  const int n = (int)p.size();
  if (want < 0 || want >= n) return -1;
  std::vector<int> last(n, -1);
  std::vector<char> need(n, 0);
  need[want] = 1;
  for (int i = n - 1; i >= 0; --i) {
    if (!need[i]) continue;
    for (int o : {p[i].a, p[i].b}) {
      if (o < 0) continue;
      if (o >= i) return -1;
      need[o] = 1;
      last[o] = std::max(last[o], i);
    }
  }
  last[want] = n;
  std::vector<int> slot(n, -1), free_slots;
  for (int s = GR_INTERP_SLOTS - 1; s >= 0; --s) free_slots.push_back(s);
  for (int i = 0; i < n; ++i) {
    if (!need[i]) continue;
    const Instr& in = p[i];
    if (in.dtype == GR_I64 || *ni >= GR_INTERP_INSTR) return -1;
    unsigned op, xa = 0, xb = 0;
    if (in.kind == IKind::LOAD) {
      if (*nl >= GR_INTERP_LOADS || in.group < 0 || in.group >= (int)g.groups.size()) return -1;
      const AccessGroup& ag = g.groups[in.group];
      int64_t off = 0;
      for (int k = 0; k < g.rank; ++k) if (!ag.structural_zero[k]) off += in.delta[k] * ag.coef[k];
      A->ldoff[*nl] = off;
      op = GI_LOAD; xa = (unsigned)in.group; xb = (unsigned)(*nl)++;
    } else if (in.kind == IKind::CONST) {
      if (in.cslot < 0 || in.cslot >= (int)g.consts.size()) return -1;
      op = GI_CONST; xa = (unsigned)in.cslot;
    } else if (in.kind == IKind::RED) {
      if (in.phase < 0 || in.phase >= GR_INTERP_PHASES) return -1;
      op = GI_RED; xa = (unsigned)in.phase;
    } else if (in.kind == IKind::ACC) {
      op = GI_RED; xa = 0;   // the accumulated sum of a contraction reaches its epilogue as phase value 0
    } else if (in.kind == IKind::UNARY || in.kind == IKind::BINARY) {
      int oc = opcode(in);
      if (oc < 0 || in.a < 0 || slot[in.a] < 0) return -1;
      op = (unsigned)oc;
      xa = (unsigned)slot[in.a];
      xb = xa;
      if (in.kind == IKind::BINARY) {
        if (in.b < 0 || slot[in.b] < 0) return -1;
        xb = (unsigned)slot[in.b];
      }
      for (int o : {in.a, in.kind == IKind::BINARY ? in.b : -1})
        if (o >= 0 && last[o] == i && slot[o] >= 0) { free_slots.push_back(slot[o]); slot[o] = -2 - slot[o]; }
    } else return -1;
    if (free_slots.empty()) return -1;
    int dst = free_slots.back();
    free_slots.pop_back();
    slot[i] = dst;
    A->code[(*ni)++] = op | ((unsigned)dst << 8) | (xa << 16) | (xb << 24);
  }
  return slot[want];
}

// A row-resident reduction sub-graph (reduction phases over the innermost dimension, then a final
// map or one value per row) as interpreter segments.  Only rows in number and length that keep the
// interpreter's run well below a compilation are taken.
bool interp_encode_rowred(const GroupPlan& g, void* out_ptr, GrInterpRowArgs* R, unsigned* grid) {
  if (g.kind != GroupKind::ROWRED || g.pair || g.out_dtype == GR_I64 || g.results.empty()) return false;
  if (g.phases.empty() || g.phases.size() > GR_INTERP_PHASES) return false;
  std::memset(R, 0, sizeof *R);
  if (!encode_operands(g, &R->m)) return false;
  const int64_t C = g.dims[g.rank - 1];
  int64_t rows = 1;
  for (int k = 0; k + 1 < g.rank; ++k) rows *= g.dims[k];
  if (C < 1 || rows < 1 || rows > (int64_t)1 << 22 || rows * C > (int64_t)1 << 28) return false;
  // the generated kernel's assignment of elements to lanes, so that both combine in the same order
  R->lanes = g.row_threads;
  R->positions = g.NP;
  if (!(R->lanes == 1 || R->lanes == 2 || R->lanes == 4 || R->lanes == 8 || R->lanes == 16 || R->lanes == 64 || R->lanes == 128 || R->lanes == 256)) return false;
  if ((int64_t)R->lanes * 4 * R->positions < C) return false;
  R->per_row = g.out_per_row ? 1 : 0;
  R->n_phase = (int)g.phases.size();
  int ni = 0, nl = 0;
  for (int s = 0; s <= R->n_phase; ++s) {
    const bool final = s == R->n_phase;
    if (!final) {
      const Phase& ph = g.phases[s];
      if (ph.in_dtype == GR_I64 || ph.out_dtype == GR_I64) return false;
      R->phase_op[s] = ph.op == GR_SUM ? 0 : (ph.op == GR_MAX ? 1 : 2);
      R->phase_int[s] = ph.in_dtype == GR_I32;
    }
    R->seg_begin[s] = ni;
    R->seg_slot[s] = encode_segment(g, g.prog, final ? g.results[0] : g.phases[s].value, &R->m, &ni, &nl);
    R->seg_end[s] = ni;
    if (R->seg_slot[s] < 0) return false;
  }
  R->m.n_instr = ni;
  R->m.out = (unsigned long long)(uintptr_t)out_ptr;
  const int rb = 256 / R->lanes;
  *grid = (unsigned)((rows + rb - 1) / rb);
  return true;
}

// A reduction over any axes, a scan or a contraction with its epilogue (sub-graphs that are cuts
// of their own) for the plain interpreter kernels.  Only sizes that keep the interpreter's run well
// below a compilation are taken.
// (`half_of_pair`: `g` is one of the two contractions that the generated code runs as one kernel; the
// interpreter takes them one after the other, and `fresh` / `fresh_ptr` name the first one's result,
// which the second reads before the node has been given its buffer)
bool interp_encode_gen(const GroupPlan& g, void* out_ptr, GrInterpGenArgs* G, unsigned* grid, bool half_of_pair, const Node* fresh, void* fresh_ptr) {
  if ((g.pair && !half_of_pair) || g.prog.empty()) return false;
  std::memset(G, 0, sizeof *G);
  const int pad = GR_INTERP_RANK - g.rank;
  int ni = 0, nl = 0;
  if (g.kind == GroupKind::REDUCE || g.kind == GroupKind::SCAN) {
    if (g.phases.size() != 1) return false;
    const Phase& ph = g.phases[0];
    if (ph.in_dtype == GR_I64 || (ph.out_dtype == GR_I64 && !(ph.in_dtype == GR_I32 && ph.op == GR_SUM))) return false;
    if (!encode_operands(g, &G->m)) return false;
    G->op = ph.op == GR_SUM ? 0 : (ph.op == GR_MAX ? 1 : 2);
    G->is_int = ph.in_dtype == GR_I32;
    G->out_i64 = ph.out_dtype == GR_I64;
    G->slot = encode_segment(g, g.prog, ph.value, &G->m, &ni, &nl);
    if (G->slot < 0) return false;
    G->m.n_instr = ni;
    G->m.out = (unsigned long long)(uintptr_t)out_ptr;
    int64_t total = 1;
    for (int k = 0; k < g.rank; ++k) total *= g.dims[k];
    if (total < 1 || total > (int64_t)1 << 28) return false;
    if (g.kind == GroupKind::REDUCE) {
      G->kind = GI_KIND_REDUCE;
      G->first_reduced = pad + g.red_kept_rank;
      G->nout = 1;
      for (int k = 0; k < g.red_kept_rank; ++k) G->nout *= g.dims[k];
      G->red_len = total / G->nout;
      if (G->nout != g.red_out || G->nout > 0x7fffffffLL) return false;
      // a workgroup per output: many outputs over a short strided range would crawl
      if (G->nout > (int64_t)1 << 22) return false;
      // few outputs over a long range: the range is cut into slices so that about 1024 workgroups run
      // (the caller provides 8 bytes per slice and launches the combining kernel afterwards)
      G->nsplit = 1;
      if (G->nout < 512 && G->red_len >= 65536) G->nsplit = std::min<int64_t>(std::max<int64_t>(1, 1024 / G->nout), G->red_len / 16384);
      if (G->nsplit < 1) G->nsplit = 1;
      *grid = (unsigned)(G->nout * G->nsplit);
      return true;
    }
    G->nsplit = 1;
    G->kind = GI_KIND_SCAN;
    const int64_t L = g.dims[g.rank - 1];
    G->red_len = L;
    G->nout = total / std::max<int64_t>(L, 1);
    if (L > (int64_t)1 << 21 || G->nout > 0x7fffffffLL) return false;   // a line is walked by one workgroup, 256 elements per step
    for (int k = 0; k < g.rank; ++k) G->m.ocoef[k + pad] = g.out_coef[k];
    *grid = (unsigned)G->nout;
    return true;
  }
  if (g.kind != GroupKind::GEMV && g.kind != GroupKind::GEMM) return false;
  if (g.out_dtype != GR_F32 || g.results.empty() || g.mat_group < 0 || g.vec_group < 0) return false;
  const AccessGroup& mg = g.groups[g.mat_group];
  const AccessGroup& vg = g.groups[g.vec_group];
  auto data_of = [&](const Node* leaf) -> void* { return leaf == fresh ? fresh_ptr : (leaf ? leaf->data : nullptr); };
  if (mg.dtype != GR_F32 || vg.dtype != GR_F32 || !data_of(mg.leaf) || !data_of(vg.leaf)) return false;
  if (!encode_operands(g, &G->m, fresh, fresh_ptr)) return false;
  G->slot = encode_segment(g, g.prog, g.results[0], &G->m, &ni, &nl);
  if (G->slot < 0) return false;
  G->m.n_instr = ni;
  G->m.out = (unsigned long long)(uintptr_t)out_ptr;
  G->mat = (unsigned long long)(uintptr_t)data_of(mg.leaf) + 4ull * (unsigned long long)mg.base;
  G->vec = (unsigned long long)(uintptr_t)data_of(vg.leaf) + 4ull * (unsigned long long)vg.base;
  G->am = mg.coef[0]; G->ak = mg.coef[1];
  G->M = g.M; G->K = g.K;
  if (g.kind == GroupKind::GEMV) {
    if ((g.gemv_mode == 2 && !half_of_pair) || g.M < 1 || g.M > 0x7fffffffLL || g.M * std::max<int64_t>(g.K, 1) > (int64_t)1 << 28) return false;
    G->kind = GI_KIND_GEMV;
    G->N = 1;
    G->bk = vg.coef[1]; G->bn = 0;
    *grid = (unsigned)g.M;
    return true;
  }
  if (g.M < 1 || g.N < 1 || g.M * g.N > (int64_t)1 << 30 || g.M * g.N * std::max<int64_t>(g.K, 1) > (int64_t)1 << 36) return false;
  G->kind = GI_KIND_GEMM;
  G->N = g.N;
  G->bk = vg.coef[0]; G->bn = vg.coef[1];
  *grid = (unsigned)((g.M * g.N + 255) / 256);
  return true;
}

gr_status interp_launch_gen(gr_ctx* c, const GrInterpGenArgs& G, unsigned grid) {
  if (c->device < 0) { c->stats.kernel_launches++; c->stats.interp_launches++; return GR_OK; }  // dry run
  static const char* const names[] = {"gr_interp_reduce", "gr_interp_scan", "gr_interp_gemv", "gr_interp_gemm", "gr_interp_combine"};
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (c->opt_profile) {
    for (hipEvent_t* ev : {&e0, &e1}) {
      if (!c->event_pool.empty()) { *ev = c->event_pool.back(); c->event_pool.pop_back(); }
      else if (hipEventCreate(ev) != hipSuccess) return fail(c, GR_ERR_HIP, "hipEventCreate failed");
    }
    (void)hipEventRecord(e0, c->stream);
  }
  int e = gr_launch_interp_gen(c->stream, &G, grid);
  if (e != 0) return fail(c, GR_ERR_HIP, std::string("interpreter launch -> ") + hipGetErrorName((hipError_t)e));
  if (c->opt_profile) {
    (void)hipEventRecord(e1, c->stream);
    c->prof.push_back({names[G.kind], e0, e1});
  }
  c->stats.kernel_launches++;
  c->stats.interp_launches++;
  return GR_OK;
}

gr_status interp_launch_rowred(gr_ctx* c, const GrInterpRowArgs& R, unsigned grid) {
  if (c->device < 0) { c->stats.kernel_launches++; c->stats.interp_launches++; return GR_OK; }  // dry run
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (c->opt_profile) {
    for (hipEvent_t* ev : {&e0, &e1}) {
      if (!c->event_pool.empty()) { *ev = c->event_pool.back(); c->event_pool.pop_back(); }
      else if (hipEventCreate(ev) != hipSuccess) return fail(c, GR_ERR_HIP, "hipEventCreate failed");
    }
    (void)hipEventRecord(e0, c->stream);
  }
  int e = gr_launch_interp_rowred(c->stream, &R, grid);
  if (e != 0) return fail(c, GR_ERR_HIP, std::string("interpreter launch -> ") + hipGetErrorName((hipError_t)e));
  if (c->opt_profile) {
    (void)hipEventRecord(e1, c->stream);
    c->prof.push_back({"gr_interp_rowred", e0, e1});
  }
  c->stats.kernel_launches++;
  c->stats.interp_launches++;
  return GR_OK;
}

gr_status interp_launch(gr_ctx* c, const GrInterpArgs& A, unsigned grid) {
  if (c->device < 0) { c->stats.kernel_launches++; c->stats.interp_launches++; return GR_OK; }  // dry run
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (c->opt_profile) {
    for (hipEvent_t* ev : {&e0, &e1}) {
      if (!c->event_pool.empty()) { *ev = c->event_pool.back(); c->event_pool.pop_back(); }
      else if (hipEventCreate(ev) != hipSuccess) return fail(c, GR_ERR_HIP, "hipEventCreate failed");
    }
    (void)hipEventRecord(e0, c->stream);
  }
  int e = gr_launch_interp_map(c->stream, &A, grid);
  if (e != 0) return fail(c, GR_ERR_HIP, std::string("interpreter launch -> ") + hipGetErrorName((hipError_t)e));
  if (c->opt_profile) {
    (void)hipEventRecord(e1, c->stream);
    c->prof.push_back({"gr_interp_map", e0, e1});
  }
  c->stats.kernel_launches++;
  c->stats.interp_launches++;
  return GR_OK;
}

}  // namespace gr
