// Internal data structures of the lazy-array library: DAG nodes (Section 2 of
// the paper: attributes operation / data / is_materialized), the context, and
// the plan handed from the partitioner to the code generator and the runtime.
#pragma once

#include <cstdint>
#include <cstring>
#include <map>
#include <memory>
#include <set>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/grumpy_hip_tuning.h"

namespace gr {

constexpr int MAXD = GR_MAX_NDIM;

enum class Kind : uint8_t { LEAF, SCALAR, CONST, UNARY, BINARY, SLICE, TRANSPOSE, REDUCE, DOT, SCAN, RESHAPE };

struct Node {
  uint64_t id = 0;
  Kind kind = Kind::LEAF;
  int op = 0;  // gr_op for UNARY / BINARY / REDUCE
  gr_dtype dtype = GR_F32;
  int ndim = 0;
  int64_t shape[MAXD] = {0};
  std::vector<Node*> in;  // predecessors (each holds one consumer reference)
  int handle_refs = 0;
  int consumer_refs = 0;
  uint64_t shash = 0;  // hash of the expression below this node (materialised nodes: of their identity)
  uint64_t walk_epoch = 0;  // numbering of the request being fingerprinted (plan cache)
  int walk_idx = -1;

  // "data" / "is_materialized"
  bool materialized = false;
  bool planned = false;  // will be materialised by an earlier sub-graph of the plan being built
  void* data = nullptr;  // device pointer to element offset 0 of the allocation
  int64_t strides[MAXD] = {0};
  int64_t offset = 0;      // elements from `data` to element (0,..,0)
  bool owns_data = false;  // allocated through the context's allocator
  bool cow_alias = false;  // data lives in another array's storage (result of a direct slice assignment):
                           // gets its own copy before that storage is written again
  size_t alloc_bytes = 0;
  // Second buffer of an array that stencil sweeps are assigned into (see gr_assign): same size as
  // `data`; outside the box [shadow_start, shadow_start + shadow_len) it holds the same cells.
  void* shadow = nullptr;
  // A second buffer lent by the caller to a wrapped array (gr_array_lend_buffer): the one of the caller's two
  // buffers that is not `data` right now.  It takes the place of a library-allocated second buffer in the
  // sweeps above and is never freed by the library.
  void* lent = nullptr;
  int64_t shadow_start[MAXD] = {0};
  int64_t shadow_len[MAXD] = {0};

  // SCALAR / CONST payload
  double value = 0.0;
  bool is_int = false;

  // SLICE: per-dimension start and step (normalised); TRANSPOSE: perm
  int64_t start[MAXD] = {0};
  int64_t step[MAXD] = {0};
  int perm[MAXD] = {0};

  // REDUCE
  bool red_axis[MAXD] = {false};
  bool keepdims = false;

  int64_t count() const {
    int64_t n = 1;
    for (int d = 0; d < ndim; ++d) n *= shape[d];
    return n;
  }
  bool is_view() const { return kind == Kind::SLICE || kind == Kind::TRANSPOSE; }
  bool is_compute() const { return kind == Kind::UNARY || kind == Kind::BINARY || kind == Kind::REDUCE || kind == Kind::DOT || kind == Kind::SCAN || kind == Kind::RESHAPE; }
  bool has_data() const { return materialized || planned; }
};

// Node containers are ordered by node id (recording order), never by address: plans must not
// depend on where the allocator happened to put a node.
struct NodeIdLess {
  bool operator()(const Node* a, const Node* b) const { return a->id < b->id; }
};
using NodeSet = std::set<const Node*, NodeIdLess>;

inline size_t itemsize(gr_dtype dt) { return dt == GR_I64 ? 8 : 4; }

// ---- plan --------------------------------------------------------------------

// Index of one operand dimension as an affine function of one iteration-space
// dimension: scale * i[src] + off  (src < 0: the constant `off`).  This is the
// index translation of Section 3.1 kept in closed form: broadcast, slicing and
// transposition all stay inside this class of maps.
struct DimMap {
  int src = -1;
  int64_t scale = 0;
  int64_t off = 0;
};
using IndexMap = std::vector<DimMap>;

enum class IKind : uint8_t { LOAD, CONST, UNARY, BINARY, RED, ACC };

// One SSA instruction of a fused point program.
struct Instr {
  IKind kind = IKind::CONST;
  int op = 0;
  gr_dtype dtype = GR_F32;
  int a = -1, b = -1;         // operand instruction ids
  int group = -1;             // LOAD: access group
  int64_t delta[MAXD] = {0};  // LOAD: shift in iteration space (original dims; later collapsed dims)
  int cslot = -1;             // CONST: slot in the constant table
  int phase = -1;             // RED: index of the reduction phase whose result this is
  bool uniform = false;       // value does not depend on the innermost iteration dimension
};

// A set of loads from one buffer that differ only by a shift in iteration space.
struct AccessGroup {
  const Node* leaf = nullptr;
  gr_dtype dtype = GR_F32;
  std::vector<int64_t> ident;  // numeric identity (see plan.cpp)
  int64_t base = 0;            // elements from leaf->data to the element read at i = 0, delta = 0
  int64_t coef[MAXD] = {0};    // elements per unit step of each iteration dimension
  bool structural_zero[MAXD] = {false};  // no leaf dimension follows this iteration dimension
  std::set<std::vector<int64_t>> deltas;  // all shifts used (length = iteration rank)
};

enum class GroupKind : uint8_t { MAP, ROWRED, REDUCE, GEMV, SCAN, GEMM };

struct Phase {
  int op = 0;  // GR_SUM / GR_MAX / GR_MIN
  gr_dtype in_dtype = GR_F32;
  gr_dtype out_dtype = GR_F32;
  int value = -1;  // instruction whose values are combined
  const Node* node = nullptr;
};

struct ConstSlot {
  gr_dtype dtype;
  double value;
};

// k extent of one split of a matrix product whose K range is divided over nsplit workgroups per output tile:
// a multiple of 32 (the longer of the two k steps of the kernels) that covers K in nsplit pieces; the last
// piece is what remains and may be short or empty.
inline int64_t gemm_split_extent(int64_t K, int64_t nsplit) {
  return nsplit > 1 ? (((K + nsplit - 1) / nsplit + 31) / 32) * 32 : K;
}

// One sub-graph of the ordered list of Algorithm 1, ready for code generation.
struct GroupPlan {
  GroupKind kind = GroupKind::MAP;
  Node* root = nullptr;
  std::vector<const Node*> members;  // lazy nodes computed inside this sub-graph
  std::vector<const Node*> leaves;   // materialised nodes it reads
  std::string note;                  // human-readable details for gr_plan_describe

  // iteration space (after collapsing)
  int rank = 0;
  int64_t dims[MAXD] = {0};
  int orig_rank = 0;
  int64_t orig_dims[MAXD] = {0};
  int collapse_to[MAXD] = {0};  // original dim -> collapsed dim (innermost original of a merged run carries shifts)

  std::vector<Instr> prog;
  std::vector<int> results;  // MAP: one per patch point; ROWRED/REDUCE/GEMV: single entry (final value) or empty
  std::vector<AccessGroup> groups;
  std::vector<ConstSlot> consts;
  std::vector<Phase> phases;

  // MAP: single-point program (boundary tiles, cache key); `prog` holds the per-lane patch
  // program and is only built when a kernel has to be generated
  NodeSet owned;
  std::vector<Instr> prog1;
  int result1 = -1;

  // output
  int64_t out_base = 0;                 // MAP: element offset of output element (0,..,0)
  int64_t out_orig_coef[MAXD] = {0};    // MAP: output strides per original iteration dimension
  bool out_unit = true;                 // MAP: innermost output stride is 1 (vector stores)
  gr_dtype out_dtype = GR_F32;
  bool out_per_row = false;  // ROWRED: one value per row instead of one per element

  // schedule
  int BX = 64, BY = 4, VR = 1, UC = 1;  // MAP
  int NP = 1;                            // ROWRED: vec4 positions per lane
  int row_threads = 64;                  // ROWRED: lanes cooperating on one row (64 or 256)
  int row_iters = 1;                     // ROWRED: rows a lane group takes in one launch (short rows, one value per row)
  bool xcd_remap = false;
  int cphase = 0;     // map: lanes own columns 4k - cphase .. 4k - cphase + 3, so that their vector stores are 16-byte aligned in the output
  int stage_mask = 0;                    // MAP: access groups (bit per group) read through a transposing LDS tile
  int diag = 0;                          // MAP with staged operands: tile rows are taken diagonally (row block + column block)
  int tail = 0;                          // MAP: columns mod 4 of a narrow array (1..3): its last lanes get straight-line code too
  int nt = 0;                            // non-temporal load hint: 0 none, 1 arrays read once, 2 all vector loads
  int red_mode = 0;                      // REDUCE: 0 thread-per-output, 1 block-per-output
  int red_vec = 0;                       // REDUCE mode 0: a thread owns four consecutive outputs (dwordx4 loads)
  int64_t red_out = 0, red_len = 0;      // REDUCE: outputs, reduced elements per output
  int red_kept_rank = 0;

  // SCAN: element stride of the output per iteration dimension (the scanned axis is the last
  // iteration dimension but need not be the output's last), mode 0 = lanes along the scanned
  // axis (it is contiguous), 1 = a thread per line; chunking of long lines
  int64_t out_coef[MAXD] = {0};
  int scan_mode = 0;
  int scan_vec = 0;   // mode 1: a thread walks four neighbouring lines (dwordx4 per step)
  int64_t scan_chunk = 0;
  int scan_nchunk = 1;

  // GEMV core
  int gemv_mode = 0;  // 0: inner stride 1 along k (row-dot); 1: inner stride 1 along m (column-accumulate);
                      // 2: row-dot fused with the column-accumulate sub-graph in `pair` (one pass over the matrix)
  std::unique_ptr<GroupPlan> pair;
  int64_t M = 0, K = 0, N = 0;  // N: GEMM only
  int mat_group = -1, vec_group = -1;  // GEMM: left (m,k) and right (k,n) operand
  int LPR = 64;       // gemv row-dot: lanes per row
  int KV = 1;         // gemv row-dot: vec4 per lane along k
  int slabs = 1;      // gemv column-accumulate: row slabs (first-stage partial vectors)
  int unroll = 8;     // gemv column-accumulate: rows in flight per lane

  std::string signature;
};

// Strided destination of the requested root (slice assignment); NULL = C-contiguous buffer.
struct OutSpec {
  int64_t base = 0;
  int64_t strides[MAXD] = {0};
};

struct PlanEntry;

struct Plan {
  std::vector<std::unique_ptr<GroupPlan>> groups;
  std::vector<Node*> planned_nodes;
  const OutSpec* out = nullptr;  // in: where the root's elements go
  bool out_honoured = true;      // out: false if the root's sub-graph can only write a contiguous buffer
  PlanEntry* entry = nullptr;    // plan cache entry the sub-graphs are on loan from (handed back on destruction)
  Plan() = default;
  Plan(const Plan&) = delete;
  Plan& operator=(const Plan&) = delete;
  ~Plan();
};

// One remembered request (see plancache.cpp): the fingerprint of the sub-DAG it was planned for,
// the sub-graph list, and for every node pointer inside that list the position of the node in
// the fingerprint's numbering, so that the list can be pointed at the nodes of a later request
// with the same fingerprint.
struct PlanEntry {
  std::vector<int64_t> key;
  std::vector<std::unique_ptr<GroupPlan>> groups;
  bool out_honoured = true;
  std::vector<int> slots;    // numbering position per pointer slot, in the order of the slot walk
  std::vector<int> planned;  // roots marked as planned, in order
  bool on_loan = false;
  uint64_t last_use = 0;
};

}  // namespace gr
