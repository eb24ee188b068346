// The context: node table, options, allocator, kernel cache, statistics.
#pragma once

#include <hip/hip_runtime_api.h>

#include <chrono>
#include <future>
#include <string>
#include <unordered_map>
#include <vector>

#include "ir.h"

// A request recorded once for replay (gr_program_*): the kernel launches of its sub-graph list with
// their argument blocks, and where in those blocks the addresses of the rebindable leaves and of
// the output go.
struct gr_program {
  gr_ctx* ctx = nullptr;
  struct Launch {
    hipFunction_t fn = nullptr;
    std::string name;
    unsigned grid = 0;
    std::vector<uint64_t> args;
    std::vector<std::pair<int, int>> patch;  // (argument slot, source): source k >= 0 = leaf k, -1 = the output
  };
  std::vector<Launch> launches;
  std::vector<std::pair<void*, size_t>> buffers;  // stored results of earlier sub-graphs and workspaces: owned
  std::vector<const gr::Node*> leaf_nodes;        // (only while recording)
  std::vector<size_t> leaf_bytes;                 // extent of each rebindable leaf from its address, for the overlap check
  size_t out_bytes = 0;
  std::vector<std::pair<int, int>> cur_patch;     // provenance of the argument block being filled (while recording)
};

struct gr_ctx {
  int device = -1;
  hipStream_t stream = nullptr;
  std::string err;

  // nodes
  std::unordered_map<uint64_t, gr::Node*> nodes;
  uint64_t next_id = 1;
  bool any_storage_alias = false;  // some node's data has lived inside another node's buffer (direct slice assignment)
  // pending reductions, scans and contractions by expression hash (merging of equal ones at record time)
  std::unordered_multimap<uint64_t, uint64_t> pending_expensive;

  // options
  int64_t opt_fusion = 1;
  int64_t opt_rowred_max_cols = 16384;
  int64_t opt_map_rows = 0, opt_map_chunks = 0;
  int64_t opt_profile = 0;
  int64_t opt_nontemporal = 1;
  int64_t opt_map_bx = 0;
  int64_t opt_rowred_threads = 0;
  int64_t opt_rowred_rows = 0;
  int64_t opt_gemm_bn = 0;
  int64_t opt_pool_limit = 0;
  int64_t opt_stage_rows = 0;
  int64_t opt_stage_diag = 1;
  int64_t opt_gemv_slabs = 0, opt_gemv_unroll = 0;
  int64_t opt_gemv_pair = 1;
  int64_t opt_async_compile = 1;
  int64_t opt_disk_cache = 1;
  int64_t opt_merge = 1;
  int64_t opt_interp = 1;
  int64_t opt_assign_swap = 1;
  int64_t opt_dry_run = 0;
  int64_t opt_stage = 1;
  int64_t opt_plan_cache = 1;
  int64_t opt_scan_threads = 0, opt_scan_min_threads = 0;
  int64_t opt_scan_one_pass = 1;
  int64_t opt_gemm_kstep = 0;
  int64_t opt_gemm_split = 0;   // matrix product: workgroups per output tile along K (0 = chosen by the planner)
  int64_t opt_gemm_big = 1;     // matrix products of operands contiguous along one dimension: tiles loaded straight into LDS
  int64_t opt_map_phase = 1;
  int64_t opt_scan_polls = 1 << 20;   // polls a tile of a one-pass scan spends on each wait before it recomputes its offset
  uint64_t options_epoch = 0;  // bumped by every gr_ctx_set_option: part of a request's fingerprint
  uintptr_t dry_next = 0x100000;  // fake device addresses handed out by a dry run

  // allocator
  void* (*alloc_fn)(size_t, void*) = nullptr;
  void (*free_fn)(void*, void*) = nullptr;
  void* alloc_user = nullptr;
  std::unordered_map<size_t, std::vector<void*>> pool_free;  // default pool: size -> free blocks
  std::unordered_map<void*, size_t> pool_all;  // every block the pool got from hipMalloc -> its size
  size_t pool_bytes = 0;                       // their sum

  // kernel cache: signature -> compiled kernel
  struct Kernel {
    hipModule_t module = nullptr;
    hipFunction_t fn = nullptr;
    hipFunction_t fn2 = nullptr;  // second stage (combine kernels; chunk totals of a scan)
    hipFunction_t fn3 = nullptr;  // scan of the chunk totals
    std::vector<char> code;
    std::string name;
    size_t src_hash = 0;          // of the source text it was compiled from (compared in the self-checking mode)
  };
  std::unordered_map<std::string, Kernel> cache;
  std::unordered_map<std::string, size_t> dry_sources;  // signature -> hash of its source, kept by dry runs in the self-checking mode

  // run-time compilations in flight (signature -> job), see runtime.cpp
  struct CompileJob {
    std::string src, log, kernel;  // kernel: name of the entry point
    bool combine = false;  // the code object also holds a combine stage
    int scan = 0;          // ... the helper kernels of a scan (1: chunk totals and offsets, 2: cell clearing of a one-pass scan)
    std::vector<char> code;
    bool ok = false;
    double ms = 0.0;
  };
  std::unordered_map<std::string, std::pair<std::shared_ptr<CompileJob>, std::future<void>>> pending;
  std::string cache_dir;       // "" = not resolved yet, "-" = unavailable

  // plan cache: fingerprint hash -> remembered requests
  std::unordered_multimap<uint64_t, std::unique_ptr<gr::PlanEntry>> plan_cache;
  uint64_t walk_epoch = 0, plan_clock = 0;

  // workspace for two-stage kernels
  void* workspace = nullptr;
  size_t workspace_bytes = 0;
  // cells in which the tiles of one-pass scans publish their totals: a buffer of their own whose cells carry
  // the number of the launch that wrote them, so that no launch has to clear them first
  void* scan_cells = nullptr;
  size_t scan_cells_bytes = 0;
  uint32_t scan_epoch = 0;

  // gr_materialize_into_static: this device's copy of the library's static device array, and the
  // part of it the running request has taken (static_mode is set for the duration of such a call)
  unsigned char* static_base = nullptr;
  size_t static_cap = 0, static_used = 0;
  bool static_mode = false;
  bool plan_static = false;     // the request being planned is one of those: the planner keeps optional partial results within the array

  // gr_program_create: the request being recorded instead of executed, and the programs alive
  gr_program* capture = nullptr;
  std::vector<gr_program*> programs;

  // profiling
  struct ProfRec {
    std::string name;
    hipEvent_t e0, e1;
  };
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> event_pool;

  gr_stats_t stats{};
};

namespace gr {

gr_status fail(gr_ctx* c, gr_status s, const std::string& msg);
Node* lookup(gr_ctx* c, gr_array a);
Node* new_node(gr_ctx* c, Kind kind);
void node_unref_consumer(gr_ctx* c, Node* n);
void node_maybe_free(gr_ctx* c, Node* n);
void drop_inputs(gr_ctx* c, Node* n);

void* ctx_alloc(gr_ctx* c, size_t bytes);
void ctx_free(gr_ctx* c, void* p, size_t bytes);

// plan.cpp
gr_status make_plan(gr_ctx* c, Node* root, Plan* plan);           // plancache.cpp: remembered or planned afresh
gr_status make_plan_uncached(gr_ctx* c, Node* root, Plan* plan);  // plan.cpp
void clear_planned(Plan* plan);
gr_status expand_patch(gr_ctx* c, GroupPlan* g);
std::string describe_plan(const Plan& plan);

// codegen.cpp
std::string generate_source(const GroupPlan& g);
std::string kernel_name(const GroupPlan& g);

// runtime.cpp
gr_status prepare_group(gr_ctx* c, GroupPlan& g);
gr_status collect_all_jobs(gr_ctx* c, bool load);
gr_status compile_group(gr_ctx* c, GroupPlan& g, gr_ctx::Kernel** out);
gr_status launch_group(gr_ctx* c, const GroupPlan& g, gr_ctx::Kernel* k, void* out_ptr, void* pair_out_ptr);
gr_status execute_plan(gr_ctx* c, Plan* plan, Node* root, void* user_out, bool check_alias);

// static_scratch.hip
gr_status static_scratch_attach(gr_ctx* c);

}  // namespace gr
