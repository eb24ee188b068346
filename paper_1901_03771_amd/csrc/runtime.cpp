// Runtime: context lifetime, device memory pool, run-time compilation through
// hipRTC with a cache keyed on the sub-graph signature (the paper names JIT
// compilation as its main overhead, Section 4.2 and Section 6; one compiled
// kernel serves every request with the same structure, whatever the extents,
// strides and constants), argument marshalling and launches on the caller's
// stream, and the materialise entry points (Section 2: the computed node gets
// its data and is_materialized = true).
#include <dlfcn.h>
#include <hip/hip_runtime_api.h>
#include <hip/hiprtc.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <sys/stat.h>
#include <sys/types.h>
#include <unistd.h>

#include "codegen.h"
#include "ctx.h"
#include "interp.h"

extern "C" void gr_launch_stream_copy(void* stream, void* dst, const void* src, size_t n16);
extern "C" void gr_launch_stream_read(void* stream, const void* src, size_t n16, void* sink);

namespace gr {

bool interp_encode(const GroupPlan& g, void* out_ptr, GrInterpArgs* A, unsigned* grid);
gr_status interp_launch(gr_ctx* c, const GrInterpArgs& A, unsigned grid);
bool interp_encode_rowred(const GroupPlan& g, void* out_ptr, GrInterpRowArgs* R, unsigned* grid);
gr_status interp_launch_rowred(gr_ctx* c, const GrInterpRowArgs& R, unsigned grid);
bool interp_encode_gen(const GroupPlan& g, void* out_ptr, GrInterpGenArgs* G, unsigned* grid, bool half_of_pair = false,
                       const Node* fresh = nullptr, void* fresh_ptr = nullptr);
gr_status interp_launch_gen(gr_ctx* c, const GrInterpGenArgs& G, unsigned grid);

static std::string hip_err(hipError_t e) { return std::string(hipGetErrorName(e)) + ": " + hipGetErrorString(e); }

#define GR_HIP(c, call)                                                                           \
  do {                                                                                            \
    hipError_t e_ = (call);                                                                       \
    if (e_ != hipSuccess) return fail((c), GR_ERR_HIP, std::string(#call) + " -> " + hip_err(e_)); \
  } while (0)

// Returns every free block of the default pool to the device.  hipFree waits for the device, so
// a block that a queued kernel still reads (freed in host order, reused in stream order) is safe.
static void pool_trim(gr_ctx* c) {
  for (auto& kv : c->pool_free) {
    for (void* p : kv.second) {
      auto it = c->pool_all.find(p);
      if (it == c->pool_all.end()) continue;
      c->pool_bytes -= it->second;
      c->pool_all.erase(it);
      (void)hipFree(p);
    }
    kv.second.clear();
  }
  c->pool_free.clear();
}

// Inside the static device array of gr_materialize_into_static?
static inline bool in_static(const gr_ctx* c, const void* p) {
  return c->static_base && (const unsigned char*)p >= c->static_base && (const unsigned char*)p < c->static_base + c->static_cap;
}

void* ctx_alloc(gr_ctx* c, size_t bytes) {
  if (bytes == 0) bytes = 256;
  if (c->static_mode) {
    // a request that must not allocate: pieces of the static array, handed out once per call
    size_t rounded = (bytes + 255) & ~(size_t)255;
    if (rounded > c->static_cap - c->static_used) return nullptr;
    void* p = c->static_base + c->static_used;
    c->static_used += rounded;
    return p;
  }
  c->stats.bytes_allocated += bytes;
  if (c->alloc_fn) return c->alloc_fn(bytes, c->alloc_user);
  if (c->device < 0) {
    // dry run on a device-less context: distinct addresses that nothing ever dereferences
    void* p = (void*)c->dry_next;
    c->dry_next += (bytes + 255) & ~(uintptr_t)255;
    return p;
  }
  size_t rounded = (bytes + 255) & ~(size_t)255;
  auto& fl = c->pool_free[rounded];
  if (!fl.empty()) {
    void* p = fl.back();
    fl.pop_back();
    return p;
  }
  // nothing of this size is free: before the pool grows past its limit (option "pool_limit"), and
  // when the device has no memory left, the free blocks of other sizes go back to the device
  if (c->opt_pool_limit > 0 && c->pool_bytes + rounded > (size_t)c->opt_pool_limit) pool_trim(c);
  void* p = nullptr;
  if (hipMalloc(&p, rounded) != hipSuccess) {
    (void)hipGetLastError();
    pool_trim(c);
    if (hipMalloc(&p, rounded) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  }
  c->pool_all.emplace(p, rounded);
  c->pool_bytes += rounded;
  return p;
}

void ctx_free(gr_ctx* c, void* p, size_t bytes) {
  if (!p || in_static(c, p)) return;
  if (bytes == 0) bytes = 256;
  if (c->free_fn) { c->free_fn(p, c->alloc_user); return; }
  if (c->device < 0) return;
  // stream order makes reuse safe: every kernel of this context runs on one stream
  c->pool_free[(bytes + 255) & ~(size_t)255].push_back(p);
}

// ---- run-time compilation: in-memory cache, on-disk cache, host threads -----------------

// hipRTC on a worker thread: touches nothing but its job.  No FMA contraction and no fast-math
// (every recorded op rounds once, as in eager evaluation); packed FP32 instructions disabled.
static void run_hiprtc(gr_ctx::CompileJob* j) {
  auto t0 = std::chrono::steady_clock::now();
  hiprtcProgram prog;
  if (hiprtcCreateProgram(&prog, j->src.c_str(), "gr_kernel.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS) {
    j->log = "hiprtcCreateProgram failed";
    return;
  }
  const char* opts[] = {"--offload-arch=gfx950", "-O3", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
  hiprtcResult r = hiprtcCompileProgram(prog, 7, opts);
  if (r != HIPRTC_SUCCESS) {
    size_t n = 0;
    hiprtcGetProgramLogSize(prog, &n);
    j->log.assign(n, '\0');
    if (n) hiprtcGetProgramLog(prog, &j->log[0]);
    hiprtcDestroyProgram(&prog);
    return;
  }
  size_t cs = 0;
  hiprtcGetCodeSize(prog, &cs);
  j->code.resize(cs);
  hiprtcGetCode(prog, j->code.data());
  hiprtcDestroyProgram(&prog);
  j->ok = true;
  j->ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
}

static const char kDiskMagic[8] = {'G', 'R', 'C', 'O', '0', '0', '0', '3'};

static std::string cache_file_name(const std::string& key) {
  uint64_t h = 1469598103934665603ull;  // FNV-1a over a tool tag and the key (the kernel's source text)
  const std::string tag = std::string("grumpy-hip-3|") + std::to_string(HIP_VERSION) + "|gfx950|O3|";
  for (unsigned char ch : tag) { h ^= ch; h *= 1099511628211ull; }
  for (unsigned char ch : key) { h ^= ch; h *= 1099511628211ull; }
  char name[64];
  snprintf(name, sizeof name, "/%016llx_%zu.co", (unsigned long long)h, key.size());
  return name;
}

static std::string disk_path(gr_ctx* c, const std::string& key) {
  if (!c->opt_disk_cache) return "";
  if (c->cache_dir.empty()) {
    const char* env = getenv("GR_CACHE_DIR");
    const char* home = getenv("HOME");
    std::string dir = env ? env : (home ? std::string(home) + "/.cache/grumpy_hip" : "");
    c->cache_dir = "-";
    if (!dir.empty()) {
      std::string cmd;
      // create the directory (and parents) with plain mkdir calls
      for (size_t i = 1; i <= dir.size(); ++i)
        if (i == dir.size() || dir[i] == '/') ::mkdir(dir.substr(0, i).c_str(), 0755);
      struct stat st;
      if (::stat(dir.c_str(), &st) == 0 && S_ISDIR(st.st_mode)) c->cache_dir = dir;
    }
  }
  if (c->cache_dir == "-") return "";
  return c->cache_dir + cache_file_name(key);
}

// The kernel pack: code objects of common sub-graphs (the benchmark programs, plain pointwise
// operations, reductions, scans and contractions) that the build step compiles ahead of time
// into the directory `kernel_pack` beside this library (or $GR_KERNEL_PACK).  Same file format
// and naming as the user's cache, read-only, consulted after it; the stored source text is
// compared in full, so a pack written by another version of the generator never matches.
static std::string pack_path(gr_ctx* c, const std::string& key) {
  if (!c->opt_disk_cache) return "";
  if (const char* env = getenv("GR_KERNEL_PACK")) return *env ? env + cache_file_name(key) : std::string();
  static const std::string dir = [] {
    Dl_info info;
    if (dladdr((const void*)&cache_file_name, &info) && info.dli_fname) {
      std::string p = info.dli_fname;
      size_t slash = p.rfind('/');
      if (slash != std::string::npos) return p.substr(0, slash) + "/kernel_pack";
    }
    return std::string();
  }();
  return dir.empty() ? "" : dir + cache_file_name(key);
}

static bool disk_load(const std::string& path, const std::string& key, std::vector<char>* code) {
  if (path.empty()) return false;
  FILE* f = fopen(path.c_str(), "rb");
  if (!f) return false;
  bool ok = false;
  char magic[8];
  uint64_t sl = 0, cl = 0;
  if (fread(magic, 1, 8, f) == 8 && std::memcmp(magic, kDiskMagic, 8) == 0 && fread(&sl, 8, 1, f) == 1 && sl == key.size()) {
    std::string stored(sl, '\0');
    if ((sl == 0 || fread(&stored[0], 1, sl, f) == sl) && stored == key && fread(&cl, 8, 1, f) == 1 && cl > 0 && cl < (1ull << 30)) {
      code->resize(cl);
      ok = fread(code->data(), 1, cl, f) == cl;
    }
  }
  fclose(f);
  return ok;
}

static void disk_store(const std::string& path, const std::string& key, const std::vector<char>& code) {
  if (path.empty()) return;
  std::string tmp = path + ".tmp" + std::to_string((long long)getpid());
  FILE* f = fopen(tmp.c_str(), "wb");
  if (!f) return;
  uint64_t sl = key.size(), cl = code.size();
  bool ok = fwrite(kDiskMagic, 1, 8, f) == 8 && fwrite(&sl, 8, 1, f) == 1 && fwrite(key.data(), 1, sl, f) == sl &&
            fwrite(&cl, 8, 1, f) == 1 && fwrite(code.data(), 1, cl, f) == cl;
  ok = (fclose(f) == 0) && ok;
  if (ok) ::rename(tmp.c_str(), path.c_str());  // atomic: readers see a whole file or none
  else ::remove(tmp.c_str());
}

// What finish_kernel needs to know about a sub-graph: kept with a compilation job so that the
// job can be collected without the plan that started it.
// (scan: 0 = no scan, 1 = the code object also holds the chunk-total and offset kernels, 2 = the cell-clearing kernel
// of a one-pass scan)
static void kernel_entry_points(const GroupPlan& g, std::string* name, bool* combine, int* scan) {
  *name = kernel_name(g);
  *combine = (g.kind == GroupKind::GEMV && g.gemv_mode >= 1) || g.kind == GroupKind::REDUCE || g.kind == GroupKind::GEMM;
  *scan = g.kind == GroupKind::SCAN ? (g.scan_mode >= 2 ? 2 : 1) : 0;
}

// Loads a code object and publishes the kernel in the in-memory cache.
static gr_status finish_kernel(gr_ctx* c, const std::string& sig, const std::string& name, bool combine, int scan,
                               std::vector<char>&& code, const std::string& src, gr_ctx::Kernel** out) {
  gr_ctx::Kernel k;
  k.code = std::move(code);
  k.name = name;
  k.src_hash = std::hash<std::string>()(src);
  if (c->device >= 0) {
    GR_HIP(c, hipModuleLoadData(&k.module, k.code.data()));
    GR_HIP(c, hipModuleGetFunction(&k.fn, k.module, k.name.c_str()));
    if (combine) GR_HIP(c, hipModuleGetFunction(&k.fn2, k.module, (k.name + "_combine").c_str()));
    if (scan == 1) {
      GR_HIP(c, hipModuleGetFunction(&k.fn2, k.module, "gr_scan_sums"));
      GR_HIP(c, hipModuleGetFunction(&k.fn3, k.module, "gr_scan_offsets"));
    }
    if (scan == 2) GR_HIP(c, hipModuleGetFunction(&k.fn2, k.module, "gr_scan_clear"));
  }
  auto ins = c->cache.emplace(sig, std::move(k));
  if (out) *out = &ins.first->second;
  return GR_OK;
}

// Starts whatever a later compile_group() of this sub-graph will need: nothing on a cache
// hit, a module load on a disk hit, otherwise a hipRTC job on a host thread.  Calling this for
// every sub-graph of a request before running the first one overlaps compilation with
// execution (the paper names JIT time as its main bottleneck and pipelining as the remedy).
static void bound_pending(gr_ctx* c);

gr_status prepare_group(gr_ctx* c, GroupPlan& g) {
  if (c->cache.count(g.signature) || c->pending.count(g.signature)) return GR_OK;
  gr_status est = expand_patch(c, &g);
  if (est != GR_OK) return est;
  // The on-disk cache is keyed by the generated source text itself (plus compiler version and
  // flags), not by the signature: a library whose generator emits other code for the same
  // structure never picks up a code object written by another build.
  std::string src = generate_source(g);
  std::vector<char> code;
  if (disk_load(disk_path(c, src), src, &code) || disk_load(pack_path(c, src), src, &code)) {
    c->stats.cache_misses++;
    c->stats.disk_hits++;
    std::string name;
    bool combine;
    int scan;
    kernel_entry_points(g, &name, &combine, &scan);
    return finish_kernel(c, g.signature, name, combine, scan, std::move(code), src, nullptr);
  }
  bound_pending(c);
  auto job = std::make_shared<gr_ctx::CompileJob>();
  job->src = std::move(src);
  kernel_entry_points(g, &job->kernel, &job->combine, &job->scan);
  if (getenv("GR_LOG")) fprintf(stderr, "---- generated kernel ----\n%s\n", job->src.c_str());
  gr_ctx::CompileJob* raw = job.get();
  std::future<void> fut = c->opt_async_compile ? std::async(std::launch::async, run_hiprtc, raw) : std::async(std::launch::deferred, run_hiprtc, raw);
  c->pending.emplace(g.signature, std::make_pair(job, std::move(fut)));
  return GR_OK;
}

// Waits for the compilation job of `sig` (or, when deferred, runs it), stores the code object
// on disk and, unless `load` is false (context teardown), publishes the kernel.
static gr_status collect_job(gr_ctx* c, const std::string& sig, gr_ctx::Kernel** out, bool load = true) {
  auto pit = c->pending.find(sig);
  if (pit == c->pending.end()) return fail(c, GR_ERR_COMPILE, "no compilation job for this sub-graph");
  pit->second.second.get();
  std::shared_ptr<gr_ctx::CompileJob> job = pit->second.first;
  c->pending.erase(pit);
  c->stats.cache_misses++;
  c->stats.compile_ms += job->ms;
  if (!job->ok) {
    if (getenv("GR_LOG")) fprintf(stderr, "%s\n", job->src.c_str());
    return fail(c, GR_ERR_COMPILE, "hipRTC: " + job->log);
  }
  disk_store(disk_path(c, job->src), job->src, job->code);
  if (!load) return GR_OK;
  return finish_kernel(c, sig, job->kernel, job->combine, job->scan, std::move(job->code), job->src, out);
}

gr_status collect_all_jobs(gr_ctx* c, bool load) {
  gr_status first = GR_OK;
  std::string first_err;
  while (!c->pending.empty()) {
    std::string sig = c->pending.begin()->first;
    gr_status st = collect_job(c, sig, nullptr, load);
    if (st != GR_OK && first == GR_OK) { first = st; first_err = c->err; }
  }
  if (first != GR_OK) c->err = first_err;
  return first;
}

// Keeps the number of compilations in flight bounded: finished ones are collected, and beyond
// the bound the caller waits for one of them (each job occupies a host thread).
static void bound_pending(gr_ctx* c) {
  const size_t limit = 16;
  if (c->pending.size() < limit) return;
  std::vector<std::string> ready;
  for (auto& kv : c->pending)
    if (kv.second.second.wait_for(std::chrono::seconds(0)) != std::future_status::timeout) ready.push_back(kv.first);
  for (const std::string& sig : ready) (void)collect_job(c, sig, nullptr);
  while (c->pending.size() >= limit) {
    std::string sig = c->pending.begin()->first;
    (void)collect_job(c, sig, nullptr);
  }
}

// True while the kernel of `g` is neither cached nor ready to be collected without waiting.
static bool still_compiling(gr_ctx* c, const GroupPlan& g) {
  if (c->cache.count(g.signature)) return false;
  auto pit = c->pending.find(g.signature);
  if (pit == c->pending.end()) return false;
  return pit->second.second.wait_for(std::chrono::seconds(0)) == std::future_status::timeout;
}

gr_status compile_group(gr_ctx* c, GroupPlan& g, gr_ctx::Kernel** out) {
  auto it = c->cache.find(g.signature);
  if (it != c->cache.end()) {
    c->stats.cache_hits++;
    *out = &it->second;
    if (c->opt_plan_cache >= 2) {
      // self-checking mode: the signature has to determine the source; a plan whose source differs from the one
      // its cached kernel was compiled from would run a kernel written for other assumptions
      gr_status est = expand_patch(c, &g);
      if (est != GR_OK) return est;
      if (std::hash<std::string>()(generate_source(g)) != it->second.src_hash)
        return fail(c, GR_ERR_UNSUPPORTED, "kernel cache: this sub-graph's source differs from the source its signature was compiled from (" + kernel_name(g) + ")");
    }
    return GR_OK;
  }
  gr_status st = prepare_group(c, g);
  if (st != GR_OK) return st;
  it = c->cache.find(g.signature);
  if (it != c->cache.end()) { *out = &it->second; return GR_OK; }  // served from disk
  return collect_job(c, g.signature, out);
}

static gr_status launch(gr_ctx* c, hipFunction_t fn, const std::string& name, int64_t grid, std::vector<uint64_t>& args) {
  if (grid <= 0) return GR_OK;
  if (grid > 0x7fffffffLL) return fail(c, GR_ERR_UNSUPPORTED, "launch: grid too large");
  if (c->capture) {
    // recorded for replay instead of launched
    gr_program::Launch l;
    l.fn = fn;
    l.name = name;
    l.grid = (unsigned)grid;
    l.args = args;
    l.patch = c->capture->cur_patch;
    c->capture->launches.push_back(std::move(l));
    return GR_OK;
  }
  if (c->device < 0) { c->stats.kernel_launches++; return GR_OK; }  // dry run: everything but the launch itself
  size_t sz = args.size() * sizeof(uint64_t);
  void* extra[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, args.data(), HIP_LAUNCH_PARAM_BUFFER_SIZE, &sz, HIP_LAUNCH_PARAM_END};
  hipEvent_t e0 = nullptr, e1 = nullptr;
  const bool profile = c->opt_profile && !c->static_mode;  // (creating an event allocates)
  if (profile) {
    for (hipEvent_t* ev : {&e0, &e1}) {
      if (!c->event_pool.empty()) { *ev = c->event_pool.back(); c->event_pool.pop_back(); }
      else GR_HIP(c, hipEventCreate(ev));
    }
    GR_HIP(c, hipEventRecord(e0, c->stream));
  }
  GR_HIP(c, hipModuleLaunchKernel(fn, (unsigned)grid, 1, 1, 256, 1, 1, 0, c->stream, nullptr, extra));
  if (profile) {
    GR_HIP(c, hipEventRecord(e1, c->stream));
    c->prof.push_back({name, e0, e1});
  }
  c->stats.kernel_launches++;
  return GR_OK;
}

// Fills one sub-graph's block of the kernel argument array.
// `fresh` / `fresh_ptr`: a node whose buffer is being written by this very launch (the first
// sub-graph's result inside a fused pair) and therefore has no data pointer yet.
// Stands for "the caller's output buffer" while a request is recorded for replay.
static void* const kReplayOut = (void*)(uintptr_t)0x10;

// `slot0`: position of this block inside the launch's whole argument array (a fused pair has two blocks).
static gr_status fill_args(gr_ctx* c, const GroupPlan& g, const ArgLayout& L, void* out_ptr, uint64_t* s,
                           const Node* fresh = nullptr, void* fresh_ptr = nullptr, int slot0 = 0) {
  for (size_t gi = 0; gi < g.groups.size(); ++gi) {
    const AccessGroup& ag = g.groups[gi];
    void* data = ag.leaf == fresh ? fresh_ptr : ag.leaf->data;
    if (!data && ag.leaf->count() > 0) return fail(c, GR_ERR_HIP, "launch: a leaf has no data");
    s[L.ptr[gi]] = (uint64_t)(uintptr_t)data;
    if (c->capture) {
      if (data == kReplayOut) c->capture->cur_patch.push_back({slot0 + L.ptr[gi], -1});
      else
        for (size_t k = 0; k < c->capture->leaf_nodes.size(); ++k)
          if (c->capture->leaf_nodes[k] == ag.leaf) { c->capture->cur_patch.push_back({slot0 + L.ptr[gi], (int)k}); break; }
    }
    s[L.base[gi]] = (uint64_t)ag.base;
    for (int k2 = 0; k2 < L.ncoef[gi]; ++k2) s[L.coef[gi] + k2] = (uint64_t)ag.coef[k2];
  }
  s[L.out] = (uint64_t)(uintptr_t)out_ptr;
  if (c->capture && out_ptr == kReplayOut) c->capture->cur_patch.push_back({slot0 + L.out, -1});
  for (int k2 = 0; k2 < g.rank; ++k2) s[L.dims + k2] = (uint64_t)g.dims[k2];
  for (size_t i = 0; i < g.consts.size(); ++i) {
    const ConstSlot& cs = g.consts[i];
    if (cs.dtype == GR_F32) { float f = (float)cs.value; uint32_t u; std::memcpy(&u, &f, 4); s[L.consts + i] = u; }
    else if (cs.dtype == GR_I32) s[L.consts + i] = (uint32_t)(int32_t)(int64_t)cs.value;
    else s[L.consts + i] = (uint64_t)(int64_t)cs.value;
  }
  return GR_OK;
}

// One-pass scan along a non-contiguous axis: tiles of 4*BX neighbouring lines; per chain of tiles
// one cell per line for every tile and for every group of `slabs` tiles.
static int64_t scan_line_tile_chains(const GroupPlan& g) {
  const int64_t D = g.dims[g.rank - 2], W = 4 * (int64_t)g.BX;
  return D > 0 ? (g.red_out / D) * ((D + W - 1) / W) : 0;
}
static int64_t scan_line_tile_cells(const GroupPlan& g) {
  const int64_t G = std::max(1, g.slabs);
  return scan_line_tile_chains(g) * ((int64_t)g.scan_nchunk + ((int64_t)g.scan_nchunk + G - 1) / G) * 4 * (int64_t)g.BX;
}

// Device memory a sub-graph's kernels need beyond inputs and output: the first-stage partial
// results of two-stage kernels.
static size_t workspace_need(const GroupPlan& g) {
  switch (g.kind) {
    case GroupKind::REDUCE: return g.slabs > 1 && g.red_out > 0 ? (size_t)g.slabs * (size_t)g.red_out * itemsize(g.out_dtype) : 0;
    case GroupKind::SCAN: {
      int64_t total = 1;
      for (int k2 = 0; k2 < g.rank; ++k2) total *= g.dims[k2];
      if (g.scan_mode == 3) return total > 0 ? (size_t)scan_line_tile_cells(g) * 8 : 0;
      if (g.scan_mode == 2)  // one 8-byte cell per tile and per group of 128 tiles
        return total > 0 ? ((size_t)g.red_out * (size_t)g.scan_nchunk + (size_t)g.red_out * (size_t)((g.scan_nchunk + 127) / 128)) * 8 : 0;
      return g.scan_nchunk > 1 && total > 0 ? (size_t)g.red_out * (size_t)g.scan_nchunk * itemsize(g.out_dtype) : 0;
    }
    case GroupKind::GEMM: return g.slabs > 1 && g.M > 0 && g.N > 0 ? (size_t)g.slabs * (size_t)g.M * (size_t)g.N * sizeof(float) : 0;
    case GroupKind::GEMV:
      if (g.M == 0) return 0;
      if (g.gemv_mode == 2) return (size_t)g.slabs * (size_t)g.K * sizeof(float);
      if (g.gemv_mode == 1) return (size_t)g.slabs * (size_t)g.M * sizeof(float);
      return 0;
    default: return 0;
  }
}

// Returns the workspace of `g` (NULL if it needs none): the context's own, grown on demand, or,
// for a request that must not allocate, a piece of the static array.
static gr_status get_workspace(gr_ctx* c, const GroupPlan& g, void** ws) {
  *ws = nullptr;
  const size_t need = workspace_need(g);
  if (need == 0) return GR_OK;
  if (c->static_mode) {
    *ws = ctx_alloc(c, need);
    return *ws ? GR_OK : fail(c, GR_ERR_OOM, "the static scratch array is too small for this request's partial results");
  }
  if (c->capture) {
    // a recorded request keeps workspaces of its own: replays must not depend on what the context's
    // shared workspace is used for in between
    *ws = ctx_alloc(c, need);
    if (!*ws) return fail(c, GR_ERR_OOM, "workspace allocation failed");
    c->capture->buffers.push_back({*ws, need});
    return GR_OK;
  }
  if (need > c->workspace_bytes) {
    if (c->workspace) ctx_free(c, c->workspace, c->workspace_bytes);
    c->workspace = ctx_alloc(c, need);
    c->workspace_bytes = c->workspace ? need : 0;
    if (!c->workspace) return fail(c, GR_ERR_OOM, "workspace allocation failed");
  }
  *ws = c->workspace;
  return GR_OK;
}

// Cells of a one-pass scan.  Ordinarily they live in a buffer that only such scans use: every cell
// carries the number of the launch that wrote it (the upper half of the 8-byte word), launches are
// numbered per context and run in stream order, so a launch tells its own cells from stale ones
// without anybody clearing them; the buffer is zeroed when it is (re)allocated and when the numbers
// wrap.  `*tag` = 0 means: the caller has to clear the cells it gets (from the shared workspace)
// and the launch uses tag 1 -- for requests that must not allocate, for requests recorded for
// replay, and while the caller's stream is being captured into a HIP graph (a replay would repeat
// the tag, and memset nodes are not recorded here).
static gr_status scan_cells(gr_ctx* c, const GroupPlan& g, size_t need, void** cells, uint32_t* tag) {
  *tag = 0;
  bool plain = c->static_mode || c->capture != nullptr || c->device < 0;
  if (!plain) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(c->stream, &cs) != hipSuccess) { (void)hipGetLastError(); plain = true; }
    else if (cs != hipStreamCaptureStatusNone) plain = true;
  }
  if (plain) {
    // while a caller captures the stream nothing may be allocated: the scans' own buffer serves if an
    // earlier launch has made it large enough (its cells are cleared like any other; tag 1 is older
    // than every launch number still to come)
    if (!c->static_mode && !c->capture && c->device >= 0 && c->scan_cells && need <= c->scan_cells_bytes) { *cells = c->scan_cells; return GR_OK; }
    return get_workspace(c, g, cells);
  }
  bool zero = false;
  if (need > c->scan_cells_bytes) {
    if (c->scan_cells) ctx_free(c, c->scan_cells, c->scan_cells_bytes);
    const size_t bytes = std::max<size_t>(need, (size_t)1 << 20);
    c->scan_cells = ctx_alloc(c, bytes);
    c->scan_cells_bytes = c->scan_cells ? bytes : 0;
    if (!c->scan_cells) return fail(c, GR_ERR_OOM, "allocation of the scan cells failed");
    zero = true;
  }
  if (++c->scan_epoch == 0) zero = true;
  if (zero) {
    GR_HIP(c, hipMemsetAsync(c->scan_cells, 0, c->scan_cells_bytes, c->stream));
    c->scan_epoch = 1;
  }
  *cells = c->scan_cells;
  *tag = c->scan_epoch;
  return GR_OK;
}

gr_status launch_group(gr_ctx* c, const GroupPlan& g, gr_ctx::Kernel* k, void* out_ptr, void* pair_out_ptr) {
  ArgLayout L = arg_layout(g);
  ArgLayout L2;
  if (g.pair) L2 = arg_layout(*g.pair);
  std::vector<uint64_t> s(L.total + (g.pair ? L2.total : 0), 0);
  if (c->capture) c->capture->cur_patch.clear();
  gr_status fst = fill_args(c, g, L, out_ptr, s.data());
  if (fst != GR_OK) return fst;
  void* ws = nullptr;
  int64_t total = 1;
  for (int k2 = 0; k2 < g.rank; ++k2) total *= g.dims[k2];
  switch (g.kind) {
    case GroupKind::MAP: {
      if (total == 0) return GR_OK;
      for (int k2 = 0; k2 < g.rank; ++k2) s[L.ocoef + k2] = (uint64_t)g.out_coef[k2];
      s[L.obase] = (uint64_t)g.out_base;
      int64_t C = g.dims[g.rank - 1], R = g.rank >= 2 ? g.dims[g.rank - 2] : 1, outer = 1;
      for (int k2 = 0; k2 + 2 < g.rank; ++k2) outer *= g.dims[k2];
      int64_t TC = (int64_t)g.BX * 4 * g.UC, TR = (int64_t)g.BY * g.VR;
      int64_t ntiles = outer * ((C + g.cphase + TC - 1) / TC) * ((R + TR - 1) / TR);
      int64_t grid = g.xcd_remap ? 8 * ((ntiles + 7) / 8) : ntiles;
      return launch(c, k->fn, k->name, grid, s);
    }
    case GroupKind::ROWRED: {
      int64_t rows = 1;
      for (int k2 = 0; k2 + 1 < g.rank; ++k2) rows *= g.dims[k2];
      if (rows == 0) return GR_OK;
      int rb = 256 / g.row_threads * g.row_iters;
      return launch(c, k->fn, k->name, (rows + rb - 1) / rb, s);
    }
    case GroupKind::REDUCE: {
      if (g.red_out == 0) return GR_OK;
      s[L.extra] = (uint64_t)g.red_out;
      s[L.extra + 1] = (uint64_t)g.red_len;
      s[L.extra + 3] = (uint64_t)g.slabs;
      if (g.slabs > 1) {
        gr_status wst = get_workspace(c, g, &ws);
        if (wst != GR_OK) return wst;
        s[L.extra + 2] = (uint64_t)(uintptr_t)ws;
      }
      int64_t units = g.red_mode == 0 ? ((g.red_vec ? g.red_out / 4 : g.red_out) + 255) / 256 : g.red_out;
      gr_status st = launch(c, k->fn, k->name, units * g.slabs, s);
      if (st != GR_OK || g.slabs <= 1) return st;
      return launch(c, k->fn2, k->name + "_combine", g.red_out >= 1024 ? (g.red_out + 255) / 256 : g.red_out, s);
    }
    case GroupKind::SCAN: {
      if (total == 0) return GR_OK;
      for (int k2 = 0; k2 < g.rank; ++k2) s[L.ocoef + k2] = (uint64_t)g.out_coef[k2];
      s[L.extra] = (uint64_t)g.red_out;
      s[L.extra + 1] = (uint64_t)g.scan_chunk;
      s[L.extra + 3] = (uint64_t)g.scan_nchunk | (g.scan_mode >= 2 ? (uint64_t)c->opt_scan_polls << 32 : 0);
      if (g.scan_mode >= 2) {
        // one pass: the tiles publish their totals in cells (cleared first unless they carry launch numbers)
        uint32_t tag = 0;
        gr_status wst = scan_cells(c, g, workspace_need(g), &ws, &tag);
        if (wst != GR_OK) return wst;
        const uint64_t low = g.scan_mode == 3 ? (uint64_t)std::max(1, g.slabs) : (uint64_t)g.scan_chunk;
        s[L.extra + 1] = low | ((uint64_t)(tag ? tag : 1u) << 32);
        s[L.extra + 2] = (uint64_t)(uintptr_t)ws;
        const int64_t cells = g.scan_mode == 3 ? scan_line_tile_cells(g) : g.red_out * g.scan_nchunk + g.red_out * ((g.scan_nchunk + 127) / 128);
        if (!tag) {
          gr_status st = launch(c, k->fn2, "gr_scan_clear", (cells + 255) / 256, s);
          if (st != GR_OK) return st;
        }
        return launch(c, k->fn, k->name, g.scan_mode == 3 ? scan_line_tile_chains(g) * g.scan_nchunk : g.red_out * g.scan_nchunk, s);
      }
      if (g.scan_mode == 1) {
        // a thread per (line, chunk)
        const int64_t blocks = ((g.scan_vec ? g.red_out / 4 : g.red_out) * g.scan_nchunk + 255) / 256;
        if (g.scan_nchunk > 1) {
          gr_status wst = get_workspace(c, g, &ws);
          if (wst != GR_OK) return wst;
          s[L.extra + 2] = (uint64_t)(uintptr_t)ws;
          gr_status st = launch(c, k->fn2, "gr_scan_sums", blocks, s);
          if (st != GR_OK) return st;
          st = launch(c, k->fn3, "gr_scan_offsets", g.red_out, s);
          if (st != GR_OK) return st;
        }
        return launch(c, k->fn, k->name, blocks, s);
      }
      if (g.scan_nchunk > 1) {
        gr_status wst = get_workspace(c, g, &ws);
        if (wst != GR_OK) return wst;
        s[L.extra + 2] = (uint64_t)(uintptr_t)ws;
        gr_status st = launch(c, k->fn2, "gr_scan_sums", g.red_out * g.scan_nchunk, s);
        if (st != GR_OK) return st;
        st = launch(c, k->fn3, "gr_scan_offsets", g.red_out, s);
        if (st != GR_OK) return st;
      }
      return launch(c, k->fn, k->name, g.red_out * g.scan_nchunk, s);
    }
    case GroupKind::GEMM: {
      if (g.M == 0 || g.N == 0) return GR_OK;
      s[L.extra] = (uint64_t)g.M;
      s[L.extra + 1] = (uint64_t)g.N;
      s[L.extra + 2] = (uint64_t)g.K;
      const int64_t bn = g.BX == 32 ? 32 : 128;
      // (VR = 2: the kernels whose tiles go straight into LDS, one workgroup per BX x BX tile)
      const int64_t tiles = g.VR == 2 ? ((g.M + g.BX - 1) / g.BX) * ((g.N + g.BX - 1) / g.BX) : ((g.M + 127) / 128) * ((g.N + bn - 1) / bn);
      const int64_t nsplit = std::max(1, g.slabs);
      const int64_t kch = gemm_split_extent(g.K, nsplit);
      s[L.extra + 3] = (uint64_t)nsplit;
      s[L.ocoef + 1] = (uint64_t)std::max<int64_t>(kch, 1);
      if (nsplit > 1) {
        gr_status wst = get_workspace(c, g, &ws);
        if (wst != GR_OK) return wst;
        s[L.ocoef] = (uint64_t)(uintptr_t)ws;
      }
      gr_status st = launch(c, k->fn, k->name, tiles * nsplit, s);
      if (st != GR_OK || nsplit <= 1) return st;
      return launch(c, k->fn2, k->name + "_combine", (g.M * g.N + 255) / 256, s);
    }
    case GroupKind::GEMV: {
      if (g.M == 0) return GR_OK;
      s[L.extra] = (uint64_t)g.M;
      s[L.extra + 1] = (uint64_t)g.K;
      if (g.gemv_mode == 2) {
        // one pass over the matrix for both contractions; the second block of arguments is the
        // column-accumulate sub-graph's (read by the combine kernel)
        const GroupPlan& p = *g.pair;
        fst = fill_args(c, p, L2, pair_out_ptr, s.data() + L.total, g.root, out_ptr, L.total);
        if (fst != GR_OK) return fst;
        gr_status wst = get_workspace(c, g, &ws);
        if (wst != GR_OK) return wst;
        s[L.extra + 2] = (uint64_t)(uintptr_t)ws;
        s[L.extra + 3] = (uint64_t)g.slabs;
        uint64_t* s2 = s.data() + L.total;
        s2[L2.extra] = (uint64_t)p.M;
        s2[L2.extra + 1] = (uint64_t)p.K;
        s2[L2.extra + 2] = (uint64_t)(uintptr_t)ws;
        s2[L2.extra + 3] = (uint64_t)g.slabs;
        gr_status st = launch(c, k->fn, k->name, g.slabs, s);
        if (st != GR_OK) return st;
        return launch(c, k->fn2, k->name + "_combine", (p.M + 15) / 16, s);
      }
      if (g.gemv_mode == 0) {
        int rpb = 256 / g.LPR;
        int64_t grid = std::min<int64_t>((g.M + rpb - 1) / rpb, 256 * 16);
        return launch(c, k->fn, k->name, grid, s);
      }
      gr_status wst = get_workspace(c, g, &ws);
      if (wst != GR_OK) return wst;
      s[L.extra + 2] = (uint64_t)(uintptr_t)ws;
      s[L.extra + 3] = (uint64_t)g.slabs;
      int64_t ncb = (g.M + (int64_t)g.BX * 4 - 1) / ((int64_t)g.BX * 4);
      gr_status st = launch(c, k->fn, k->name, ncb * g.slabs, s);
      if (st != GR_OK) return st;
      return launch(c, k->fn2, k->name + "_combine", (g.M + 15) / 16, s);
    }
  }
  return GR_OK;
}

// Address range [lo, hi) touched by a strided array.
static void extent_of(const Node* n, uintptr_t* lo, uintptr_t* hi) {
  int64_t mn = n->offset, mx = n->offset;
  for (int d = 0; d < n->ndim; ++d) {
    if (n->shape[d] == 0) { *lo = *hi = 0; return; }
    int64_t span = (n->shape[d] - 1) * n->strides[d];  // both factors are bounded when the node is recorded
    if (span < 0) mn += span; else mx += span;
  }
  *lo = (uintptr_t)n->data + mn * itemsize(n->dtype);
  *hi = (uintptr_t)n->data + (mx + 1) * itemsize(n->dtype);
}

// Materialised, or a chain of views that ends at a materialised array.
static bool has_storage(const Node* n) {
  while (!n->materialized) {
    if (!n->is_view()) return false;
    n = n->in[0];
  }
  return true;
}

// Results of earlier sub-graphs that a non-allocating request stored in the static array exist
// only for the duration of that request (the next call overwrites them): their nodes go back to
// being unevaluated, with their inputs, and can be evaluated again later.
static void static_unbind(gr_ctx* c, Plan* plan) {
  if (!c->static_mode) return;
  for (auto& gp : plan->groups)
    for (Node* r : {gp->root, gp->pair ? gp->pair->root : (Node*)nullptr}) {
      if (!r || !r->materialized || !in_static(c, r->data)) continue;
      r->data = nullptr;
      r->owns_data = false;
      r->alloc_bytes = 0;
      if (r->count() > 0) r->materialized = false;  // (an empty array needs no storage)
    }
}

gr_status execute_plan(gr_ctx* c, Plan* plan, Node* root, void* user_out, bool check_alias) {
  if (c->device < 0 && !c->opt_dry_run) return fail(c, GR_ERR_NODEVICE, "context has no device");
  if (user_out && check_alias) {
    uintptr_t olo = (uintptr_t)user_out, ohi = olo + root->count() * itemsize(root->dtype);
    for (const auto& g : plan->groups)
      for (const GroupPlan* gp : {g.get(), g->pair.get()}) {
        if (!gp) continue;
        for (const Node* l : gp->leaves) {
          if (!l->materialized) continue;
          uintptr_t lo, hi;
          extent_of(l, &lo, &hi);
          if (lo < ohi && olo < hi) return fail(c, GR_ERR_ALIAS, "output buffer overlaps an input of the request");
        }
      }
  }
  static gr_ctx::Kernel dry_kernel;  // stands for any kernel in a dry run that does not compile
  const bool no_compile = c->device < 0 && c->opt_dry_run >= 2;
  if (c->static_mode) {
    // A request that must not allocate: checked in full before the first launch.  Every kernel
    // has to be loaded already (loading a code object allocates device memory), and the stored
    // results of earlier sub-graphs plus the partial results of two-stage kernels have to fit
    // the static array.
    size_t need = 0;
    for (auto& gp : plan->groups) {
      if (!no_compile && !c->cache.count(gp->signature))
        return fail(c, GR_ERR_UNSUPPORTED, "materialize_into_static: a kernel of this request is not loaded yet; call gr_plan_compile "
                                           "(or evaluate a request of the same structure with gr_materialize_into) once first");
      for (const Node* r : {(const Node*)gp->root, gp->pair ? (const Node*)gp->pair->root : nullptr}) {
        if (!r || (r == root && user_out)) continue;
        size_t nb = (size_t)r->count() * itemsize(r->dtype);
        need += ((nb ? nb : 256) + 255) & ~(size_t)255;
      }
      need += (workspace_need(*gp) + 255) & ~(size_t)255;
    }
    if (need > c->static_cap)
      return fail(c, GR_ERR_OOM, "materialize_into_static: the request needs " + std::to_string(need) + " bytes for intermediate and partial results; "
                                 "the static scratch array holds " + std::to_string(c->static_cap));
  }
  c->stats.materialize_calls++;
  for (auto& gp : plan->groups) {
    if (c->static_mode) break;
    if (no_compile || c->opt_interp >= 2) continue;  // no kernel wanted (yet)
    gr_status pst = prepare_group(c, *gp);
    if (pst != GR_OK) return pst;
  }
  for (auto& gp : plan->groups) {
    GroupPlan& g = *gp;
    gr_ctx::Kernel* k = nullptr;
    // A map sub-graph whose kernel is still in the compiler runs through the byte-code
    // interpreter instead of waiting; the job stays pending and a later request collects it.
    // (option "interp" = 2: every map sub-graph the interpreter covers, compiled or not)
    const bool try_interp = !c->static_mode && !c->capture &&
                            (c->opt_interp >= 2 || (c->opt_interp == 1 && still_compiling(c, g)));
    if (no_compile) k = &dry_kernel;
    if (no_compile && c->opt_plan_cache >= 2) {
      // self-checking dry run: nothing is compiled, but the source is generated and has to be the one that any
      // earlier sub-graph with this signature produced (the kernel cache is keyed by the signature)
      gr_status est = expand_patch(c, &g);
      if (est != GR_OK) { static_unbind(c, plan); return est; }
      const size_t h = std::hash<std::string>()(generate_source(g));
      auto ins = c->dry_sources.emplace(g.signature, h);
      if (!ins.second && ins.first->second != h) {
        static_unbind(c, plan);
        return fail(c, GR_ERR_UNSUPPORTED, "kernel cache: this sub-graph's source differs from the source of an earlier one with the same signature (" + kernel_name(g) + ")");
      }
    }
    gr_status st = (try_interp || no_compile) ? GR_OK : compile_group(c, g, &k);
    if (st != GR_OK) { static_unbind(c, plan); return st; }
    // output buffers: the caller's for the requested root, the allocator's otherwise
    Node* roots[2] = {g.root, g.pair ? g.pair->root : nullptr};
    void* outs[2] = {nullptr, nullptr};
    size_t nbytes[2] = {0, 0};
    bool own[2] = {false, false};
    for (int q = 0; q < 2 && roots[q]; ++q) {
      nbytes[q] = (size_t)roots[q]->count() * itemsize(roots[q]->dtype);
      if (roots[q] == root && user_out) outs[q] = user_out;
      else {
        outs[q] = ctx_alloc(c, nbytes[q]);
        if (!outs[q]) { if (q == 1 && own[0]) ctx_free(c, outs[0], nbytes[0]); static_unbind(c, plan); return fail(c, GR_ERR_OOM, "allocator returned NULL"); }
        own[q] = true;
      }
    }
    bool interpreted = false;
    if (try_interp) {
      GrInterpArgs ia;
      unsigned igrid = 0;
      int64_t total = 1;
      for (int k2 = 0; k2 < g.rank; ++k2) total *= g.dims[k2];
      if (g.pair) {
        // two contractions that share one generated kernel: the interpreter runs them one after the other
        GrInterpGenArgs ga, gb;
        unsigned grid_b = 0;
        if (total > 0 && interp_encode_gen(g, outs[0], &ga, &igrid, true) && interp_encode_gen(*g.pair, outs[1], &gb, &grid_b, true, g.root, outs[0])) {
          st = interp_launch_gen(c, ga, igrid);
          if (st == GR_OK) st = interp_launch_gen(c, gb, grid_b);
          interpreted = true;
        }
      } else if (total == 0 && g.kind == GroupKind::MAP) interpreted = true;  // nothing to compute
      else if (g.kind == GroupKind::MAP && interp_encode(g, outs[0], &ia, &igrid)) {
        st = interp_launch(c, ia, igrid);
        interpreted = true;
      } else if (g.kind == GroupKind::ROWRED) {
        GrInterpRowArgs ra;
        if (interp_encode_rowred(g, outs[0], &ra, &igrid)) {
          st = interp_launch_rowred(c, ra, igrid);
          interpreted = true;
        }
      } else if (g.kind != GroupKind::MAP && total > 0) {
        // reductions over any axes, scans, contractions with their epilogues
        GrInterpGenArgs ga;
        if (interp_encode_gen(g, outs[0], &ga, &igrid)) {
          void* part = nullptr;
          const size_t part_bytes = ga.nsplit > 1 ? (size_t)igrid * 8 : 0;
          if (part_bytes) part = ctx_alloc(c, part_bytes);
          if (part_bytes && !part) ga.nsplit = 1, igrid = (unsigned)ga.nout;   // no room for partial results: one workgroup per output
          ga.partial = (unsigned long long)(uintptr_t)part;
          st = interp_launch_gen(c, ga, igrid);
          if (st == GR_OK && ga.nsplit > 1) {
            ga.kind = GI_KIND_COMBINE;
            st = interp_launch_gen(c, ga, (unsigned)ga.nout);
          }
          if (part) ctx_free(c, part, part_bytes);   // (the pool hands blocks out again in stream order)
          interpreted = true;
        }
      }
    }
    if (!interpreted) {
      if (!k) st = compile_group(c, g, &k);
      if (st == GR_OK) st = launch_group(c, g, k, outs[0], outs[1]);
    }
    if (st != GR_OK) {
      for (int q = 0; q < 2; ++q) if (own[q]) ctx_free(c, outs[q], nbytes[q]);
      static_unbind(c, plan);
      return st;
    }
    c->stats.groups_executed += g.pair ? 2 : 1;
    for (int q = 0; q < 2 && roots[q]; ++q) {
      Node* r = roots[q];
      // a plain copy of an array that already had data (or of a view of one: a view stays a view
      // of its base, it is never bound to the buffer its elements were copied to)
      if (has_storage(r)) continue;
      // the node now has data and stays materialised (Section 2)
      r->data = outs[q];
      r->owns_data = own[q];
      r->alloc_bytes = own[q] ? nbytes[q] : 0;
      r->offset = 0;
      int64_t sstride = 1;
      for (int d = r->ndim - 1; d >= 0; --d) { r->strides[d] = sstride; sstride *= r->shape[d]; }
      if (r == root && plan->out && plan->out_honoured) {
        // written straight into another array's storage (slice assignment): the node's data
        // is that region until the storage is written again
        r->offset = plan->out->base;
        for (int d = 0; d < r->ndim; ++d) r->strides[d] = plan->out->strides[d];
        r->cow_alias = true;
        c->any_storage_alias = true;
      }
      r->materialized = true;
      r->planned = false;
    }
  }
  // The plan's marks are cleared while every node it names is still alive: releasing the
  // predecessors below may free intermediate roots that nothing else refers to.
  clear_planned(plan);
  static_unbind(c, plan);
  // Predecessors of materialised nodes are no longer needed.  Roots are visited in execution
  // (topological) order: dropping a root's inputs can only free nodes upstream of it, which
  // includes earlier roots that nothing else refers to, never a root still to be visited.
  for (auto& gp : plan->groups) {
    if (gp->root->materialized) drop_inputs(c, gp->root);  // (a view keeps its base)
    if (gp->pair && gp->pair->root->materialized) drop_inputs(c, gp->pair->root);
  }
  return GR_OK;
}

// Runs the planner's sub-graph list of `root` with recording switched on (c->capture): kernels are
// compiled and loaded, stored results of earlier sub-graphs and workspaces are allocated for the
// program to keep, every launch is written down instead of issued, and the nodes are left as
// they were (nothing becomes materialised, no input is released).
static gr_status record_plan(gr_ctx* c, Plan* plan, Node* root) {
  gr_program* P = c->capture;
  for (auto& gp : plan->groups) {
    gr_status pst = prepare_group(c, *gp);  // all compilations of the request start together
    if (pst != GR_OK) return pst;
  }
  std::vector<Node*> bound;
  gr_status st = GR_OK;
  for (auto& gp : plan->groups) {
    GroupPlan& g = *gp;
    gr_ctx::Kernel* k = nullptr;
    st = compile_group(c, g, &k);
    if (st != GR_OK) break;
    Node* roots[2] = {g.root, g.pair ? g.pair->root : nullptr};
    void* outs[2] = {nullptr, nullptr};
    for (int q = 0; q < 2 && roots[q] && st == GR_OK; ++q) {
      if (roots[q] == root) { outs[q] = kReplayOut; continue; }
      const size_t nb = (size_t)roots[q]->count() * itemsize(roots[q]->dtype);
      outs[q] = ctx_alloc(c, nb);
      if (!outs[q]) st = fail(c, GR_ERR_OOM, "allocator returned NULL");
      else P->buffers.push_back({outs[q], nb});
    }
    if (st != GR_OK) break;
    st = launch_group(c, g, k, outs[0], outs[1]);
    if (st != GR_OK) break;
    for (int q = 0; q < 2 && roots[q]; ++q) {
      Node* r = roots[q];
      if (has_storage(r)) continue;
      // visible to the later sub-graphs of this recording only
      r->data = outs[q];
      r->owns_data = false;
      r->alloc_bytes = 0;
      r->offset = 0;
      int64_t sstride = 1;
      for (int d = r->ndim - 1; d >= 0; --d) { r->strides[d] = sstride; sstride *= r->shape[d]; }
      r->materialized = true;
      r->planned = false;
      bound.push_back(r);
    }
  }
  clear_planned(plan);
  for (Node* r : bound) { r->data = nullptr; r->materialized = false; }
  return st;
}

static void program_free(gr_ctx* c, gr_program* P) {
  for (auto& b : P->buffers) ctx_free(c, b.first, b.second);
  for (size_t i = 0; i < c->programs.size(); ++i)
    if (c->programs[i] == P) { c->programs.erase(c->programs.begin() + i); break; }
  delete P;
}

}  // namespace gr

using namespace gr;

extern "C" {

gr_status gr_program_create(gr_ctx* ctx, gr_array root, const gr_array* leaves, int nleaves, gr_program** out) {
  if (!ctx || !out || nleaves < 0 || (nleaves > 0 && !leaves)) return GR_ERR_ARG;
  Node* x = lookup(ctx, root);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "program_create: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "program_create: a bare scalar has no array value");
  if (ctx->device < 0 && !ctx->opt_dry_run) return fail(ctx, GR_ERR_NODEVICE, "context has no device");
  std::unique_ptr<gr_program> P(new gr_program());
  P->ctx = ctx;
  for (int i = 0; i < nleaves; ++i) {
    const Node* l = lookup(ctx, leaves[i]);
    if (!l) return fail(ctx, GR_ERR_HANDLE, "program_create: bad leaf handle");
    if (l->kind != Kind::LEAF || !l->data) return fail(ctx, GR_ERR_ARG, "program_create: a rebindable input must be an array made by gr_array_from_device");
    for (const Node* m : P->leaf_nodes) if (m == l) return fail(ctx, GR_ERR_ARG, "program_create: the same leaf is listed twice");
    uintptr_t lo, hi;
    extent_of(l, &lo, &hi);
    if (lo < (uintptr_t)l->data) return fail(ctx, GR_ERR_UNSUPPORTED, "program_create: a rebindable input reaches below its address (negative strides)");
    P->leaf_nodes.push_back(l);
    P->leaf_bytes.push_back(hi > (uintptr_t)l->data ? (size_t)(hi - (uintptr_t)l->data) : 0);
  }
  P->out_bytes = (size_t)x->count() * itemsize(x->dtype);
  Plan plan;
  gr_status st = make_plan(ctx, x, &plan);
  if (st != GR_OK) return st;
  ctx->capture = P.get();
  st = record_plan(ctx, &plan, x);
  ctx->capture = nullptr;
  clear_planned(&plan);
  P->leaf_nodes.clear();
  P->cur_patch.clear();
  if (st != GR_OK) {
    for (auto& b : P->buffers) ctx_free(ctx, b.first, b.second);
    return st;
  }
  ctx->programs.push_back(P.get());
  *out = P.release();
  return GR_OK;
}

gr_status gr_program_run(gr_program* prog, void* const* leaf_ptrs, void* out_ptr) {
  if (!prog) return GR_ERR_ARG;
  gr_ctx* c = prog->ctx;
  const size_t nl = prog->leaf_bytes.size();
  if ((nl > 0 && !leaf_ptrs) || (prog->out_bytes > 0 && !out_ptr)) return fail(c, GR_ERR_ARG, "program_run: NULL pointer");
  const uintptr_t olo = (uintptr_t)out_ptr, ohi = olo + prog->out_bytes;
  for (size_t k = 0; k < nl; ++k) {
    if (!leaf_ptrs[k] && prog->leaf_bytes[k]) return fail(c, GR_ERR_ARG, "program_run: NULL input");
    const uintptr_t lo = (uintptr_t)leaf_ptrs[k], hi = lo + prog->leaf_bytes[k];
    if (lo < ohi && olo < hi) return fail(c, GR_ERR_ALIAS, "output buffer overlaps an input of the request");
  }
  for (gr_program::Launch& l : prog->launches) {
    for (const auto& pt : l.patch) l.args[pt.first] = (uint64_t)(uintptr_t)(pt.second < 0 ? out_ptr : leaf_ptrs[pt.second]);
    gr_status st = launch(c, l.fn, l.name, l.grid, l.args);
    if (st != GR_OK) return st;
  }
  return GR_OK;
}

gr_status gr_program_destroy(gr_program* prog) {
  if (!prog) return GR_ERR_ARG;
  program_free(prog->ctx, prog);
  return GR_OK;
}

gr_status gr_ctx_create(gr_ctx** out, int device, void* hip_stream) {
  if (!out) return GR_ERR_ARG;
  gr_ctx* c = new gr_ctx();
  c->device = device;
  c->stream = (hipStream_t)hip_stream;
  if (const char* pc = getenv("GR_PLAN_CACHE")) c->opt_plan_cache = atoi(pc);  // initial value of option "plan_cache"
  if (device >= 0) {
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || device >= n) {
      delete c;
      return fail(nullptr, GR_ERR_NODEVICE, "no such HIP device");
    }
    e = hipSetDevice(device);
    if (e != hipSuccess) { delete c; return fail(nullptr, GR_ERR_HIP, "hipSetDevice: " + hip_err(e)); }
    gr_status sst = static_scratch_attach(c);  // this device's copy of the static array (gr_materialize_into_static)
    if (sst != GR_OK) { delete c; return sst; }
  }
  *out = c;
  return GR_OK;
}

gr_status gr_sync(gr_ctx* ctx) {
  if (!ctx) return GR_ERR_ARG;
  if (ctx->device < 0) return GR_OK;
  GR_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return GR_OK;
}

gr_status gr_ctx_destroy(gr_ctx* ctx) {
  if (!ctx) return GR_ERR_ARG;
  if (ctx->device >= 0) (void)hipStreamSynchronize(ctx->stream);
  (void)collect_all_jobs(ctx, false);  // finished code objects go to the on-disk cache; nothing is loaded any more
  std::vector<Node*> all;
  for (auto& kv : ctx->nodes) all.push_back(kv.second);
  for (Node* n : all) {
    if (n->owns_data && n->data) ctx_free(ctx, n->data, n->alloc_bytes);
    if (n->shadow && n->shadow != n->lent) ctx_free(ctx, n->shadow, n->alloc_bytes);
    delete n;
  }
  ctx->nodes.clear();
  while (!ctx->programs.empty()) program_free(ctx, ctx->programs.back());
  if (ctx->workspace) ctx_free(ctx, ctx->workspace, ctx->workspace_bytes);
  if (ctx->scan_cells) ctx_free(ctx, ctx->scan_cells, ctx->scan_cells_bytes);
  for (auto& kv : ctx->cache) if (kv.second.module) (void)hipModuleUnload(kv.second.module);
  for (auto& p : ctx->prof) { (void)hipEventDestroy(p.e0); (void)hipEventDestroy(p.e1); }
  for (hipEvent_t e : ctx->event_pool) (void)hipEventDestroy(e);
  for (auto& kv : ctx->pool_all) (void)hipFree(kv.first);
  delete ctx;
  return GR_OK;
}

gr_status gr_compile_wait(gr_ctx* ctx) {
  if (!ctx) return GR_ERR_ARG;
  return collect_all_jobs(ctx, true);
}

gr_status gr_ctx_set_stream(gr_ctx* ctx, void* hip_stream) {
  if (!ctx) return GR_ERR_ARG;
  // buffers of the pool are reused in stream order: work queued on the old stream has to be
  // finished before another stream may touch them
  if (ctx->device >= 0 && (hipStream_t)hip_stream != ctx->stream) GR_HIP(ctx, hipStreamSynchronize(ctx->stream));
  ctx->stream = (hipStream_t)hip_stream;
  return GR_OK;
}

static bool resolves_to_data(const Node* n) {
  while (!n->materialized) {
    if (!n->is_view()) return false;
    n = n->in[0];
  }
  return true;
}

gr_status gr_materialize(gr_ctx* ctx, gr_array a) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "materialize: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "materialize: a bare scalar has no array value");
  if (resolves_to_data(x)) return GR_OK;
  if (ctx->device < 0 && !ctx->opt_dry_run) return fail(ctx, GR_ERR_NODEVICE, "context has no device");
  Plan plan;
  gr_status st = make_plan(ctx, x, &plan);
  if (st != GR_OK) return st;
  st = execute_plan(ctx, &plan, x, nullptr, true);
  clear_planned(&plan);
  return st;
}

gr_status gr_materialize_into(gr_ctx* ctx, gr_array a, void* dptr, size_t bytes) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "materialize_into: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "materialize_into: a bare scalar has no array value");
  size_t need = (size_t)x->count() * itemsize(x->dtype);
  if (bytes != need) return fail(ctx, GR_ERR_ARG, "materialize_into: buffer size does not match the array");
  if (need > 0 && !dptr) return fail(ctx, GR_ERR_ARG, "materialize_into: NULL buffer");
  if (((uintptr_t)dptr) % itemsize(x->dtype)) return fail(ctx, GR_ERR_ARG, "materialize_into: buffer not aligned to the element size");
  if (ctx->device < 0 && !ctx->opt_dry_run) return fail(ctx, GR_ERR_NODEVICE, "context has no device");
  Plan plan;
  gr_status st = make_plan(ctx, x, &plan);
  if (st != GR_OK) return st;
  st = execute_plan(ctx, &plan, x, dptr, true);
  clear_planned(&plan);
  return st;
}

}  // extern "C"

// ---- slice assignment -----------------------------------------------------------

namespace gr {

static bool resolve_view_rt(const Node* n, const Node** base, int64_t* offset, int64_t* strides) {
  if (n->materialized) {
    *base = n;
    *offset = n->offset;
    for (int d = 0; d < n->ndim; ++d) strides[d] = n->strides[d];
    return true;
  }
  if (!n->is_view()) return false;
  int64_t st[MAXD];
  if (!resolve_view_rt(n->in[0], base, offset, st)) return false;
  if (n->kind == Kind::SLICE) {
    for (int d = 0; d < n->ndim; ++d) { *offset += n->start[d] * st[d]; strides[d] = st[d] * n->step[d]; }
  } else {
    for (int d = 0; d < n->ndim; ++d) strides[d] = st[n->perm[d]];
  }
  return true;
}

static void view_extent(const Node* base, int ndim, const int64_t* shape, int64_t offset, const int64_t* strides, uintptr_t* lo, uintptr_t* hi) {
  int64_t mn = offset, mx = offset;
  for (int d = 0; d < ndim; ++d) {
    if (shape[d] == 0) { *lo = *hi = 0; return; }
    int64_t span = (shape[d] - 1) * strides[d];
    if (span < 0) mn += span; else mx += span;
  }
  *lo = (uintptr_t)base->data + mn * itemsize(base->dtype);
  *hi = (uintptr_t)base->data + (mx + 1) * itemsize(base->dtype);
}

// Does the (unevaluated) array `n` read memory in [lo, hi)?
static bool reads_range(const Node* n, uintptr_t lo, uintptr_t hi, std::set<const Node*>* seen) {
  if (!seen->insert(n).second) return false;
  if (n->materialized) {
    uintptr_t a, b;
    extent_of(n, &a, &b);
    return a < hi && lo < b;
  }
  for (const Node* p : n->in) if (reads_range(p, lo, hi, seen)) return true;
  return false;
}

// Gives a node whose data lives inside another array's storage (the result of a direct slice
// assignment) a buffer of its own.
static gr_status unshare(gr_ctx* ctx, gr_array id) {
  auto it = ctx->nodes.find(id);  // (not lookup(): the node may be held by views only, without a handle)
  Node* n = it == ctx->nodes.end() ? nullptr : it->second;
  if (!n || !n->cow_alias) return GR_OK;
  size_t bytes = (size_t)n->count() * itemsize(n->dtype);
  void* buf = ctx_alloc(ctx, bytes);
  if (!buf) return fail(ctx, GR_ERR_OOM, "allocator returned NULL");
  Plan cp;
  gr_status st = make_plan(ctx, n, &cp);  // a plain strided copy of an array that has data
  if (st == GR_OK) st = execute_plan(ctx, &cp, n, buf, false);
  clear_planned(&cp);
  if (st != GR_OK) { ctx_free(ctx, buf, bytes); return st; }
  n->data = buf; n->owns_data = true; n->alloc_bytes = bytes; n->offset = 0; n->cow_alias = false;
  int64_t sstride = 1;
  for (int k = n->ndim - 1; k >= 0; --k) { n->strides[k] = sstride; sstride *= n->shape[k]; }
  return GR_OK;
}

// Copies the box `shape` at element offset `off` (strides `strides`) from `src` to the same
// place in `dst`.
static gr_status copy_box(gr_ctx* ctx, gr_dtype dt, int nd, const int64_t* shape, const int64_t* strides, int64_t off, void* src, void* dst) {
  gr_array h = 0;
  gr_status st = gr_array_from_device(ctx, (char*)src + off * (int64_t)itemsize(dt), dt, nd, shape, strides, &h);
  if (st != GR_OK) return st;
  Node* t = lookup(ctx, h);
  OutSpec os;
  os.base = off;
  for (int k = 0; k < nd; ++k) os.strides[k] = strides[k];
  Plan wp;
  wp.out = &os;
  st = make_plan(ctx, t, &wp);
  if (st == GR_OK) st = execute_plan(ctx, &wp, t, dst, false);
  clear_planned(&wp);
  gr_release(ctx, h);
  return st;
}

// The second buffer of `b` stops mirroring it as soon as `b` is written in any other way.
static void drop_shadow(gr_ctx* ctx, Node* b) {
  if (!b->shadow) return;
  if (b->shadow != b->lent) ctx_free(ctx, b->shadow, b->alloc_bytes);  // (a lent buffer only stops being a mirror)
  b->shadow = nullptr;
}

// Is the destination a unit-step box of a C-contiguous array whose storage the library owns,
// and is the rest of that array small next to the box?  Then a value that reads the destination's
// storage at shifted positions (a stencil sweep) can be written into a second buffer, the rest
// copied over, and the two buffers swapped: half the traffic of "evaluate, then copy".
static bool swap_candidate(const Node* base, const Node* d, const OutSpec& spec, int64_t* start) {
  if ((!base->owns_data && !base->lent) || base->cow_alias || base->offset != 0 || d->ndim != base->ndim) return false;
  int64_t s = 1, rest = spec.base;
  for (int k = base->ndim - 1; k >= 0; --k) { if (base->strides[k] != s) return false; s *= base->shape[k]; }
  for (int k = 0; k < base->ndim; ++k) {
    if (spec.strides[k] != base->strides[k]) return false;
    start[k] = rest / base->strides[k];
    rest -= start[k] * base->strides[k];
    if (start[k] < 0 || start[k] + d->shape[k] > base->shape[k]) return false;
  }
  if (rest != 0) return false;
  const int64_t box = d->count(), all = base->count();
  return box > 0 && (all - box) * 4 <= box;
}

}  // namespace gr

extern "C" gr_status gr_array_lend_buffer(gr_ctx* ctx, gr_array a, void* dptr2, size_t bytes) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "lend_buffer: bad handle");
  if (x->kind != Kind::LEAF || !x->data || x->owns_data) return fail(ctx, GR_ERR_ARG, "lend_buffer: not an array made by gr_array_from_device");
  int64_t s = 1;
  for (int k = x->ndim - 1; k >= 0; --k) { if (x->shape[k] != 1 && x->strides[k] != s) return fail(ctx, GR_ERR_ARG, "lend_buffer: the array is not C-contiguous"); s *= x->shape[k]; }
  const size_t need = (size_t)x->count() * itemsize(x->dtype);
  if (x->offset != 0 || bytes != need || need == 0) return fail(ctx, GR_ERR_ARG, "lend_buffer: buffer size does not match the array");
  if (!dptr2 || ((uintptr_t)dptr2) % itemsize(x->dtype)) return fail(ctx, GR_ERR_ARG, "lend_buffer: NULL or misaligned buffer");
  const uintptr_t lo = (uintptr_t)x->data, lo2 = (uintptr_t)dptr2;
  if (lo < lo2 + need && lo2 < lo + need) return fail(ctx, GR_ERR_ALIAS, "lend_buffer: the two buffers overlap");
  drop_shadow(ctx, x);
  x->lent = dptr2;
  return GR_OK;
}

extern "C" gr_status gr_assign(gr_ctx* ctx, gr_array dst, gr_array value) {
  if (!ctx) return GR_ERR_ARG;
  Node* d = lookup(ctx, dst);
  Node* v = lookup(ctx, value);
  if (!d || !v) return fail(ctx, GR_ERR_HANDLE, "assign: bad handle");
  if (d->kind == Kind::SCALAR || v->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "assign: bare scalar operand");
  const Node* base = nullptr;
  OutSpec spec;
  if (!resolve_view_rt(d, &base, &spec.base, spec.strides)) return fail(ctx, GR_ERR_UNSUPPORTED, "assign: destination is not (a view of) a materialised array");
  if (v->dtype != d->dtype) return fail(ctx, GR_ERR_DTYPE, "assign: element types differ");
  if (v->ndim != d->ndim) return fail(ctx, GR_ERR_SHAPE, "assign: shapes differ");
  for (int k = 0; k < d->ndim; ++k) {
    if (v->shape[k] != d->shape[k]) return fail(ctx, GR_ERR_SHAPE, "assign: shapes differ");
    if (d->shape[k] > 1 && spec.strides[k] == 0) return fail(ctx, GR_ERR_UNSUPPORTED, "assign: destination elements overlap");
  }
  if (ctx->device < 0 && !ctx->opt_dry_run) return fail(ctx, GR_ERR_NODEVICE, "context has no device");
  if (d->count() == 0) return GR_OK;
  uintptr_t lo, hi;
  view_extent(base, d->ndim, d->shape, spec.base, spec.strides, &lo, &hi);

  // 1. Arrays recorded earlier that read this storage keep the values they had when recorded:
  //    evaluate them now.  Results of earlier direct assignments that still live inside this
  //    storage get their own copy.
  std::vector<gr_array> pending, aliases;
  for (auto& kv : ctx->nodes) {
    Node* n = kv.second;
    if (n == v || n->kind == Kind::SCALAR) continue;
    if (n->materialized) {
      // (also one that only views refer to: the destination itself may be a view of it)
      if (n->cow_alias) { uintptr_t a, b; extent_of(n, &a, &b); if (a < hi && lo < b) aliases.push_back(n->id); }
      continue;
    }
    if (n->handle_refs <= 0) continue;
    if (n->is_view()) { const Node* vb; int64_t o, st[MAXD]; if (resolve_view_rt(n, &vb, &o, st)) continue; }  // aliases see the new contents
    std::set<const Node*> seen;
    if (reads_range(n, lo, hi, &seen)) pending.push_back(n->id);
  }
  for (gr_array id : pending) {
    gr_status st = gr_materialize(ctx, id);
    if (st != GR_OK) return st;
  }
  for (gr_array id : aliases) {
    gr_status st = unshare(ctx, id);
    if (st != GR_OK) return st;
  }
  v = lookup(ctx, value);
  if (!v) return fail(ctx, GR_ERR_HANDLE, "assign: value handle vanished");

  // 2. Can one fused kernel write the destination directly?  Only if the value is still
  //    unevaluated, its last sub-graph is a map, and that sub-graph reads the destination's
  //    storage at exactly the positions it writes (or not at all).
  bool direct = false;
  // (the destination's own base may just have moved to a buffer of its own)
  resolve_view_rt(d, &base, &spec.base, spec.strides);
  view_extent(base, d->ndim, d->shape, spec.base, spec.strides, &lo, &hi);
  const Node* vb = nullptr; int64_t vo, vst[MAXD];
  const bool value_has_data = resolve_view_rt(v, &vb, &vo, vst);
  if (!value_has_data) {
    Plan plan;
    plan.out = &spec;
    gr_status st = make_plan(ctx, v, &plan);
    if (st != GR_OK) return st;
    bool safe = plan.out_honoured;
    if (safe) {
      const GroupPlan& g = *plan.groups.back();
      for (const AccessGroup& ag : g.groups) {
        if (!ag.leaf->materialized) continue;
        uintptr_t a, b;
        extent_of(ag.leaf, &a, &b);
        if (!(a < hi && lo < b)) continue;
        bool same = ag.leaf->data == base->data && ag.base == g.out_base && ag.deltas.size() == 1;
        for (int k = 0; same && k < g.rank; ++k) if (ag.coef[k] != g.out_coef[k]) same = false;
        if (!same) safe = false;
      }
      // earlier sub-graphs of the plan finish before the last one starts: no hazard there
    }
    int64_t start[MAXD];
    if (safe) {
      drop_shadow(ctx, const_cast<Node*>(base));
      st = execute_plan(ctx, &plan, v, base->data, false);
      clear_planned(&plan);
      if (st != GR_OK) return st;
      direct = true;
    } else if (ctx->opt_assign_swap && plan.out_honoured && swap_candidate(base, d, spec, start)) {
      // 2b. The value reads the destination's storage where it does not write it (a stencil sweep).
      //     Write it into a second buffer, copy the cells outside the destination, swap the buffers:
      //     views resolve through the owning node, so they all see the new storage.
      clear_planned(&plan);
      Node* b = const_cast<Node*>(base);
      std::vector<gr_array> inside;
      for (auto& kv : ctx->nodes)
        if (kv.second->materialized && kv.second->cow_alias && kv.second->data == b->data) inside.push_back(kv.first);
      for (gr_array id : inside) {
        st = unshare(ctx, id);
        if (st != GR_OK) return st;
      }
      v = lookup(ctx, value);
      if (!v) return fail(ctx, GR_ERR_HANDLE, "assign: value handle vanished");
      const size_t bytes = (size_t)b->count() * itemsize(b->dtype);
      // the buffer this array was swapped out of by the last sweep over the same box already holds
      // the cells outside the box: nothing to copy
      bool mirrored = b->shadow != nullptr && (b->shadow == b->lent || bytes == b->alloc_bytes);
      for (int k = 0; mirrored && k < b->ndim; ++k) mirrored = b->shadow_start[k] == start[k] && b->shadow_len[k] == d->shape[k];
      if (!mirrored) drop_shadow(ctx, b);
      // the second buffer: the mirror left by the last sweep, else the buffer the caller lent, else a new one
      void* fresh = mirrored ? b->shadow : (b->lent ? b->lent : ctx_alloc(ctx, bytes));
      if (!fresh) return fail(ctx, GR_ERR_OOM, "allocator returned NULL");
      b->shadow = nullptr;
      Plan p2;
      p2.out = &spec;
      st = make_plan(ctx, v, &p2);
      if (st == GR_OK && !p2.out_honoured) st = fail(ctx, GR_ERR_UNSUPPORTED, "assign: plan changed between two passes");
      if (st == GR_OK) st = execute_plan(ctx, &p2, v, fresh, false);
      clear_planned(&p2);
      // the cells around the box: per dimension a slab below and a slab above it
      int64_t shp[MAXD], off = 0;
      for (int k = 0; k < b->ndim; ++k) shp[k] = b->shape[k];
      for (int k = 0; st == GR_OK && !mirrored && k < b->ndim; ++k) {
        const int64_t lo_n = start[k], hi_n = b->shape[k] - (start[k] + d->shape[k]);
        if (lo_n > 0) { shp[k] = lo_n; st = copy_box(ctx, b->dtype, b->ndim, shp, b->strides, off, b->data, fresh); }
        if (st == GR_OK && hi_n > 0) {
          shp[k] = hi_n;
          st = copy_box(ctx, b->dtype, b->ndim, shp, b->strides, off + (start[k] + d->shape[k]) * b->strides[k], b->data, fresh);
        }
        shp[k] = d->shape[k];
        off += start[k] * b->strides[k];
      }
      if (st != GR_OK) {
        // the value may already be bound to the abandoned buffer: give it a buffer of its own first
        v = lookup(ctx, value);
        if (v && v->materialized && v->cow_alias && v->data == fresh) (void)unshare(ctx, value);
        if (fresh != b->lent) ctx_free(ctx, fresh, bytes);
        return st;
      }
      // the old buffer becomes the mirror: outside the box it equals the new one
      if (b->lent) b->lent = b->data;  // the caller's two buffers trade places
      b->shadow = b->data;
      b->data = fresh;
      for (int k = 0; k < b->ndim; ++k) { b->shadow_start[k] = start[k]; b->shadow_len[k] = d->shape[k]; }
      ctx->stats.assign_swaps++;
      direct = true;
    } else {
      clear_planned(&plan);
    }
  }
  if (direct) return GR_OK;

  // 3. General case (NumPy's own cost model): finish the value in its own buffer, then copy.
  drop_shadow(ctx, const_cast<Node*>(base));
  if (!value_has_data) {
    gr_status st = gr_materialize(ctx, value);
    if (st != GR_OK) return st;
    v = lookup(ctx, value);
  } else {
    // the value is an alias of materialised data; if it overlaps the destination it is
    // copied to a temporary first (overlapping source and destination)
    uintptr_t a, b;
    view_extent(vb, v->ndim, v->shape, vo, vst, &a, &b);
    if (a < hi && lo < b) {
      size_t bytes = (size_t)v->count() * itemsize(v->dtype);
      void* buf = ctx_alloc(ctx, bytes);
      if (!buf) return fail(ctx, GR_ERR_OOM, "allocator returned NULL");
      Plan cp;
      gr_status st = make_plan(ctx, v, &cp);
      if (st == GR_OK) st = execute_plan(ctx, &cp, v, buf, false);
      clear_planned(&cp);
      if (st != GR_OK) { ctx_free(ctx, buf, bytes); return st; }
      // copy tmp -> destination through a temporary leaf node
      gr_array tmp_h = 0;
      st = gr_array_from_device(ctx, buf, v->dtype, v->ndim, v->shape, nullptr, &tmp_h);
      if (st != GR_OK) { ctx_free(ctx, buf, bytes); return st; }
      Node* t = lookup(ctx, tmp_h);
      Plan wp;
      wp.out = &spec;
      st = make_plan(ctx, t, &wp);
      if (st == GR_OK) st = execute_plan(ctx, &wp, t, base->data, false);
      clear_planned(&wp);
      gr_release(ctx, tmp_h);
      ctx_free(ctx, buf, bytes);  // stream order: the copy kernel is already queued before any reuse
      return st;
    }
  }
  Plan wp;
  wp.out = &spec;
  gr_status st = make_plan(ctx, v, &wp);
  if (st == GR_OK) st = execute_plan(ctx, &wp, v, base->data, false);
  clear_planned(&wp);
  return st;
}

extern "C" {

static gr_status copy_out(const std::string& s, char* buf, size_t cap, size_t* needed) {
  if (needed) *needed = s.size() + 1;
  if (buf && cap) {
    size_t n = std::min(cap - 1, s.size());
    std::memcpy(buf, s.data(), n);
    buf[n] = '\0';
  }
  return GR_OK;
}

gr_status gr_plan_describe(gr_ctx* ctx, gr_array a, char* buf, size_t cap, size_t* needed) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "plan_describe: bad handle");
  Plan plan;
  gr_status st = make_plan(ctx, x, &plan);
  if (st != GR_OK) return st;
  std::string s = describe_plan(plan);
  clear_planned(&plan);
  return copy_out(s, buf, cap, needed);
}

gr_status gr_plan_source(gr_ctx* ctx, gr_array a, int index, char* buf, size_t cap, size_t* needed) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "plan_source: bad handle");
  Plan plan;
  gr_status st = make_plan(ctx, x, &plan);
  if (st != GR_OK) return st;
  if (index < 0 || index >= (int)plan.groups.size()) { clear_planned(&plan); return fail(ctx, GR_ERR_ARG, "plan_source: no such sub-graph"); }
  st = expand_patch(ctx, plan.groups[index].get());
  if (st != GR_OK) { clear_planned(&plan); return st; }
  std::string s = generate_source(*plan.groups[index]);
  clear_planned(&plan);
  return copy_out(s, buf, cap, needed);
}

gr_status gr_plan_compile(gr_ctx* ctx, gr_array a) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "plan_compile: bad handle");
  // twice: as gr_materialize would plan the request, and as the entry point that must not allocate would (the planner
  // then keeps optional partial results within the static scratch array, which can select other kernels)
  gr_status st = GR_OK;
  std::string first;
  for (int pass = 0; pass < 2 && st == GR_OK; ++pass) {
    Plan plan;
    ctx->plan_static = pass == 1;
    st = make_plan(ctx, x, &plan);
    ctx->plan_static = false;
    if (st != GR_OK) return st;
    const std::string text = describe_plan(plan);
    if (pass == 0) first = text;
    else if (text == first) { clear_planned(&plan); break; }   // the same plan: nothing more to compile
    for (auto& g : plan.groups) {
      st = prepare_group(ctx, *g);
      if (st != GR_OK) break;
    }
    for (auto& g : plan.groups) {
      if (st != GR_OK) break;
      gr_ctx::Kernel* k = nullptr;
      st = compile_group(ctx, *g, &k);
    }
    clear_planned(&plan);
  }
  return st;
}

gr_status gr_profile_reset(gr_ctx* ctx) {
  if (!ctx) return GR_ERR_ARG;
  if (ctx->device >= 0 && !ctx->prof.empty()) GR_HIP(ctx, hipStreamSynchronize(ctx->stream));
  for (auto& p : ctx->prof) { ctx->event_pool.push_back(p.e0); ctx->event_pool.push_back(p.e1); }
  ctx->prof.clear();
  return GR_OK;
}

gr_status gr_profile_read(gr_ctx* ctx, const char* prefix, uint64_t* launches, double* total_ms) {
  if (!ctx || !launches || !total_ms) return GR_ERR_ARG;
  std::string pre(prefix ? prefix : "");
  *launches = 0;
  *total_ms = 0.0;
  if (ctx->device >= 0) GR_HIP(ctx, hipStreamSynchronize(ctx->stream));
  for (auto& p : ctx->prof) {
    if (p.name.compare(0, pre.size(), pre) != 0) continue;
    float ms = 0.f;
    GR_HIP(ctx, hipEventElapsedTime(&ms, p.e0, p.e1));
    *launches += 1;
    *total_ms += ms;
  }
  return GR_OK;
}

gr_status gr_stream_copy(gr_ctx* ctx, void* dst, const void* src, size_t bytes) {
  if (!ctx || !dst || !src) return GR_ERR_ARG;
  if (ctx->device < 0) return fail(ctx, GR_ERR_NODEVICE, "context has no device");
  if (bytes % 16 || ((uintptr_t)dst % 16) || ((uintptr_t)src % 16)) return fail(ctx, GR_ERR_ARG, "stream_copy: size and pointers must be multiples of 16");
  uintptr_t d = (uintptr_t)dst, s = (uintptr_t)src;
  if (d < s + bytes && s < d + bytes) return fail(ctx, GR_ERR_ALIAS, "stream_copy: buffers overlap");
  if (bytes == 0) return GR_OK;
  gr_launch_stream_copy(ctx->stream, dst, src, bytes / 16);
  GR_HIP(ctx, hipGetLastError());
  return GR_OK;
}

gr_status gr_stream_read(gr_ctx* ctx, const void* src, size_t bytes, void* sink) {
  if (!ctx || !src || !sink) return GR_ERR_ARG;
  if (ctx->device < 0) return fail(ctx, GR_ERR_NODEVICE, "context has no device");
  if (bytes % 16 || ((uintptr_t)src % 16) || ((uintptr_t)sink % 4)) return fail(ctx, GR_ERR_ARG, "stream_read: size and pointer must be multiples of 16");
  if (bytes == 0) return GR_OK;
  gr_launch_stream_read(ctx->stream, src, bytes / 16, sink);
  GR_HIP(ctx, hipGetLastError());
  return GR_OK;
}

}  // extern "C"
