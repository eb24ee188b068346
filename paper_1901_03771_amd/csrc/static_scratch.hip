// gr_materialize_into_static: gr_materialize_into for callers that cannot allocate device
// memory (code under HIP graph capture, tight serving loops, harnesses that forbid it).
// Everything such a request needs beyond the caller's inputs and output -- the stored results
// of earlier sub-graphs and the first-stage partial results of two-stage kernels -- comes from
// one file-scope device array; every GPU the library runs on holds its own copy of the array,
// at its own address, until the process ends.
#include <hip/hip_runtime.h>

#include <mutex>

#include "ctx.h"

#define GR_STATIC_SCRATCH_BYTES (16u << 20)

// In host code this name is only a stand-in for the device symbol, never a device address:
// host code below uses the per-device address obtained from hipGetSymbolAddress.  (The symbol
// lookup is by name: the compiler gives a file-scope static device variable a global symbol in
// the code object because host code refers to it; attribute "used" would keep the symbol local
// and the lookup would fail.)
static __device__ __align__(256) unsigned char scratch[GR_STATIC_SCRATCH_BYTES];

namespace gr {

static std::mutex g_lock;
static constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];  // per device: address of that device's copy of `scratch`

// Called by gr_ctx_create with the context's device current: looks the array's address on that
// device up once and keeps it.
gr_status static_scratch_attach(gr_ctx* c) {
  if (c->device < 0) return GR_OK;
  if (c->device >= kMaxDevices) return fail(nullptr, GR_ERR_ARG, "device index beyond the static scratch table");
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_ptr[c->device]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(nullptr, GR_ERR_HIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorName(e) + ": " + hipGetErrorString(e));
    g_scratch_ptr[c->device] = ptr;
  }
  c->static_base = (unsigned char*)g_scratch_ptr[c->device];
  c->static_cap = GR_STATIC_SCRATCH_BYTES;
  return GR_OK;
}

}  // namespace gr

using namespace gr;

extern "C" gr_status gr_static_scratch_bytes(size_t* bytes) {
  if (!bytes) return GR_ERR_ARG;
  *bytes = GR_STATIC_SCRATCH_BYTES;
  return GR_OK;
}

extern "C" gr_status gr_materialize_into_static(gr_ctx* ctx, gr_array a, void* dptr, size_t bytes) {
  if (!ctx) return GR_ERR_ARG;
  Node* x = lookup(ctx, a);
  if (!x) return fail(ctx, GR_ERR_HANDLE, "materialize_into_static: bad handle");
  if (x->kind == Kind::SCALAR) return fail(ctx, GR_ERR_UNSUPPORTED, "materialize_into_static: a bare scalar has no array value");
  size_t need = (size_t)x->count() * itemsize(x->dtype);
  if (bytes != need) return fail(ctx, GR_ERR_ARG, "materialize_into_static: buffer size does not match the array");
  if (need > 0 && !dptr) return fail(ctx, GR_ERR_ARG, "materialize_into_static: NULL buffer");
  if (((uintptr_t)dptr) % itemsize(x->dtype)) return fail(ctx, GR_ERR_ARG, "materialize_into_static: buffer not aligned to the element size");
  if (ctx->device < 0 && !ctx->opt_dry_run) return fail(ctx, GR_ERR_NODEVICE, "context has no device");
  if (ctx->device < 0) {
    // dry run on a device-less context: an address range that nothing ever dereferences
    ctx->static_base = (unsigned char*)(uintptr_t)0x7f0000000000ull;
    ctx->static_cap = GR_STATIC_SCRATCH_BYTES;
  }
  if (!ctx->static_base) return fail(ctx, GR_ERR_HIP, "materialize_into_static: the static scratch array has no address on this device");
  Plan plan;  // (host memory only)
  ctx->plan_static = true;
  gr_status st = make_plan(ctx, x, &plan);
  ctx->plan_static = false;
  if (st != GR_OK) return st;
  ctx->static_mode = true;
  ctx->static_used = 0;  // every call starts at the beginning of the array: calls that overlap on one GPU race
  st = execute_plan(ctx, &plan, x, dptr, true);
  ctx->static_mode = false;
  clear_planned(&plan);
  return st;
}
