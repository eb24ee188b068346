/*
 * grumpy_hip.h -- C ABI of the fused lazy-array evaluator for MI355X (gfx950).
 *
 * The calls follow the paper's statement of the problem (arxiv 1901.03771):
 *   - an array handle is one node of the DAG G=(V,E)              (Section 2)
 *   - input arrays enter as materialised leaves                    (Section 2, Section 4.1)
 *   - every operation is recorded, not executed; shape and element type of
 *     the result are inferred with NumPy semantics, broadcast included
 *                                                                  (Section 1, Section 2)
 *   - values are produced when asked for: the DAG is walked back to the
 *     materialised nodes, split into an ordered list of sub-graphs
 *     (Algorithm 1), and each sub-graph runs as one fused kernel whose point
 *     function translates output indices back to leaf indices
 *                                                                  (Section 2, Section 3.1, Section 3.2)
 *   - the computed node then stays materialised and is a leaf of every
 *     later request                                                (Section 2)
 *
 * Conventions
 *   - Every function returns a gr_status (0 = GR_OK).  On error nothing is
 *     recorded, *out is untouched, and gr_last_error(ctx) describes it.
 *   - "device pointer" = address in the memory of the context's GPU.
 *     "host pointer" = ordinary process memory.  All shape / stride / axis
 *     arguments are host pointers and are copied before the call returns.
 *   - Strides and offsets count ELEMENTS, not bytes.
 *   - Recording calls never touch the device.  Kernels are launched
 *     asynchronously on the context's stream by gr_materialize* and
 *     gr_assign; the library only waits inside gr_sync, gr_ctx_set_stream
 *     and gr_ctx_destroy (and where its default pool hands memory back to
 *     the device, see option "pool_limit").
 *   - A context is not thread-safe.
 *   - Supported element types: f32 and i32 for computation; i64 only as the
 *     result of an i32 sum (NumPy's default on Linux).  Mixed i32/f32
 *     arithmetic would promote to f64 in NumPy and is refused
 *     (GR_ERR_DTYPE).
 */
#ifndef GRUMPY_HIP_H
#define GRUMPY_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gr_ctx gr_ctx;
typedef uint64_t gr_array; /* opaque node id; 0 is never a valid handle */

typedef enum {
  GR_OK = 0,
  GR_ERR_HANDLE = 1,      /* unknown or released handle */
  GR_ERR_SHAPE = 2,       /* shapes do not broadcast / inner dimensions differ */
  GR_ERR_DTYPE = 3,       /* element types not combinable without f64 */
  GR_ERR_AXIS = 4,        /* axis out of range or repeated */
  GR_ERR_UNSUPPORTED = 5, /* valid NumPy, outside this library's vocabulary */
  GR_ERR_ARG = 6,         /* NULL pointer, bad rank, bad enum, bad size */
  GR_ERR_COMPILE = 7,     /* run-time compilation of a fused kernel failed */
  GR_ERR_HIP = 8,         /* a HIP runtime call failed */
  GR_ERR_OOM = 9,         /* the allocator returned NULL */
  GR_ERR_ALIAS = 10,      /* output buffer overlaps an input of the request */
  GR_ERR_NODEVICE = 11    /* context was created without a device */
} gr_status;

typedef enum { GR_F32 = 0, GR_I32 = 1, GR_I64 = 2 } gr_dtype;

typedef enum {
  /* unary (Section 1 / Section 2: pointwise NumPy operations) */
  GR_NEG = 0, GR_ABS = 1, GR_EXP = 2, GR_LOG = 3, GR_SQRT = 4, GR_SQUARE = 5, GR_TANH = 6, GR_ERF = 7,
  /* binary, NumPy broadcasting */
  GR_ADD = 16, GR_SUB = 17, GR_MUL = 18, GR_DIV = 19, GR_MAXIMUM = 20, GR_MINIMUM = 21,
  GR_POW_INT = 22, /* array ** integer scalar: only the exponent 2 (recorded as GR_SQUARE, as NumPy evaluates x**2); anything else GR_ERR_UNSUPPORTED */
  /* reductions (Section 3.2: associative and commutative binary operator) */
  GR_SUM = 32, GR_MAX = 33, GR_MIN = 34
} gr_op;

#define GR_MAX_NDIM 8

/* ---- context ------------------------------------------------------------ */

/* Creates a context bound to HIP device `device` and to `hip_stream`
 * (a hipStream_t passed as void*, borrowed; NULL = the default stream).
 * device = -1 creates a device-less context: recording, partitioning and
 * code generation work, gr_materialize* return GR_ERR_NODEVICE. */
gr_status gr_ctx_create(gr_ctx** out, int device, void* hip_stream);

/* Waits for the stream, releases every node, buffer, module and workspace
 * the context owns.  Borrowed leaf buffers are not freed. */
gr_status gr_ctx_destroy(gr_ctx* ctx);

/* Replaces the stream later launches go to (borrowed).  Waits for the work
 * already queued on the old stream: the context reuses its buffers in stream
 * order. */
gr_status gr_ctx_set_stream(gr_ctx* ctx, void* hip_stream);

/* Installs the device allocator used for materialised results and
 * workspaces.  alloc(bytes, user) returns a device pointer aligned to at
 * least 256 bytes or NULL; free_(ptr, user) releases it.  Both may be called
 * from any library call.  Default: a grow-only pool over hipMalloc that is
 * emptied by gr_ctx_destroy. */
gr_status gr_ctx_set_allocator(gr_ctx* ctx, void* (*alloc)(size_t bytes, void* user),
                               void (*free_)(void* ptr, void* user), void* user);

/* Integer options (host string key).  The keys below change WHAT the library does; keys that only
 * tune HOW a kernel is scheduled (patch sizes, lanes per row, slab counts, tile shapes, thresholds)
 * are listed in grumpy_hip_tuning.h and go through the same call.
 *   "fusion"          1 (default) fuse per Algorithm 1 as relaxed below; 0 =
 *                     one kernel per recorded op, every intermediate stored
 *                     (the eager execution model the paper starts from)
 *   "rowred_max_cols" longest row (elements) a reduction may keep resident
 *                     in registers and still fuse with its consumers
 *   "gemv_pair"       1 (default) = a contraction A.v whose epilogue result r
 *                     feeds the contraction A^T.r runs with it in one pass
 *                     over A; 0 = two passes
 *   "async_compile"   1 (default) = the kernels of all sub-graphs of a request
 *                     are compiled concurrently on host threads while earlier
 *                     sub-graphs already run (compilation overlapped with
 *                     execution, Section 6 of the paper); 0 = one after another
 *   "disk_cache"      1 (default) = compiled code objects are kept in
 *                     $GR_CACHE_DIR (default ~/.cache/grumpy_hip) keyed on
 *                     the generated kernel source (and compiler version and
 *                     flags), so another build of the library never reads
 *                     them by mistake.  A miss there is looked up in the
 *                     kernel pack next: the directory "kernel_pack" beside
 *                     the shared library (or $GR_KERNEL_PACK; empty = none),
 *                     same file format, written at build time for common
 *                     sub-graphs, never written at run time.
 *                     0 = in-memory cache only, no pack
 *   "interp"          1 (default) = a sub-graph whose kernel is still in the
 *                     run-time compiler is evaluated by a precompiled byte-code
 *                     interpreter of the point function instead of waiting (f32 /
 *                     i32 programs within fixed size limits: maps, row-resident
 *                     reductions, reductions over any axes, scans, contractions
 *                     with their epilogues; everything else waits as with 0).
 *                     Maps and row-resident reductions give the bits of the
 *                     compiled kernel; a float sum of the other kinds is
 *                     associated differently (integer, max and min results are
 *                     exact).  The compilation goes on in the background and
 *                     later requests use the compiled kernel; 0 = always wait for
 *                     the compiler; 2 = interpret every sub-graph the
 *                     interpreter covers (for testing it)
 *   "assign_swap"     1 (default) = gr_assign of a value that reads the
 *                     destination's storage at shifted positions (a stencil
 *                     sweep), into a unit-step box that covers at least 4/5 of
 *                     an array whose storage the library owns, writes a second
 *                     buffer, copies the cells outside the box and swaps the
 *                     two buffers; 0 = always evaluate, then copy
 *   "pool_limit"      bytes the default pool may hold before a request for a size
 *                     it has no free block of makes it return its free blocks of
 *                     other sizes to the device first; 0 (default) = no limit
 *                     (the same happens whenever the device runs out of memory)
 *   "plan_cache"      1 (default) = a request whose sub-DAG has the structure of an
 *                     earlier one (node kinds, shapes, strides of stored arrays,
 *                     slice bounds, scalar values, sharing of operands, recording
 *                     order) reuses that request's partition and index maps
 *                     instead of planning again (iterative programs record the
 *                     same expression every sweep); 0 = plan every request;
 *                     2 = reuse, but also plan afresh and fail the request
 *                     (GR_ERR_UNSUPPORTED) if the two plans differ (self-check);
 *                     the environment variable GR_PLAN_CACHE gives the value a
 *                     new context starts with
 *   "dry_run"         on a device-less context only: 1 = materialise and assign
 *                     calls run everything except the kernel launches
 *                     (partitioning, code generation, compilation, buffer and
 *                     node bookkeeping; buffers get addresses that are never
 *                     dereferenced), so the host logic can be exercised
 *                     without a GPU; 2 = the same without compiling; 0
 *                     (default) = such calls return GR_ERR_NODEVICE
 *   "merge"           1 (default) = a reduction, scan or contraction recorded
 *                     while a node with the same pending expression is still
 *                     waiting to be evaluated returns a handle to that node
 *                     (common subexpressions, Section 5 of the paper); the two
 *                     handles then share value and storage; 0 = never
 *   "profile"         1 = bracket every launch with HIP events (gr_profile_*)
 * Unknown key: GR_ERR_ARG. */
gr_status gr_ctx_set_option(gr_ctx* ctx, const char* key, int64_t value);

/* Blocks until all work launched by this context has finished. */
gr_status gr_sync(gr_ctx* ctx);

/* Text of the last error of this context ("" if none).  The pointer stays
 * valid until the next failing call on the context.  ctx = NULL returns the
 * text of the last failed gr_ctx_create. */
const char* gr_last_error(gr_ctx* ctx);

/* ---- leaves (Section 2: when recording starts, inputs are the only nodes that hold values) */

/* Wraps an existing device buffer as a materialised leaf.  `dptr` points at
 * element (0,..,0); strides_elems = NULL means C-contiguous.  BORROWED: the
 * caller keeps the memory alive and unmodified until every array that
 * depends on this leaf has been materialised or released.
 * Limits (GR_ERR_ARG): the product of the non-zero extents, and the largest
 * element offset the strides reach, stay at or below 2^40; `dptr` is aligned
 * to the element size.  Results that would exceed 2^40 elements (a broadcast,
 * an outer-product-like dot, a reshape) are refused with GR_ERR_SHAPE. */
gr_status gr_array_from_device(gr_ctx* ctx, void* dptr, gr_dtype dtype, int ndim, const int64_t* shape,
                               const int64_t* strides_elems, gr_array* out);

/* Lends the library a second device buffer for `a`, a C-contiguous array made by gr_array_from_device, of
 * the same size (`bytes` = count * itemsize, not overlapping the first).  A slice assignment whose value reads
 * the array's storage at shifted positions -- a stencil sweep, Listing 6 of the paper -- into a unit-step box
 * covering at least 4/5 of the array then writes the new contents into the other of the two buffers, copies the
 * cells outside the box once, and makes that buffer the array's storage: 8 bytes per element and sweep instead
 * of the 16 of "evaluate into a temporary, copy back" (which remains what happens to wrapped memory without a
 * second buffer).  From then on the array's contents are in ONE of the two buffers: gr_data_ptr says which
 * after every assignment; the other holds the previous sweep's cells.  Both stay borrowed (never freed by the
 * library) and must stay alive as long as the array. */
gr_status gr_array_lend_buffer(gr_ctx* ctx, gr_array a, void* dptr2, size_t bytes);

/* A Python-style number.  It has no element type of its own: in a binary op
 * it takes the array operand's type (rounded to binary32 first when it meets
 * f32; an integer-valued one may meet i32; a fractional one with i32 is
 * GR_ERR_DTYPE).  It cannot be materialised. */
gr_status gr_scalar(gr_ctx* ctx, double value, int is_integer, gr_array* out);

/* ---- recording (Section 2: nodes with is_materialized = false) ---------- */

gr_status gr_unary(gr_ctx* ctx, gr_op op, gr_array a, gr_array* out);
gr_status gr_binary(gr_ctx* ctx, gr_op op, gr_array a, gr_array b, gr_array* out);

/* gr_binary with a Python-style number as one operand, in one call:
 * scalar_on_left = 0 records op(a, value), 1 records op(value, a).  Same
 * typing rule and errors as gr_scalar followed by gr_binary. */
gr_status gr_binary_scalar(gr_ctx* ctx, gr_op op, gr_array a, double value, int is_integer, int scalar_on_left,
                           gr_array* out);

/* Basic slicing with Python rules on the first `nspec` dimensions (step >= 1;
 * has_start/has_stop = 0 mean "omitted"); the rest are taken whole.  The
 * result is a view: an index transformation, no data is moved (Section 3.1). */
gr_status gr_slice(gr_ctx* ctx, gr_array a, int nspec, const int64_t* start, const int64_t* stop,
                   const int64_t* step, const uint8_t* has_start, const uint8_t* has_stop, gr_array* out);

/* Axis permutation as a view; perm = NULL reverses the axes, so element
 * (i,j) of the result is element (j,i) of a 2-D operand (Section 3.1). */
gr_status gr_transpose(gr_ctx* ctx, gr_array a, const int* perm, gr_array* out);

/* Reshape (Section 2 lists it with the n-D transpose among the recorded
 * operations): the elements of `a` in row-major order under the new shape
 * (host array of `ndim` extents with the same product; one extent may be -1 and
 * is then inferred).  The result is an array of its own: evaluating it copies
 * (fused with whatever pointwise expression `a` still is), so writes through it
 * never reach `a` (NumPy returns a view where it can; values are the same).
 * Consumers read the stored result.  GR_ERR_SHAPE if the counts differ. */
gr_status gr_reshape(gr_ctx* ctx, gr_array a, int ndim, const int64_t* shape, gr_array* out);

/* GR_SUM / GR_MAX / GR_MIN over `axes` (naxes = 0: all axes).  Negative axes
 * count from the end.  i32 sums give i64.  max/min over an empty range:
 * GR_ERR_SHAPE. */
gr_status gr_reduce(gr_ctx* ctx, gr_op op, gr_array a, const int* axes, int naxes, int keepdims, gr_array* out);

/* Inclusive scan along one axis (the map-scan primitive of Section 3.2):
 * GR_SUM = np.cumsum, GR_MAX / GR_MIN = np.maximum/minimum.accumulate.  The
 * result has the operand's shape; an i32 running sum gives i64.  A scan is a
 * fusion boundary on its output side: its operand expression is fused into the
 * scan kernel, its consumers read the stored result. */
gr_status gr_scan(gr_ctx* ctx, gr_op op, gr_array a, int axis, gr_array* out);

/* np.dot for f32: (M,K).(K,N) -> (M,N), (M,K).(K,) -> (M,) and (K,).(K,) -> ().
 * Either operand may be any strided view (a transposed matrix is folded into
 * the kernel, Section 2).  Operands are materialised first; pointwise consumers
 * of the same shape run as the contraction kernel's epilogue.  The matrix-matrix
 * product runs on the matrix cores (MFMA, f32 inputs and accumulation). */
gr_status gr_dot(gr_ctx* ctx, gr_array a, gr_array b, gr_array* out);

/* ---- materialisation (Section 2, Algorithm 1, Section 3) ---------------- */

/* Computes `a` into memory obtained from the context's allocator; the buffer
 * belongs to the node and is freed when the node dies. */
gr_status gr_materialize(gr_ctx* ctx, gr_array a);

/* Computes `a` into the caller's C-contiguous device buffer of `bytes` bytes
 * (must equal count * itemsize).  The buffer must not overlap any leaf the
 * request reads (GR_ERR_ALIAS) and stays owned by the caller, who keeps it
 * alive while the node or anything recorded on top of it is in use.  An array
 * that already has data, or a view of one, is copied: it keeps its own storage
 * (a view stays a view of its base) and no reference to `dptr` is kept. */
gr_status gr_materialize_into(gr_ctx* ctx, gr_array a, void* dptr, size_t bytes);

/* gr_materialize_into for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result and
 * errors as gr_materialize_into, and the same kernels; the call itself allocates and frees no
 * device memory and calls no allocating library routine (the context's allocator callbacks are
 * not called for anything the request needs).
 *   - Everything the request needs beyond its leaves and `dptr` -- the stored results of
 *     earlier sub-graphs of the request, the first-stage partial results of two-stage kernels
 *     (reductions split over workgroups, chunked scans, column-accumulate and one-pass
 *     contractions, split-K matrix products) -- lives in one static device array of
 *     gr_static_scratch_bytes() = 16 MiB inside the library (every GPU the library runs on
 *     holds its own copy until the process ends).  A request that needs more is refused with
 *     GR_ERR_OOM before anything is launched; the message names both sizes.
 *   - Every kernel of the request must already be loaded on this context (loading a code
 *     object allocates): call gr_plan_compile(ctx, a) once beforehand.  Evaluating a request
 *     of the same structure with gr_materialize / gr_materialize_into also serves, unless the
 *     planner picks other kernels when partial results have to fit the static array (a matrix
 *     product whose K it would otherwise divide over more workgroups than fit).  Otherwise
 *     GR_ERR_UNSUPPORTED, nothing launched.  Option "profile" is ignored by this call.
 *   - Results of earlier sub-graphs exist only while the request runs: after the call those
 *     arrays are unevaluated again (and can be evaluated later); only `a` keeps its value, in
 *     `dptr`, as with gr_materialize_into.  Arrays that lose their last reference during the
 *     call are released as usual (the default pool keeps their blocks; an installed free
 *     callback is called for them).
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents;
 *     nothing in it needs to start at zero (every partial result is written before it is
 *     read).  Calls that overlap on one GPU -- two contexts, or two streams -- race. */
gr_status gr_materialize_into_static(gr_ctx* ctx, gr_array a, void* dptr, size_t bytes);

/* Size in bytes of the static device array behind gr_materialize_into_static. */
gr_status gr_static_scratch_bytes(size_t* bytes);

/* ---- record once, run many times (Section 4.2, Section 6: at small array sizes the time goes into
 * everything around the kernels -- recording, partitioning, code generation -- not into the kernels) */

typedef struct gr_program gr_program;

/* Prepares the evaluation of `root` for replay.  The DAG below `root` is partitioned as for
 * gr_materialize_into (Algorithm 1), its kernels are compiled and loaded, buffers for the stored
 * results of earlier sub-graphs and for partial results are allocated (the program owns them),
 * and the launches are written down with their arguments; nothing runs and no node changes.
 * `leaves` (host array of `nleaves` handles made by gr_array_from_device, each at most once) are
 * the inputs a run may rebind; every other stored array the request reads stays bound to the
 * address it has now and must stay alive while the program is used.  The program belongs to the
 * context and dies with it at the latest. */
gr_status gr_program_create(gr_ctx* ctx, gr_array root, const gr_array* leaves, int nleaves, gr_program** out);

/* Evaluates the recorded request on new data: leaf_ptrs (host array, one device pointer per
 * rebindable leaf, in the order given to gr_program_create) point at arrays of the same element
 * type, shape and strides as the leaves the program was made from; the result is written to the
 * C-contiguous device buffer out_ptr (GR_ERR_ALIAS if it overlaps an input).  Launches only:
 * asynchronous on the context's stream, no planning, no allocation, no node is touched.  Runs
 * of one program are ordered by the stream; its internal buffers make concurrent runs on
 * different streams unsafe. */
gr_status gr_program_run(gr_program* prog, void* const* leaf_ptrs, void* out_ptr);

gr_status gr_program_destroy(gr_program* prog);

/* Slice assignment dst[...] = value with NumPy semantics (Listing 6 of the
 * paper: center[:] = 0.2*(center+north+east+west+south)).  `dst` must be a
 * materialised array or a slice/transpose view of one (the storage is
 * WRITTEN by the library, also when it is a borrowed leaf); `value` must
 * have dst's shape and element type.  The right-hand side is finished before
 * the destination changes: if it reads the destination's storage at other
 * positions than it writes (a stencil), it is evaluated into a temporary and
 * copied; otherwise one fused kernel writes the destination directly.
 * Every view of the storage sees the new contents; recorded but unevaluated
 * arrays that read the storage are evaluated first, so they keep the values
 * they had when recorded.  Runs asynchronously on the context's stream. */
gr_status gr_assign(gr_ctx* ctx, gr_array dst, gr_array value);

/* ---- inspection --------------------------------------------------------- */

gr_status gr_ndim(gr_ctx* ctx, gr_array a, int* ndim);
gr_status gr_shape(gr_ctx* ctx, gr_array a, int64_t* shape /* >= ndim entries */);
gr_status gr_dtype_of(gr_ctx* ctx, gr_array a, gr_dtype* dtype);
gr_status gr_is_materialized(gr_ctx* ctx, gr_array a, int* flag);
/* Device pointer to element (0,..,0) and element strides of a materialised
 * array (a view of a materialised array counts). */
gr_status gr_data_ptr(gr_ctx* ctx, gr_array a, void** dptr, int64_t* strides /* >= ndim entries */);

/* ---- lifetime ----------------------------------------------------------- */

/* A node lives while a handle or a node recorded on top of it refers to it. */
gr_status gr_retain(gr_ctx* ctx, gr_array a);
gr_status gr_release(gr_ctx* ctx, gr_array a);

/* ---- planning without execution (host only; works without a device) ----- */

/* Writes a text description of the ordered sub-graph list that
 * gr_materialize(a) would execute (one line per sub-graph: kind, root,
 * member nodes, leaves) into buf (host, NUL-terminated, truncated to cap).
 * *needed receives the full length including the NUL. */
gr_status gr_plan_describe(gr_ctx* ctx, gr_array a, char* buf, size_t cap, size_t* needed);

/* Same for the generated HIP source of sub-graph `index` of that list. */
gr_status gr_plan_source(gr_ctx* ctx, gr_array a, int index, char* buf, size_t cap, size_t* needed);

/* Compiles every sub-graph of the plan for gfx950 without running it (works
 * without a device), and the kernels that gr_materialize_into_static would use
 * for the same request where they differ; returns GR_ERR_COMPILE with the
 * compiler log in gr_last_error on failure. */
gr_status gr_plan_compile(gr_ctx* ctx, gr_array a);

/* Blocks until every run-time compilation started by earlier requests has
 * finished, loads the kernels and writes their code objects to the on-disk
 * cache (Section 6 of the paper: compilation runs beside execution; this is
 * the point where a caller who wants the compiled kernels from now on waits
 * for them).  GR_ERR_COMPILE with the first compiler log on failure. */
gr_status gr_compile_wait(gr_ctx* ctx);

/* ---- statistics and profiling ------------------------------------------- */

typedef struct {
  uint64_t nodes_recorded;
  uint64_t nodes_alive;
  uint64_t materialize_calls;
  uint64_t groups_executed;   /* sub-graphs run */
  uint64_t kernel_launches;
  uint64_t cache_hits;        /* kernel cache, keyed on the sub-graph signature */
  uint64_t cache_misses;      /* = run-time compilations */
  double compile_ms;          /* total time inside the run-time compiler */
  uint64_t bytes_allocated;   /* by the context's allocator, cumulative */
  uint64_t disk_hits;         /* cache misses served from the on-disk code-object cache */
  uint64_t nodes_merged;      /* recordings answered with an equal pending node (option "merge") */
  uint64_t interp_launches;   /* sub-graphs evaluated by the byte-code interpreter (option "interp") */
  uint64_t assign_swaps;      /* slice assignments done by writing a second buffer and swapping (option "assign_swap") */
  uint64_t plan_hits;         /* requests answered with a remembered plan (option "plan_cache") */
  uint64_t pool_bytes;        /* device memory the default pool holds right now (in use or free for reuse) */
} gr_stats_t;

gr_status gr_stats(gr_ctx* ctx, gr_stats_t* out);

/* With option "profile" = 1 every launch is bracketed by two HIP events on
 * the context's stream.  gr_profile_read waits for the stream and returns,
 * for the kernel kind whose name starts with `prefix` (host string; "" =
 * all), the number of launches and their summed duration since the last
 * gr_profile_reset. */
gr_status gr_profile_reset(gr_ctx* ctx);
gr_status gr_profile_read(gr_ctx* ctx, const char* prefix, uint64_t* launches, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* GRUMPY_HIP_H */
