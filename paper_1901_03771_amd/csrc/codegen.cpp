// Kernel generator: turns one planned sub-graph into HIP source for gfx950.
//
// Section 3 of the paper generates, from a point function and an iteration
// space, a `map` kernel (one GPU thread per point) or a `map-reduce` kernel
// (per-block combine in shared memory, second kernel for the block partials).
// The skeletons below keep that contract (the point function is the SSA
// program built by the planner) and replace the launch shapes with ones
// fitted to CDNA4:
//
//   MAP     each lane owns a patch of VR rows x UC chunks of 4 consecutive
//           columns; loads and stores are dwordx4; values shared between the
//           points of a patch (broadcast operands, overlapping slice views)
//           are loaded and computed once per patch and stay in registers.
//   ROWRED  a row is held in registers by 16 / 64 / 256 lanes across all
//           reduction phases and the final map (wave shuffles, LDS only
//           across the four waves of a 256-lane row).
//   REDUCE  generic reduction root: a thread or a workgroup per output.
//   GEMV    bandwidth-bound contraction kernels (row-dot, and
//           column-accumulate with a deterministic second combine stage in
//           the manner of the paper's two-kernel reduction) whose epilogue
//           is the point function of the dot's pointwise consumers.
#include "codegen.h"

#include <algorithm>
#include <functional>
#include <map>
#include <set>
#include <sstream>

#include "ctx.h"

namespace gr {

char access_class(const AccessGroup& ag, int dim) {
  if (ag.structural_zero[dim]) return 'Z';
  if (ag.coef[dim] == 1 && ag.dtype != GR_I64) return '1';
  return 'G';
}

// Arrays that are streamed through once (unit stride, not re-read through shifted
// views, not broadcast along rows) bypass cache retention; operands that lanes
// share stay cacheable.
bool nontemporal_group(const GroupPlan& g, int group) {
  const AccessGroup& ag = g.groups[group];
  if ((g.nt & 7) == 0 || ag.dtype == GR_I64) return false;
  if (g.kind == GroupKind::GEMV) return group == g.mat_group;
  if (g.kind == GroupKind::GEMM) return false;  // operand tiles are re-read by other workgroups: keep them cacheable
  // (tiles of neighbouring lines of a scan: lanes run along the innermost line dimension)
  const int lane_dim = g.kind == GroupKind::SCAN && g.scan_mode == 3 ? g.rank - 2 : g.rank - 1;
  if (access_class(ag, lane_dim) != '1') return false;
  if ((g.nt & 7) >= 2) return true;
  if (ag.deltas.size() > 1) return false;
  // read once = the operand follows every outer iteration dimension; one that is broadcast along
  // any of them is read again by other rows or planes and stays cacheable
  for (int k = 0; k < g.rank; ++k) if (k != lane_dim && ag.structural_zero[k]) return false;
  return true;
}

ArgLayout arg_layout(const GroupPlan& g) {
  ArgLayout L;
  int s = 0;
  for (size_t i = 0; i < g.groups.size(); ++i) {
    bool core = (g.kind == GroupKind::GEMV || g.kind == GroupKind::GEMM) && ((int)i == g.mat_group || (int)i == g.vec_group);
    int nc = core ? 2 : g.rank;
    L.ptr.push_back(s++);
    L.base.push_back(s++);
    L.coef.push_back(s);
    L.ncoef.push_back(nc);
    s += nc;
  }
  L.out = s++;
  L.dims = s;
  s += g.rank;
  L.consts = s;
  s += (int)g.consts.size();
  L.extra = s;
  s += 4;
  L.ocoef = s;
  if (g.kind == GroupKind::SCAN || g.kind == GroupKind::MAP) s += g.rank;
  if (g.kind == GroupKind::GEMM) s += 2;  // split-K: workspace pointer, k extent of one split
  L.obase = s;
  if (g.kind == GroupKind::MAP) s += 1;
  L.total = s;
  return L;
}

std::string kernel_name(const GroupPlan& g) {
  switch (g.kind) {
    case GroupKind::MAP: return "gr_map";
    case GroupKind::ROWRED: return "gr_rowred";
    case GroupKind::REDUCE: return "gr_reduce";
    case GroupKind::SCAN: return "gr_scan";
    case GroupKind::GEMM: return "gr_gemm";
    case GroupKind::GEMV: return g.gemv_mode == 2 ? "gr_gemv_pair" : (g.gemv_mode ? "gr_gemv_colacc" : "gr_gemv_rowdot");
  }
  return "gr_kernel";
}

namespace {

const char* cty(gr_dtype dt) { return dt == GR_F32 ? "float" : (dt == GR_I32 ? "int" : "long long"); }
const char* vty4(gr_dtype dt) { return dt == GR_F32 ? "f4u" : "i4u"; }
const char* vty2(gr_dtype dt) { return dt == GR_F32 ? "f2u" : "i2u"; }

struct Em {
  const GroupPlan& g;
  ArgLayout L;
  std::ostringstream o;
  int slot_base = 0;     // first slot of this sub-graph's block inside the kernel's argument array
  int total_slots = 0;   // size of the whole argument array
  std::string qp = "q";  // name prefix of the per-group base pointers
  explicit Em(const GroupPlan& gp) : g(gp), L(arg_layout(gp)) { total_slots = L.total; }
  std::string slot(int n) const { return "a.s[" + std::to_string(slot_base + n) + "]"; }

  // *(const T*)(addr), with the non-temporal hint where the group streams
  std::string ld(int group, const std::string& type, const std::string& addr) const {
    if (nontemporal_group(g, group)) return "__builtin_nontemporal_load((const GM " + type + "*)(" + addr + "))";
    return "*(const GM " + type + "*)(" + addr + ")";
  }

  std::string S(int n) const { return "((long long)" + slot(n) + ")"; }
  std::string dim(int k) const { return S(L.dims + k); }
  std::string cst(int cslot) const {
    const ConstSlot& c = g.consts[cslot];
    std::string s = slot(L.consts + cslot);
    if (c.dtype == GR_F32) return "__uint_as_float((unsigned)" + s + ")";
    if (c.dtype == GR_I32) return "((int)" + s + ")";
    return "((long long)" + s + ")";
  }
  std::string coef(int grp, int k) const { return S(L.coef[grp] + k); }

  static std::string unop(int op, gr_dtype dt, const std::string& x) {
    if (dt == GR_F32) switch (op) {
      case GR_NEG: return "(-" + x + ")";
      case GR_ABS: return "__builtin_fabsf(" + x + ")";
      case GR_EXP: return "gr_expf(" + x + ")";
      case GR_LOG: return "gr_logf(" + x + ")";
      case GR_SQRT: return "gr_sqrtf(" + x + ")";
      case GR_SQUARE: return "(" + x + " * " + x + ")";
      case GR_TANH: return "tanhf(" + x + ")";
      case GR_ERF: return "gr_erff(" + x + ")";
    }
    switch (op) {  // i32: two's-complement wrap-around through unsigned arithmetic
      case GR_NEG: return "((int)(0u - (unsigned)" + x + "))";
      case GR_ABS: return "(" + x + " < 0 ? (int)(0u - (unsigned)" + x + ") : " + x + ")";
      case GR_SQUARE: return "((int)((unsigned)" + x + " * (unsigned)" + x + "))";
    }
    return "0";
  }
  static std::string binop(int op, gr_dtype dt, const std::string& x, const std::string& y) {
    if (dt == GR_F32) switch (op) {
      case GR_ADD: return "(" + x + " + " + y + ")";
      case GR_SUB: return "(" + x + " - " + y + ")";
      case GR_MUL: return "(" + x + " * " + y + ")";
      case GR_DIV: return "(" + x + " / " + y + ")";
      case GR_MAXIMUM: return "gr_maxf(" + x + ", " + y + ")";
      case GR_MINIMUM: return "gr_minf(" + x + ", " + y + ")";
    }
    switch (op) {
      case GR_ADD: return "((int)((unsigned)" + x + " + (unsigned)" + y + "))";
      case GR_SUB: return "((int)((unsigned)" + x + " - (unsigned)" + y + "))";
      case GR_MUL: return "((int)((unsigned)" + x + " * (unsigned)" + y + "))";
      case GR_MAXIMUM: return "(" + x + " >= " + y + " ? " + x + " : " + y + ")";
      case GR_MINIMUM: return "(" + x + " <= " + y + " ? " + x + " : " + y + ")";
    }
    return "0";
  }

  // combine(acc, x) for a reduction phase
  static std::string combine(const Phase& p, const std::string& acc, const std::string& x) {
    if (p.op == GR_SUM) {
      if (p.out_dtype == GR_I64) return "(" + acc + " + (long long)" + x + ")";
      return "(" + acc + " + " + x + ")";
    }
    if (p.in_dtype == GR_F32) return std::string(p.op == GR_MAX ? "gr_maxf(" : "gr_minf(") + acc + ", " + x + ")";
    return "(" + acc + (p.op == GR_MAX ? " >= " : " <= ") + x + " ? " + acc + " : " + x + ")";
  }
  static std::string identity(const Phase& p) {
    if (p.op == GR_SUM) return p.out_dtype == GR_F32 ? "0.0f" : (p.out_dtype == GR_I64 ? "0ll" : "0");
    if (p.in_dtype == GR_F32) return p.op == GR_MAX ? "(-__builtin_inff())" : "__builtin_inff()";
    return p.op == GR_MAX ? "(-2147483647 - 1)" : "2147483647";
  }
  static std::string zero(gr_dtype dt) { return dt == GR_F32 ? "0.0f" : (dt == GR_I64 ? "0ll" : "0"); }
};

// gr_erff, gr_divc: the text the interpreter kernels are compiled from as well
#define GR_DEVICE_MATH_SOURCE(...) #__VA_ARGS__
const char* const kDeviceMath =
#include "device_math.h"
    ;
#undef GR_DEVICE_MATH_SOURCE

void prelude(Em& e) {
  // every pointer the kernels dereference is a global-memory pointer (arguments arrive as
  // integers, so the address space has to be stated for global_load/global_store to be used)
  e.o << "#define GM __attribute__((address_space(1)))\n"
         "typedef float f4 __attribute__((ext_vector_type(4)));\n"
         "typedef f4 f4u __attribute__((aligned(4)));\n"
         "typedef float f2 __attribute__((ext_vector_type(2)));\n"
         "typedef f2 f2u __attribute__((aligned(4)));\n"
         "typedef int i4 __attribute__((ext_vector_type(4)));\n"
         "typedef i4 i4u __attribute__((aligned(4)));\n"
         "typedef int i2 __attribute__((ext_vector_type(2)));\n"
         "typedef i2 i2u __attribute__((aligned(4)));\n"
         "struct Args { unsigned long long s[" << e.total_slots << "]; };\n"
         // linear index -> coordinates: rem % d with rem /= d, in 32-bit arithmetic whenever both fit
         // (a 64-bit division is a long instruction sequence, paid per row or per element)
         "static __device__ __forceinline__ long long gr_peel(long long& rem, long long d) {\n"
         "  if ((((unsigned long long)rem) | ((unsigned long long)d)) >> 32) { const long long i = rem % d; rem /= d; return i; }\n"
         "  const unsigned r = (unsigned)rem, dd = (unsigned)d, q = r / dd;\n  rem = q;\n  return r - q * dd;\n}\n"
         // the math helpers' test for a rare argument somewhere in the wave and the barrier that keeps its
         // block a branch; straight-line code in matrix-product kernels, whose epilogues run over up to
         // 256 accumulators per lane and would spill around branches, and in the matrix-vector kernels, whose
         // epilogue sits in the loop over rows: a wave-wide vote there keeps the compiler from overlapping the
         // rows' loads (measured on the logistic-regression step: 85.9 us without the vote, 88.7 with it), and in
         // the scans, whose tiles are loaded ahead in the same way (running sum of exp over 2^27 values: 210 against 268 us)
         << (e.g.kind == GroupKind::GEMM || e.g.kind == GroupKind::GEMV || e.g.kind == GroupKind::SCAN ? "#define GR_ANY_LANE(c) true\n#define GR_KEEP_BRANCH\n"
                                         : "#define GR_ANY_LANE(c) (__builtin_amdgcn_ballot_w64(c) != 0ull)\n#define GR_KEEP_BRANCH __builtin_amdgcn_sched_barrier(0)\n")
         << "static __device__ __forceinline__ float gr_maxf(float a, float b) { return (a >= b || a != a) ? a : b; }\n"
         "static __device__ __forceinline__ float gr_minf(float a, float b) { return (a <= b || a != a) ? a : b; }\n"
         // Correctly rounded square root in five instructions instead of the compiler's sixteen: the
         // hardware's reciprocal square root (1 ulp), then one Newton step on s = x*y with the residual
         // x - s*s taken exactly by an fma.  For every argument of magnitude 2^-96 or more, for zeros,
         // infinities, NaNs and negative numbers the result has the bits of the IEEE square root (all
         // 2^32 arguments are compared on the device by the test suite); below 2^-96 the residual would
         // underflow, so a wave in which any lane holds such an argument takes the library routine.
         // Zeros and infinity are put right by a select that only a wave holding an argument outside
         // [2^-96, inf) executes; other lanes of such a wave keep their value.
         "static __device__ __forceinline__ float gr_sqrtf(float x) {\n"
         "  const float y = __builtin_amdgcn_rsqf(x);\n"
         "  const float s = x * y, h = 0.5f * y;\n"
         "  float t = __builtin_fmaf(__builtin_fmaf(-s, s, x), h, s);\n"
         "  if (GR_ANY_LANE(!(x >= 0x1p-96f && x < __builtin_inff()))) {\n"
         "    GR_KEEP_BRANCH;\n"
         "    const bool tiny = __builtin_fabsf(x) < 0x1p-96f && x != 0.0f;\n"
         "    if (GR_ANY_LANE(tiny)) return sqrtf(x);\n"
         "    t = (x == 0.0f || x == __builtin_inff()) ? x : t;\n"
         "  }\n"
         "  return t;\n}\n"
         << kDeviceMath << "\n"
         "static __device__ __forceinline__ float gr_xor(float v, int m) { return __shfl_xor(v, m, 64); }\n"
         "static __device__ __forceinline__ int gr_xor(int v, int m) { return __shfl_xor(v, m, 64); }\n"
         "static __device__ __forceinline__ long long gr_xor(long long v, int m) {\n"
         "  int lo = __shfl_xor((int)(v & 0xffffffffll), m, 64), hi = __shfl_xor((int)(v >> 32), m, 64);\n"
         "  return ((long long)hi << 32) | (unsigned int)lo;\n}\n";
}

// Emits gr_comb<ph>(a, b) and the lane / block reduction helpers for a phase.
void phase_helpers(Em& e, int ph, int lanes) {
  const Phase& p = e.g.phases[ph];
  const char* T = cty(p.out_dtype);
  // combining two partial results never converts (unlike combining an element into an i64 sum)
  std::string comb;
  if (p.op == GR_SUM) comb = "(x + y)";
  else if (p.out_dtype == GR_F32) comb = std::string(p.op == GR_MAX ? "gr_maxf" : "gr_minf") + "(x, y)";
  else comb = std::string("(x ") + (p.op == GR_MAX ? ">=" : "<=") + " y ? x : y)";
  e.o << "static __device__ __forceinline__ " << T << " gr_comb" << ph << "(" << T << " x, " << T << " y) { return " << comb << "; }\n";
  int w = std::min(lanes, 64);
  e.o << "static __device__ __forceinline__ " << T << " gr_lanes" << ph << "(" << T << " v) {\n";
  for (int m = w / 2; m > 0; m >>= 1) e.o << "  v = gr_comb" << ph << "(v, gr_xor(v, " << m << "));\n";
  e.o << "  return v;\n}\n";
}

// ---- point program emission (scalar) -----------------------------------------

// Emits the instructions of `prog` needed for `want` as scalar statements.
// load_expr(instr) gives the expression of a LOAD; acc_expr the dot result.
void emit_scalar_program(Em& e, const std::vector<Instr>& prog, const std::vector<int>& want,
                         const std::function<std::string(const Instr&, int)>& load_expr, const std::string& acc_expr,
                         const std::string& prefix, const std::string& indent, std::vector<char>* done_io = nullptr) {
  std::vector<char> need(prog.size(), 0);
  std::vector<int> work(want);
  while (!work.empty()) {
    int i = work.back();
    work.pop_back();
    if (i < 0 || need[i]) continue;
    if (done_io && (*done_io)[i]) continue;
    need[i] = 1;
    if (prog[i].a >= 0) work.push_back(prog[i].a);
    if (prog[i].b >= 0) work.push_back(prog[i].b);
  }
  auto name = [&](int i) { return prefix + std::to_string(i); };
  for (size_t i = 0; i < prog.size(); ++i) {
    if (!need[i]) continue;
    const Instr& in = prog[i];
    e.o << indent << "const " << cty(in.dtype) << ' ' << name((int)i) << " = ";
    switch (in.kind) {
      case IKind::LOAD: e.o << load_expr(in, (int)i); break;
      case IKind::CONST: e.o << e.cst(in.cslot); break;
      case IKind::UNARY: e.o << Em::unop(in.op, in.dtype, name(in.a)); break;
      case IKind::BINARY:
        // a quotient whose divisor is a scalar constant of the program: the same in every lane
        if (in.op == GR_DIV && in.dtype == GR_F32 && in.b >= 0 && prog[in.b].kind == IKind::CONST) e.o << "gr_divc(" << name(in.a) << ", " << name(in.b) << ")";
        else e.o << Em::binop(in.op, in.dtype, name(in.a), name(in.b));
        break;
      case IKind::RED: e.o << "red" << in.phase; break;
      case IKind::ACC: e.o << acc_expr; break;
    }
    e.o << ";\n";
    if (done_io) (*done_io)[i] = 1;
  }
}

// Common kernel head: Args, extents.
void kernel_head(Em& e, const std::string& name) {
  e.o << "extern \"C\" __global__ __launch_bounds__(256) void " << name << "(Args a) {\n";
}

// Declares p<g>: pointer of each access group advanced by its base offset.
void group_pointers(Em& e, const std::string& indent, const std::vector<int>& skip = {}) {
  for (size_t gi = 0; gi < e.g.groups.size(); ++gi) {
    if (std::find(skip.begin(), skip.end(), (int)gi) != skip.end()) continue;
    const AccessGroup& ag = e.g.groups[gi];
    e.o << indent << "const GM " << cty(ag.dtype) << "* const " << e.qp << gi << " = (const GM " << cty(ag.dtype) << "*)" << e.slot(e.L.ptr[gi])
        << " + " << e.S(e.L.base[gi]) << ";\n";
  }
}

// ---- MAP ----------------------------------------------------------------------

void gen_map(Em& e) {
  const GroupPlan& g = e.g;
  const int rank = g.rank;
  const int TC = g.BX * 4 * g.UC, TR = g.BY * g.VR;
  const int cd = rank - 1, rd = rank - 2;
  prelude(e);
  kernel_head(e, kernel_name(g));
  e.o << "  const long long C = " << e.dim(cd) << ";\n";
  e.o << "  const long long R = " << (rank >= 2 ? e.dim(rd) : std::string("1")) << ";\n";
  // tile bookkeeping in 32-bit unsigned arithmetic (the grid has fewer than 2^31 tiles)
  e.o << "  const unsigned nbx = (unsigned)((C + " << g.cphase + TC - 1 << ") / " << TC << "), nby = (unsigned)((R + " << TR - 1 << ") / " << TR << ");\n";
  e.o << "  unsigned tile = blockIdx.x;\n";
  if (g.xcd_remap) {
    // consecutive tiles go to the same XCD (workgroups are dealt round-robin over the 8 XCDs),
    // so tiles that share halo rows also share an L2
    e.o << "  { unsigned outer = 1;\n";
    for (int k = 0; k + 2 < rank; ++k) e.o << "    outer *= (unsigned)" << e.dim(k) << ";\n";
    e.o << "    const unsigned ntiles = nbx * nby * outer, per = (ntiles + 7) / 8;\n"
           "    tile = (blockIdx.x % 8) * per + blockIdx.x / 8;\n"
           "    if (tile >= ntiles) return; }\n";
  }
  if (g.diag)
    // A transposed operand of a matrix whose rows are a power of two long: the tiles of one row
    // block lie megabytes apart in it, on few memory channels.  Workgroups in flight together
    // take different row blocks as well as different column blocks.  Column blocks next to each
    // other share cache lines of the output when its rows are not a multiple of 128 bytes long:
    // they go to the same XCD (workgroups are dealt round-robin over the 8 XCDs), whose L2 then
    // merges the two halves of such a line into one write.
    e.o << "  const unsigned slab = nbx * nby, olin = tile / slab, sl = tile % slab;\n"
           "  unsigned bx, by;\n"
           "  if ((nbx & 7) == 0) { const unsigned nq = nbx >> 3, l = sl >> 3; bx = (sl & 7) * nq + l % nq; by = (l / nq + bx) % nby; }\n"
           "  else { bx = sl % nbx; by = (sl / nbx + bx) % nby; }\n";
  else
    e.o << "  const unsigned bx = tile % nbx, t2 = tile / nbx, by = t2 % nby, olin = t2 / nby;\n";
  if (rank > 2) {
    e.o << "  unsigned orem = olin;\n";
    for (int k = rank - 3; k >= 0; --k) e.o << "  const long long i" << k << " = orem % (unsigned)" << e.dim(k) << "; orem /= (unsigned)" << e.dim(k) << ";\n";
  }
  e.o << "  const int tx = threadIdx.x % " << g.BX << ", ty = threadIdx.x / " << g.BX << ";\n";
  e.o << "  const long long r0 = (long long)by * " << TR << " + ty * " << g.VR << ", c0 = (long long)bx * " << TC << " + tx * 4" << (g.cphase ? " - " + std::to_string(g.cphase) : std::string()) << ";\n";
  group_pointers(e, "  ");
  for (size_t gi = 0; gi < g.groups.size(); ++gi) {
    const AccessGroup& ag = g.groups[gi];
    e.o << "  const GM " << cty(ag.dtype) << "* const p" << gi << " = q" << gi;
    for (int k = 0; k + 2 < rank; ++k) if (!ag.structural_zero[k]) e.o << " + i" << k << " * " << e.coef((int)gi, k);
    if (rank >= 2 && !ag.structural_zero[rd]) e.o << " + r0 * " << e.coef((int)gi, rd);
    char cc = access_class(ag, cd);
    if (cc == '1') e.o << " + c0";
    else if (cc == 'G') e.o << " + c0 * " << e.coef((int)gi, cd);
    e.o << ";\n";
  }
  // output strides are arguments: a C-contiguous result or the strided view of a slice assignment
  e.o << "  const long long oc = " << (g.out_unit ? std::string("1") : e.S(e.L.ocoef + cd)) << ", orow = " << (rank >= 2 ? e.S(e.L.ocoef + rd) : std::string("0")) << ";\n";
  e.o << "  GM " << cty(g.out_dtype) << "* const po = (GM " << cty(g.out_dtype) << "*)" << e.slot(e.L.out) << " + " << e.S(e.L.obase);
  for (int k = 0; k + 2 < rank; ++k) e.o << " + i" << k << " * " << e.S(e.L.ocoef + k);
  e.o << " + r0 * orow + c0 * oc;\n";

  // static part of a load's address: shifts times runtime coefficients
  auto shift_expr = [&](const Instr& in, bool with_col) {
    const AccessGroup& ag = g.groups[in.group];
    std::ostringstream s;
    bool any = false;
    for (int k = 0; k < rank; ++k) {
      if (in.delta[k] == 0 || ag.structural_zero[k]) continue;
      if (k == cd) {
        if (!with_col) continue;
        if (access_class(ag, cd) == '1') s << (any ? " + " : "") << in.delta[k];
        else s << (any ? " + " : "") << in.delta[k] << " * " << e.coef(in.group, k);
      } else s << (any ? " + " : "") << in.delta[k] << " * " << e.coef(in.group, k);
      any = true;
    }
    if (!any) s << "0";
    return s.str();
  };

  // ---- transposed operands: the workgroup's tile (64 columns by 64 or 128 rows) goes through LDS, loaded along the
  // operand's own contiguous dimension (the rows of the iteration space) ----
  if (g.stage_mask) {
    for (size_t gi = 0; gi < g.groups.size(); ++gi) {
      if (!(g.stage_mask >> gi & 1)) continue;
      const AccessGroup& ag = g.groups[gi];
      const char* T = cty(ag.dtype);
      const char* V4 = vty4(ag.dtype);
      // tile: 64 columns by STR = BY * VR rows of the iteration space, i.e. 64 runs of STR
      // contiguous elements of the operand
      const int STR = g.BY * g.VR, TPR = STR / 4, RPP = 256 / TPR, NPASS = 64 / RPP;
      // Row cc of the tile is rotated by 4 * (cc / 4) elements: a lane's four-element writes
      // (along the operand's contiguous dimension) and its four-element reads (rows of its patch,
      // one column) both touch every LDS bank once per eight lanes.
      const char* V4A = ag.dtype == GR_F32 ? "f4" : "i4";
      e.o << "  __shared__ __attribute__((aligned(16))) " << T << " tg" << gi << "[64][" << STR << "];\n";
      e.o << "  { const GM " << T << "* const pt = q" << gi;
      for (int k = 0; k + 2 < rank; ++k) if (!ag.structural_zero[k]) e.o << " + i" << k << " * " << e.coef((int)gi, k);
      e.o << " + (long long)by * " << STR << " + (long long)bx * 64 * " << e.coef((int)gi, cd) << ";\n";
      e.o << "    const int c1 = threadIdx.x / " << TPR << ", r4 = (threadIdx.x % " << TPR << ") * 4;\n";
      // interior tiles: every load is issued before the first LDS store
      e.o << "    if ((long long)bx * 64 + 64 <= C && (long long)by * " << STR << " + " << STR << " <= R) {\n"
             "      " << V4 << " w[" << NPASS << "];\n"
             "      _Pragma(\"unroll\") for (int i = 0; i < " << NPASS << "; ++i) w[i] = *(const GM " << V4 << "*)(pt + (c1 + " << RPP << " * i) * " << e.coef((int)gi, cd) << " + r4);\n"
             "      _Pragma(\"unroll\") for (int i = 0; i < " << NPASS << "; ++i) { const int cc = c1 + " << RPP << " * i;"
             " *(" << V4A << "*)&tg" << gi << "[cc][(r4 + 4 * (cc >> 2)) & " << STR - 1 << "] = w[i]; }\n"
             "    } else\n";
      e.o << "    for (int i = 0; i < " << NPASS << "; ++i) {\n      const int cc = c1 + " << RPP << " * i;\n"
             "      const long long gc = (long long)bx * 64 + cc, gr = (long long)by * " << STR << " + r4;\n"
             "      if (gc < C && gr + 4 <= R) { const " << V4 << " w = *(const GM " << V4 << "*)(pt + cc * " << e.coef((int)gi, cd) << " + r4);"
             " *(" << V4A << "*)&tg" << gi << "[cc][(r4 + 4 * (cc >> 2)) & " << STR - 1 << "] = w; }\n"
             "      else if (gc < C) { for (int j = 0; j < 4; ++j) if (gr + j < R) tg" << gi << "[cc][(r4 + j + 4 * (cc >> 2)) & " << STR - 1 << "] = pt[cc * " << e.coef((int)gi, cd) << " + r4 + j]; }\n"
             "    }\n  }\n";
    }
    e.o << "  __syncthreads();\n";
  }
  // ---- lanes whose whole patch lies inside the array: straight-line ----
  e.o << "  if (r0 + " << g.VR << " <= R && c0 + " << (g.UC - 1) * g.BX * 4 + 4 << " <= C" << (g.cphase ? " && c0 >= 0" : "") << ") {\n";
  // group the contiguous loads of the patch program into vector loads
  std::map<int, std::string> load_name;  // instr -> expression
  {
    // key: group + all deltas but the column one
    std::map<std::vector<int64_t>, std::vector<std::pair<int64_t, int>>> rows;
    std::vector<char> used(g.prog.size(), 0);
    {  // only loads reachable from the results
      std::vector<int> work(g.results.begin(), g.results.end());
      while (!work.empty()) {
        int i = work.back();
        work.pop_back();
        if (i < 0 || used[i]) continue;
        used[i] = 1;
        work.push_back(g.prog[i].a);
        work.push_back(g.prog[i].b);
      }
    }
    int nl = 0;
    std::set<std::string> staged_done;
    for (size_t i = 0; i < g.prog.size(); ++i) {
      const Instr& in = g.prog[i];
      if (in.kind != IKind::LOAD || !used[i]) continue;
      const AccessGroup& ag = g.groups[in.group];
      if (g.stage_mask >> in.group & 1) {
        // element (row r0 + dr, column c0 + dc) of the iteration space sits at [column][row] of the
        // tile (rotated): four rows of one column are one 16-byte LDS read
        const int dc = (int)in.delta[cd], dr = (int)in.delta[rd];
        const std::string nm = "S" + std::to_string(in.group) + "_" + std::to_string(dc) + "_" + std::to_string(dr / 4);
        if (staged_done.insert(nm).second)
          e.o << "    const " << (ag.dtype == GR_F32 ? "f4" : "i4") << ' ' << nm << " = *(const " << (ag.dtype == GR_F32 ? "f4" : "i4") << "*)&tg" << in.group
              << "[tx * 4 + " << dc << "][(ty * " << g.VR << " + " << dr / 4 * 4 << " + 4 * tx) & " << g.BY * g.VR - 1 << "];\n";
        load_name[(int)i] = nm + "[" + std::to_string(dr % 4) + "]";
        continue;
      }
      if (access_class(ag, cd) != '1') {
        load_name[(int)i] = "p" + std::to_string(in.group) + "[" + shift_expr(in, true) + "]";
        continue;
      }
      std::vector<int64_t> key{in.group};
      for (int k = 0; k < rank; ++k) if (k != cd) key.push_back(in.delta[k]);
      rows[key].push_back({in.delta[cd], (int)i});
    }
    for (auto& kv : rows) {
      auto& v = kv.second;
      std::sort(v.begin(), v.end());
      const Instr& first = g.prog[v[0].second];
      const AccessGroup& ag = g.groups[first.group];
      std::string rowoff = shift_expr(first, false);
      size_t i = 0;
      while (i < v.size()) {
        size_t run = 1;
        while (i + run < v.size() && v[i + run].first == v[i].first + (int64_t)run) ++run;
        size_t pos = 0;
        while (pos < run) {
          size_t take = run - pos >= 4 ? 4 : (run - pos >= 2 ? 2 : 1);
          int64_t dc = v[i + pos].first;
          std::string nm = "L" + std::to_string(nl++);
          std::string addr = "p" + std::to_string(first.group) + " + (" + rowoff + ") + " + std::to_string(dc);
          const char* lt = take == 4 ? vty4(ag.dtype) : (take == 2 ? vty2(ag.dtype) : cty(ag.dtype));
          e.o << "    const " << lt << ' ' << nm << " = " << e.ld(first.group, lt, addr) << ";\n";
          for (size_t q = 0; q < take; ++q)
            load_name[v[i + pos + q].second] = take == 1 ? nm : nm + "[" + std::to_string(q) + "]";
          pos += take;
        }
        i += run;
      }
    }
  }
  emit_scalar_program(e, g.prog, g.results,
                      [&](const Instr&, int id) { return load_name[id]; }, "0.0f", "t", "    ");
  {
    int ri = 0;
    for (int v = 0; v < g.VR; ++v)
      for (int u = 0; u < g.UC; ++u) {
        std::string off = std::to_string(v) + " * orow + " + std::to_string(u * g.BX * 4) + " * oc";
        if (g.out_dtype == GR_I64 || !g.out_unit) {
          for (int j = 0; j < 4; ++j) e.o << "    po[" << off << " + " << j << " * oc] = t" << g.results[ri + j] << ";\n";
        } else {
          const char* vt = g.out_dtype == GR_F32 ? "f4u" : "i4u";
          e.o << "    { " << vt << " ov; ov[0] = t" << g.results[ri] << "; ov[1] = t" << g.results[ri + 1] << "; ov[2] = t" << g.results[ri + 2]
              << "; ov[3] = t" << g.results[ri + 3] << "; " << ((g.nt & 8) ? "__builtin_nontemporal_store(ov, (GM " + std::string(vt) + "*)(po + " + off + "))" : "*(GM " + std::string(vt) + "*)(po + " + off + ") = ov") << "; }\n";
        }
        ri += 4;
      }
  }
  // ---- narrow arrays: the lanes of the last, incomplete group of four columns (all rows of
  // their patch inside): the same patch program restricted to the columns that exist, scalar
  // loads and stores, no guards ----
  if (g.tail > 0) {
    e.o << "  } else if (r0 + " << g.VR << " <= R && c0 + " << g.tail << " == C) {\n";
    std::vector<int> want;
    for (int v = 0; v < g.VR; ++v)
      for (int j = 0; j < g.tail; ++j) want.push_back(g.results[(size_t)v * 4 + j]);
    emit_scalar_program(e, g.prog, want,
                        [&](const Instr& in, int) { return "p" + std::to_string(in.group) + "[" + shift_expr(in, true) + "]"; },
                        "0.0f", "w", "    ");
    for (int v = 0; v < g.VR; ++v)
      for (int j = 0; j < g.tail; ++j)
        e.o << "    po[" << v << " * orow + " << j << " * oc] = w" << g.results[(size_t)v * 4 + j] << ";\n";
  }
  // ---- lanes on the array's edge: one guarded point at a time ----
  e.o << "  } else {\n"
         "    for (int v = 0; v < " << g.VR << "; ++v)\n"
         "      for (int u = 0; u < " << g.UC << "; ++u)\n"
         "        for (int j = 0; j < 4; ++j) {\n"
         "          const long long cj = (long long)u * " << g.BX * 4 << " + j;\n"
         "          if (r0 + v < R && c0 + cj < C" << (g.cphase ? " && c0 + cj >= 0" : "") << ") {\n";
  emit_scalar_program(e, g.prog1, {g.result1},
                      [&](const Instr& in, int) {
                        const AccessGroup& ag = g.groups[in.group];
                        std::string s = "p" + std::to_string(in.group) + "[" + shift_expr(in, true);
                        if (rank >= 2 && !ag.structural_zero[rd]) s += " + v * " + e.coef(in.group, rd);
                        char cc = access_class(ag, cd);
                        if (cc == '1') s += " + cj";
                        else if (cc == 'G') s += " + cj * " + e.coef(in.group, cd);
                        return s + "]";
                      },
                      "0.0f", "s", "            ");
  e.o << "            po[v * orow + cj * oc] = s" << g.result1 << ";\n"
         "          }\n        }\n  }\n}\n";
}

// ---- ROWRED -------------------------------------------------------------------

void gen_rowred(Em& e) {
  const GroupPlan& g = e.g;
  const int rank = g.rank, cd = rank - 1;
  const int RT = g.row_threads, NP = g.NP, RB = 256 / RT;
  const int nph = (int)g.phases.size();
  prelude(e);
  for (int ph = 0; ph < nph; ++ph) phase_helpers(e, ph, RT);

  // stage of first computation and liveness across stages
  const int nstage = nph + 1;
  std::vector<int> stage_of(g.prog.size(), -1);
  std::vector<std::vector<int>> stage_instrs(nstage);
  std::vector<char> keep(g.prog.size(), 0);
  for (int s = 0; s < nstage; ++s) {
    int want = s < nph ? g.phases[s].value : (g.results.empty() ? -1 : g.results[0]);
    std::vector<int> work{want};
    std::vector<char> seen(g.prog.size(), 0);
    while (!work.empty()) {
      int i = work.back();
      work.pop_back();
      if (i < 0 || seen[i]) continue;
      seen[i] = 1;
      if (stage_of[i] >= 0 && stage_of[i] < s) { keep[i] = 1; continue; }
      stage_of[i] = s;
      work.push_back(g.prog[i].a);
      work.push_back(g.prog[i].b);
    }
    for (size_t i = 0; i < g.prog.size(); ++i) if (stage_of[i] == s) stage_instrs[s].push_back((int)i);
  }

  kernel_head(e, kernel_name(g));
  e.o << "  const long long C = " << e.dim(cd) << ";\n  long long ROWS = 1;\n";
  for (int k = 0; k < cd; ++k) e.o << "  ROWS *= " << e.dim(k) << ";\n";
  e.o << "  const int lane = threadIdx.x % " << RT << ";\n";
  // several rows per lane group (short rows, one value per row): the per-row code below is written
  // once into `body` and placed in two loops, see the end of this function
  const int RPT = (g.row_iters > 1 && RT <= 64 && g.out_per_row) ? g.row_iters : 1;
  // exact: the row is exactly as wide as the lanes' positions, no column guards anywhere
  auto emit_body = [&](bool exact) {
  if (RPT > 1) {
    e.o << "      const long long row = ((long long)blockIdx.x * " << RPT << " + rr) * " << RB << " + threadIdx.x / " << RT << ";\n      const bool row_ok = true;\n";
  } else if (RT <= 64) {
    // no workgroup barrier in this variant: lanes of rows past the end simply leave
    e.o << "  const long long row = (long long)blockIdx.x * " << RB << " + threadIdx.x / " << RT << ";\n";
    e.o << "  if (row >= ROWS) return;\n  const bool row_ok = true;\n";
  } else {
    // rows span several waves and combine through LDS behind a barrier every wave reaches:
    // lanes of a row past the end recompute the last row and skip the stores
    e.o << "  const long long row_raw = (long long)blockIdx.x * " << RB << " + threadIdx.x / " << RT << ";\n";
    e.o << "  const bool row_ok = row_raw < ROWS;\n  const long long row = row_ok ? row_raw : ROWS - 1;\n";
    e.o << "  __shared__ long long gr_sm[" << std::max(nph, 1) << "][4];\n";
  }
  e.o << "  (void)row_ok;\n";
  if (cd >= 1) {
    e.o << "  long long rrem = row;\n";
    for (int k = cd - 1; k >= 0; --k) {
      if (k == 0) e.o << "  const long long i0 = rrem;\n";  // what is left is below the outermost extent
      else e.o << "  const long long i" << k << " = gr_peel(rrem, " << e.dim(k) << ");\n";
    }
  }
  group_pointers(e, "  ");
  for (size_t gi = 0; gi < g.groups.size(); ++gi) {
    const AccessGroup& ag = g.groups[gi];
    e.o << "  const GM " << cty(ag.dtype) << "* const p" << gi << " = q" << gi;
    for (int k = 0; k < cd; ++k) if (!ag.structural_zero[k]) e.o << " + i" << k << " * " << e.coef((int)gi, k);
    e.o << ";\n";
  }
  if (RPT > 1) e.o << "//@@SPLIT\n";  // up to here: from the row number to the row's pointers
  // kept per-element values live in registers across stages
  for (size_t i = 0; i < g.prog.size(); ++i)
    if (keep[i] && !g.prog[i].uniform) e.o << "  " << cty(g.prog[i].dtype) << " k" << i << "[" << NP << "][4];\n";
  for (int ph = 0; ph < nph; ++ph) e.o << "  " << cty(g.phases[ph].out_dtype) << " red" << ph << ";\n";

  auto shift_expr = [&](const Instr& in) {
    const AccessGroup& ag = g.groups[in.group];
    std::ostringstream s;
    bool any = false;
    for (int k = 0; k < cd; ++k) {
      if (in.delta[k] == 0 || ag.structural_zero[k]) continue;
      s << (any ? " + " : "") << in.delta[k] << " * " << e.coef(in.group, k);
      any = true;
    }
    if (!any) s << "0";
    return s.str();
  };
  auto name = [&](int i, bool in_loop) -> std::string {
    const Instr& in = g.prog[i];
    if (in.uniform) return "u" + std::to_string(i);
    if (keep[i]) return "k" + std::to_string(i) + "[p][j]";
    (void)in_loop;
    return "t" + std::to_string(i);
  };
  auto expr = [&](int i) -> std::string {
    const Instr& in = g.prog[i];
    switch (in.kind) {
      case IKind::CONST: return e.cst(in.cslot);
      case IKind::UNARY: return Em::unop(in.op, in.dtype, name(in.a, true));
      case IKind::BINARY:
        if (in.op == GR_DIV && in.dtype == GR_F32 && in.b >= 0 && g.prog[in.b].kind == IKind::CONST) return "gr_divc(" + name(in.a, true) + ", " + name(in.b, true) + ")";
        return Em::binop(in.op, in.dtype, name(in.a, true), name(in.b, true));
      case IKind::RED: return "red" + std::to_string(in.phase);
      default: return "0";
    }
  };

  for (int s = 0; s < nstage; ++s) {
    const bool final_stage = s == nph;
    if (final_stage && g.results.empty()) break;
    e.o << "  // ---- " << (final_stage ? "final map" : "reduction phase") << " " << s << "\n";
    // row-uniform values first
    for (int i : stage_instrs[s]) {
      const Instr& in = g.prog[i];
      if (!in.uniform) continue;
      e.o << "  const " << cty(in.dtype) << " u" << i << " = ";
      if (in.kind == IKind::LOAD) e.o << "p" << in.group << "[" << shift_expr(in) << "]";
      else e.o << expr(i);
      e.o << ";\n";
    }
    if (final_stage && g.out_per_row) {
      if (RPT > 1) e.o << "  GR_ROW_RESULT(" << name(g.results[0], false) << ");\n";
      else e.o << "  if (lane == 0 && row_ok) ((GM " << cty(g.out_dtype) << "*)" << e.slot(e.L.out) << ")[row] = " << name(g.results[0], false) << ";\n";
      break;
    }
    const Phase* ph = final_stage ? nullptr : &g.phases[s];
    if (ph) e.o << "  " << cty(ph->out_dtype) << " acc" << s << " = " << Em::identity(*ph) << ";\n";
    if (final_stage)
      e.o << "  GM " << cty(g.out_dtype) << "* const po = (GM " << cty(g.out_dtype) << "*)" << e.slot(e.L.out) << " + row * C;\n";
    bool any_elem = false;
    for (int i : stage_instrs[s]) if (!g.prog[i].uniform) any_elem = true;
    int want = ph ? ph->value : g.results[0];
    if (!any_elem && !(keep[want] && !g.prog[want].uniform) && g.prog[want].uniform) {
      // the combined value does not depend on the column: combine it C times
      // (only sums and extrema exist: a sum of C equal values, an extremum of them)
      // handled below by the generic loop with the uniform name.
    }
    // two bodies: unguarded positions 0..NP-2, guarded last position
    for (int pass = 0; pass < 2; ++pass) {
      const bool guarded = pass == 1;
      if (exact && guarded) continue;
      const int np_unguarded = exact ? NP : NP - 1;
      if (!guarded && np_unguarded == 0) continue;
      if (!guarded) e.o << "#pragma unroll\n  for (int p = 0; p < " << np_unguarded << "; ++p) {\n";
      else e.o << "  { const int p = " << NP - 1 << ";\n";
      e.o << "    const long long c = (long long)p * " << RT * 4 << " + lane * 4;\n";
      // loads of this stage
      for (int i : stage_instrs[s]) {
        const Instr& in = g.prog[i];
        if (in.kind != IKind::LOAD || in.uniform) continue;
        const AccessGroup& ag = g.groups[in.group];
        char cc = access_class(ag, cd);
        std::string base = "p" + std::to_string(in.group) + " + (" + shift_expr(in) + ")";
        e.o << "    " << cty(in.dtype) << " l" << i << "[4];\n";
        std::string idx = cc == '1' ? "(c + " + std::to_string(in.delta[cd]) + ")" : "(c + " + std::to_string(in.delta[cd]) + ") * " + e.coef(in.group, cd);
        std::string step = cc == '1' ? "1" : e.coef(in.group, cd);
        if (cc == '1') {
          if (guarded) e.o << "    if (c + 4 <= C) ";
          else e.o << "    ";
          e.o << "{ const " << vty4(in.dtype) << " w = " << e.ld(in.group, vty4(in.dtype), base + " + " + idx) << "; l" << i << "[0] = w[0]; l" << i
              << "[1] = w[1]; l" << i << "[2] = w[2]; l" << i << "[3] = w[3]; }\n";
          if (guarded)
            e.o << "    else { for (int j = 0; j < 4; ++j) l" << i << "[j] = (c + j < C) ? (" << base << ")[" << idx << " + j] : " << Em::zero(in.dtype) << "; }\n";
        } else {
          e.o << "    for (int j = 0; j < 4; ++j) l" << i << "[j] = " << (guarded ? "(c + j < C) ? " : "") << "(" << base << ")[" << idx << " + j * " << step << "]"
              << (guarded ? " : " + Em::zero(in.dtype) : std::string()) << ";\n";
        }
      }
      if (final_stage && g.out_dtype != GR_I64) e.o << "    " << (g.out_dtype == GR_F32 ? "f4u" : "i4u") << " ov;\n";
      e.o << "#pragma unroll\n    for (int j = 0; j < 4; ++j) {\n";
      for (int i : stage_instrs[s]) {
        const Instr& in = g.prog[i];
        if (in.uniform) continue;
        std::string rhs = in.kind == IKind::LOAD ? "l" + std::to_string(i) + "[j]" : expr(i);
        if (keep[i]) e.o << "      k" << i << "[p][j] = " << rhs << ";\n";
        else e.o << "      const " << cty(in.dtype) << " t" << i << " = " << rhs << ";\n";
      }
      if (ph) {
        std::string upd = "acc" + std::to_string(s) + " = " + Em::combine(*ph, "acc" + std::to_string(s), name(want, true)) + ";";
        if (guarded) e.o << "      if (c + j < C) " << upd << "\n";
        else e.o << "      " << upd << "\n";
      } else {
        if (g.out_dtype == GR_I64) e.o << "      if (row_ok" << (guarded ? " && c + j < C" : "") << ") po[c + j] = " << name(want, true) << ";\n";
        else e.o << "      ov[j] = " << name(want, true) << ";\n";
      }
      e.o << "    }\n";
      if (final_stage && g.out_dtype != GR_I64) {
        const char* vt = g.out_dtype == GR_F32 ? "f4u" : "i4u";
        const std::string st = (g.nt & 8) ? "__builtin_nontemporal_store(ov, (GM " + std::string(vt) + "*)(po + c))" : "*(GM " + std::string(vt) + "*)(po + c) = ov";
        if (guarded) e.o << "    if (row_ok) { if (c + 4 <= C) " << st << "; else { for (int j = 0; j < 4; ++j) if (c + j < C) po[c + j] = ov[j]; } }\n";
        else e.o << "    if (row_ok) " << st << ";\n";
      }
      e.o << "  }\n";
    }
    if (ph) {
      e.o << "  acc" << s << " = gr_lanes" << s << "(acc" << s << ");\n";
      if (RT > 64) {
        const char* T = cty(ph->out_dtype);
        e.o << "  { " << T << "* sm = (" << T << "*)gr_sm[" << s << "];\n"
               "    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = acc" << s << ";\n"
               "    __syncthreads();\n";
        if (RT == 256) e.o << "    acc" << s << " = gr_comb" << s << "(gr_comb" << s << "(sm[0], sm[1]), gr_comb" << s << "(sm[2], sm[3])); }\n";
        else e.o << "    const int w0 = (threadIdx.x >> 7) * 2;\n    acc" << s << " = gr_comb" << s << "(sm[w0], sm[w0 + 1]); }\n";
      }
      e.o << "  red" << s << " = acc" << s << ";\n";
    }
  }
  };  // emit_body
  if (RPT == 1) emit_body(false);
  else {
    // the per-row code as text: without column guards for the workgroups whose rows all exist when
    // the rows are exactly as wide as the lanes' positions, with guards for everything else
    std::string body_exact, body_guarded;
    for (int v = 0; v < 2; ++v) {
      std::ostringstream tmp;
      e.o.swap(tmp);
      emit_body(v == 0);
      e.o.swap(tmp);
      (v == 0 ? body_exact : body_guarded) = tmp.str();
    }
    const std::string T = cty(g.out_dtype);
    const std::string out = "((GM " + T + "*)" + e.slot(e.L.out) + ")";
    const std::string mark = "//@@SPLIT\n";
    const std::string setup = body_exact.substr(0, body_exact.find(mark)), stages = body_exact.substr(body_exact.find(mark) + mark.size());
    body_guarded.erase(body_guarded.find(mark), mark.size());
    e.o << "  if (((long long)blockIdx.x * " << RPT << " + " << RPT << ") * " << RB << " <= ROWS && C == " << RT * 4 * NP << ") {\n"
           "    // all rows of the workgroup exist and are exactly as wide as the lanes' positions: no guards;\n"
           "    // the rows' pointers first (index arithmetic with branches), then straight-line code in which\n"
           "    // the loads of the " << RPT << " rows overlap; the results are stored at the end\n"
           "    " << T << " outv[" << RPT << "];\n";
    for (size_t gi = 0; gi < g.groups.size(); ++gi) e.o << "    const GM " << cty(g.groups[gi].dtype) << "* P" << gi << "[" << RPT << "];\n";
    e.o << "#pragma unroll\n    for (int rr = 0; rr < " << RPT << "; ++rr) {\n" << setup;
    for (size_t gi = 0; gi < g.groups.size(); ++gi) e.o << "      P" << gi << "[rr] = p" << gi << ";\n";
    e.o << "    }\n#define GR_ROW_RESULT(v) outv[rr] = (v)\n#pragma unroll\n    for (int rr = 0; rr < " << RPT << "; ++rr) {\n      const bool row_ok = true;\n      (void)row_ok;\n";
    for (size_t gi = 0; gi < g.groups.size(); ++gi) e.o << "      const GM " << cty(g.groups[gi].dtype) << "* const p" << gi << " = P" << gi << "[rr];\n";
    e.o << stages << "    }\n#undef GR_ROW_RESULT\n"
           "    if (lane == 0) {\n";
    for (int rr = 0; rr < RPT; ++rr)
      e.o << "      " << out << "[((long long)blockIdx.x * " << RPT << " + " << rr << ") * " << RB << " + threadIdx.x / " << RT << "] = outv[" << rr << "];\n";
    e.o << "    }\n  } else {\n"
           "#define GR_ROW_RESULT(v) do { if (lane == 0) " << out << "[row] = (v); } while (0)\n"
           "    for (int rr = 0; rr < " << RPT << "; ++rr) {\n      if (((long long)blockIdx.x * " << RPT << " + rr) * " << RB << " + threadIdx.x / " << RT << " >= ROWS) break;\n"
        << body_guarded << "    }\n#undef GR_ROW_RESULT\n  }\n";
  }
  e.o << "}\n";
}

// ---- REDUCE (generic reduction root) --------------------------------------------

void gen_reduce(Em& e) {
  const GroupPlan& g = e.g;
  const int rank = g.rank, kr = g.red_kept_rank;
  const Phase& ph = g.phases[0];
  const char* T = cty(ph.out_dtype);
  prelude(e);
  phase_helpers(e, 0, 64);
  // Stage 1 (Section 3.2: map fused with a per-block combine): every output's reduced range is
  // cut into NSPLIT chunks; a thread (mode 0) or a workgroup (mode 1) combines one chunk.
  kernel_head(e, kernel_name(g));
  e.o << "  const long long NOUT = " << e.S(e.L.extra) << ", LEN = " << e.S(e.L.extra + 1) << ", NSPLIT = " << e.S(e.L.extra + 3) << ";\n";
  if (g.red_mode == 0 && g.red_vec) {
    e.o << "  const long long blocks_o = (NOUT / 4 + 255) / 256;\n"
           "  const long long o = 4 * ((long long)(blockIdx.x % blocks_o) * 256 + threadIdx.x), split = blockIdx.x / blocks_o;\n"
           "  if (o >= NOUT) return;\n";
  } else if (g.red_mode == 0) {
    e.o << "  const long long blocks_o = (NOUT + 255) / 256;\n"
           "  const long long o = (long long)(blockIdx.x % blocks_o) * 256 + threadIdx.x, split = blockIdx.x / blocks_o;\n"
           "  if (o >= NOUT) return;\n";
  } else {
    e.o << "  const long long o = blockIdx.x % NOUT, split = blockIdx.x / NOUT;\n  __shared__ long long gr_sm[4];\n";
  }
  e.o << "  const long long chunk = (LEN + NSPLIT - 1) / NSPLIT, jbeg = split * chunk, jend = (jbeg + chunk < LEN) ? jbeg + chunk : LEN;\n";
  e.o << "  long long orem = o;\n";
  for (int k = kr - 1; k >= 0; --k) {
    if (k == 0) e.o << "  const long long i0 = orem;\n";
    else e.o << "  const long long i" << k << " = gr_peel(orem, " << e.dim(k) << ");\n";
  }
  group_pointers(e, "  ");
  for (size_t gi = 0; gi < g.groups.size(); ++gi) {
    const AccessGroup& ag = g.groups[gi];
    e.o << "  const GM " << cty(ag.dtype) << "* const p" << gi << " = q" << gi;
    for (int k = 0; k < kr; ++k) if (!ag.structural_zero[k]) e.o << " + i" << k << " * " << e.coef((int)gi, k);
    e.o << ";\n";
  }
  e.o << "  " << T << " acc = " << Em::identity(ph) << ";\n";
  // mode 1 over one contiguous reduced dimension: lanes take four consecutive elements with one
  // dwordx4 per array and keep four partial results; the ragged end goes through the scalar loop
  // (several reduced dimensions: the same when the innermost one holds a multiple of four, so that
  // four consecutive elements never straddle it; chunks are then cut at multiples of four)
  const int rd = rank - 1;
  bool vec = g.red_mode == 1 && rank > kr && (rank == kr + 1 || g.red_vec);
  for (size_t i = 0; vec && i < g.prog.size(); ++i) {
    const Instr& in = g.prog[i];
    if (in.dtype == GR_I64) vec = false;
    if (in.kind == IKind::LOAD && !g.groups[in.group].structural_zero[rd] && access_class(g.groups[in.group], rd) != '1') vec = false;
  }
  if (vec && rank > kr + 1) e.o << "  const long long chunk4 = (chunk + 3) / 4 * 4, jbeg4 = split * chunk4, jend4 = (jbeg4 + chunk4 < LEN) ? jbeg4 + chunk4 : LEN;\n";
  if (g.red_mode == 0 && g.red_vec) {
    // four consecutive outputs per thread: one dwordx4 per array and reduced element
    const int kd = kr - 1;
    // (four steps of j written out with all loads first, like the loop of the workgroup-per-chunk kernels below:
    // "#pragma unroll 4" is dropped by the compiler when the body holds a wave-wide vote)
    e.o << "  " << T << " acc1 = acc, acc2 = acc, acc3 = acc;\n";
    auto loads0 = [&](int u, const char* ind) {
      const std::string su = "_" + std::to_string(u);
      if (rank > kr) {
        e.o << ind << "long long jrem" << su << " = j + " << u << ";\n";
        for (int k = rank - 1; k >= kr; --k) {
          if (k == kr) e.o << ind << "const long long i" << k << su << " = jrem" << su << ";\n";
          else e.o << ind << "const long long i" << k << su << " = gr_peel(jrem" << su << ", " << e.dim(k) << ");\n";
        }
      }
      for (size_t i = 0; i < g.prog.size(); ++i) {
        const Instr& in = g.prog[i];
        if (in.kind != IKind::LOAD) continue;
        const AccessGroup& ag = g.groups[in.group];
        std::ostringstream at;
        at << "p" << in.group << " + 0";
        for (int k = 0; k < rank; ++k) {
          if (ag.structural_zero[k]) continue;
          if (k >= kr) at << " + (i" << k << su << " + " << in.delta[k] << ") * " << e.coef(in.group, k);
          else if (in.delta[k]) at << " + " << in.delta[k] << (k == kd ? std::string("") : " * " + e.coef(in.group, k));
        }
        if (ag.structural_zero[kd]) e.o << ind << "const " << cty(in.dtype) << " u" << i << su << " = (" << at.str() << ")[0];\n";
        else e.o << ind << "const " << vty4(in.dtype) << " w" << i << su << " = " << e.ld(in.group, vty4(in.dtype), at.str()) << ";\n";
      }
    };
    auto compute0 = [&](int u, const std::string& ind) {
      const std::string su = "_" + std::to_string(u);
      e.o << ind << "{\n";
      for (int k = rank - 1; k >= kr; --k) e.o << ind << "  const long long i" << k << " = i" << k << su << "; (void)i" << k << ";\n";
      for (int c4 = 0; c4 < 4; ++c4) {
        const std::string pre = "v" + std::to_string(c4) + "_";
        emit_scalar_program(e, g.prog, {ph.value},
                            [&](const Instr& in, int id) {
                              const AccessGroup& ag = g.groups[in.group];
                              if (ag.structural_zero[kd]) return "u" + std::to_string(id) + su;
                              return "w" + std::to_string(id) + su + "[" + std::to_string(c4) + "]";
                            },
                            "0.0f", pre, ind + "  ");
        const std::string a = c4 == 0 ? "acc" : "acc" + std::to_string(c4);
        e.o << ind << "  " << a << " = " << Em::combine(ph, a, pre + std::to_string(ph.value)) << ";\n";
      }
      e.o << ind << "}\n";
    };
    e.o << "  long long j = jbeg;\n  for (; j + 4 <= jend; j += 4) {\n";
    for (int u = 0; u < 4; ++u) loads0(u, "    ");
    e.o << "    __builtin_amdgcn_sched_barrier(0);\n";
    for (int u = 0; u < 4; ++u) compute0(u, "    ");
    e.o << "  }\n  for (; j < jend; ++j) {\n";
    loads0(0, "    ");
    compute0(0, "    ");
    e.o << "  }\n";
    e.o << "  GM " << T << "* const dst = NSPLIT > 1 ? (GM " << T << "*)" << e.slot(e.L.extra + 2) << " + split * NOUT : (GM " << T << "*)" << e.slot(e.L.out) << ";\n";
    e.o << "  dst[o] = acc; dst[o + 1] = acc1; dst[o + 2] = acc2; dst[o + 3] = acc3;\n}\n";
  } else {
  if (vec) {
    const bool multi = rank > kr + 1;
    const char* jb = multi ? "jbeg4" : "jbeg";
    const char* je = multi ? "jend4" : "jend";
    e.o << "  long long j = " << jb << " + 4 * (long long)threadIdx.x;\n  {\n    " << T << " acc1 = acc, acc2 = acc, acc3 = acc;\n";
    // Four vector loads per array in flight: the loop body is written out four times here, all loads first, because the
    // compiler cannot unroll a loop with a remainder once the body holds a wave-wide vote (the math helpers' tests for
    // rare arguments), and one load in flight per lane leaves HBM waiting (measured on sum(sqrt(x)) over 2^27 elements).
    // Every accumulator still takes its elements in increasing order of j: the same sums as a loop of single steps.
    const int U = 4;
    auto emit_loads = [&](int u, const char* ind) {
      const std::string su = "_" + std::to_string(u), jx = "(j + " + std::to_string(1024 * u) + ")";
      if (multi) {
        e.o << ind << "long long jrem" << su << " = " << jx << ";\n";
        for (int k = rank - 1; k >= kr; --k) {
          if (k == kr) e.o << ind << "const long long i" << k << su << " = jrem" << su << ";\n";
          else e.o << ind << "const long long i" << k << su << " = gr_peel(jrem" << su << ", " << e.dim(k) << ");\n";
        }
      } else e.o << ind << "const long long i" << kr << su << " = " << jx << ";\n";
      for (size_t i = 0; i < g.prog.size(); ++i) {
        const Instr& in = g.prog[i];
        if (in.kind != IKind::LOAD) continue;
        const AccessGroup& ag = g.groups[in.group];
        std::ostringstream base;
        base << "p" << in.group << " + 0";
        for (int k = 0; k < kr; ++k) if (!ag.structural_zero[k] && in.delta[k]) base << " + " << in.delta[k] << " * " << e.coef(in.group, k);
        for (int k = kr; k < rank; ++k) {
          if (ag.structural_zero[k]) continue;
          if (k == rd) base << " + i" << k << su << " + " << in.delta[k];
          else base << " + (i" << k << su << " + " << in.delta[k] << ") * " << e.coef(in.group, k);
        }
        if (ag.structural_zero[rd]) e.o << ind << "const " << cty(in.dtype) << " u" << i << su << " = (" << base.str() << ")[0];\n";
        else e.o << ind << "const " << vty4(in.dtype) << " w" << i << su << " = " << e.ld(in.group, vty4(in.dtype), base.str()) << ";\n";
      }
    };
    auto emit_compute = [&](int u, const std::string& ind) {
      const std::string su = "_" + std::to_string(u);
      e.o << ind << "{\n";
      for (int k = rank - 1; k >= kr; --k) e.o << ind << "  const long long i" << k << " = i" << k << su << "; (void)i" << k << ";\n";
      for (int c4 = 0; c4 < 4; ++c4) {
        const std::string pre = "v" + std::to_string(c4) + "_";
        emit_scalar_program(e, g.prog, {ph.value},
                            [&](const Instr& in, int id) {
                              const AccessGroup& ag = g.groups[in.group];
                              if (ag.structural_zero[rd]) return "u" + std::to_string(id) + su;
                              return "w" + std::to_string(id) + su + "[" + std::to_string(c4) + "]";
                            },
                            "0.0f", pre, (ind + "  ").c_str());
        const std::string a = c4 == 0 ? "acc" : "acc" + std::to_string(c4);
        e.o << ind << "  " << a << " = " << Em::combine(ph, a, pre + std::to_string(ph.value)) << ";\n";
      }
      e.o << ind << "}\n";
    };
    e.o << "    for (; j + " << 4 + 1024 * (U - 1) << " <= " << je << "; j += " << 1024 * U << ") {\n";
    for (int u = 0; u < U; ++u) emit_loads(u, "      ");
    e.o << "      __builtin_amdgcn_sched_barrier(0);\n";   // (or the scheduler waits for the first load before it issues the others)
    for (int u = 0; u < U; ++u) emit_compute(u, "      ");
    e.o << "    }\n";
    e.o << "    for (; j + 4 <= " << je << "; j += 1024) {\n";
    emit_loads(0, "      ");
    emit_compute(0, "      ");
    e.o << "    }\n    acc = gr_comb0(gr_comb0(acc, acc1), gr_comb0(acc2, acc3));\n  }\n";
    e.o << "  for (; j < " << je << "; ++j) {\n";   // at most one lane still has (fewer than four) elements
  } else {
    // one element per step (of a thread, or of each of a workgroup's 256 threads): four steps written out with their
    // loads first, for the same reason as above; the accumulator takes the elements in the order of j
    const int STEP = g.red_mode == 0 ? 1 : 256;
    auto idx = [&](const std::string& su, const std::string& jx, const char* ind) {
      if (rank > kr) {
        e.o << ind << "long long jrem" << su << " = " << jx << ";\n";
        for (int k = rank - 1; k >= kr; --k) {
          if (k == kr) e.o << ind << "const long long i" << k << su << " = jrem" << su << ";\n";
          else e.o << ind << "const long long i" << k << su << " = gr_peel(jrem" << su << ", " << e.dim(k) << ");\n";
        }
      }
    };
    e.o << "  long long j = " << (g.red_mode == 0 ? "jbeg" : "jbeg + threadIdx.x") << ";\n  for (; j + " << 3 * STEP << " < jend; j += " << 4 * STEP << ") {\n";
    for (int u = 0; u < 4; ++u) {
      const std::string su = "_" + std::to_string(u);
      idx(su, "j + " + std::to_string(u * STEP), "    ");
      for (size_t i = 0; i < g.prog.size(); ++i) {
        const Instr& in = g.prog[i];
        if (in.kind != IKind::LOAD) continue;
        const AccessGroup& ag = g.groups[in.group];
        e.o << "    const " << cty(in.dtype) << " l" << i << su << " = p" << in.group << "[0";
        for (int k = 0; k < rank; ++k) {
          if (ag.structural_zero[k]) continue;
          if (k >= kr) e.o << " + (i" << k << su << " + " << in.delta[k] << ") * " << e.coef(in.group, k);
          else if (in.delta[k]) e.o << " + " << in.delta[k] << " * " << e.coef(in.group, k);
        }
        e.o << "];\n";
      }
    }
    e.o << "    __builtin_amdgcn_sched_barrier(0);\n";
    for (int u = 0; u < 4; ++u) {
      const std::string su = "_" + std::to_string(u);
      e.o << "    {\n";
      for (int k = rank - 1; k >= kr; --k) e.o << "      const long long i" << k << " = i" << k << su << "; (void)i" << k << ";\n";
      emit_scalar_program(e, g.prog, {ph.value}, [&](const Instr&, int id) { return "l" + std::to_string(id) + su; }, "0.0f", "t", "      ");
      e.o << "      acc = " << Em::combine(ph, "acc", "t" + std::to_string(ph.value)) << ";\n    }\n";
    }
    e.o << "  }\n  for (; j < jend; j += " << STEP << ") {\n";
  }
  if (rank > kr) {
    e.o << "    long long jrem = j;\n";
    for (int k = rank - 1; k >= kr; --k) {
      if (k == kr) e.o << "    const long long i" << k << " = jrem;\n";
      else e.o << "    const long long i" << k << " = gr_peel(jrem, " << e.dim(k) << ");\n";
    }
  }
  emit_scalar_program(e, g.prog, {ph.value},
                      [&](const Instr& in, int) {
                        const AccessGroup& ag = g.groups[in.group];
                        std::ostringstream s;
                        s << "p" << in.group << "[0";
                        for (int k = 0; k < rank; ++k) {
                          if (ag.structural_zero[k]) continue;
                          if (k >= kr) s << " + (i" << k << " + " << in.delta[k] << ") * " << e.coef(in.group, k);
                          else if (in.delta[k]) s << " + " << in.delta[k] << " * " << e.coef(in.group, k);
                        }
                        s << "]";
                        return s.str();
                      },
                      "0.0f", "t", "    ");
  e.o << "    acc = " << Em::combine(ph, "acc", "t" + std::to_string(ph.value)) << ";\n  }\n";
  e.o << "  GM " << T << "* const dst = NSPLIT > 1 ? (GM " << T << "*)" << e.slot(e.L.extra + 2) << " + split * NOUT : (GM " << T << "*)" << e.slot(e.L.out) << ";\n";
  if (g.red_mode == 1) {
    e.o << "  acc = gr_lanes0(acc);\n"
           "  " << T << "* const sm = (" << T << "*)gr_sm;\n"
           "  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = acc;\n"
           "  __syncthreads();\n"
           "  acc = gr_comb0(gr_comb0(sm[0], sm[1]), gr_comb0(sm[2], sm[3]));\n"
           "  if (threadIdx.x == 0) dst[o] = acc;\n";
  } else {
    e.o << "  dst[o] = acc;\n";
  }
  e.o << "}\n";
  }
  // Stage 2 (Section 3.2: "a separate kernel ... only uses the binary operation"): combines the
  // NSPLIT partial results of every output in a fixed order.
  kernel_head(e, kernel_name(g) + "_combine");
  e.o << "  const long long NOUT = " << e.S(e.L.extra) << ", NSPLIT = " << e.S(e.L.extra + 3) << ";\n";
  e.o << "  const GM " << T << "* const ws = (const GM " << T << "*)" << e.slot(e.L.extra + 2) << ";\n";
  e.o << "  GM " << T << "* const out = (GM " << T << "*)" << e.slot(e.L.out) << ";\n";
  e.o << "  __shared__ long long gr_sm[4];\n";
  e.o << "  if (NOUT >= 1024) {\n"
         "    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;\n"
         "    if (o < NOUT) {\n      " << T << " acc = ws[o];\n"
         "      long long s = 1;\n"
         "      for (; s + 8 <= NSPLIT; s += 8) {\n"   // eight independent loads in flight, combined in the fixed order
         "        const " << T << " v0 = ws[s * NOUT + o], v1 = ws[(s + 1) * NOUT + o], v2 = ws[(s + 2) * NOUT + o], v3 = ws[(s + 3) * NOUT + o];\n"
         "        const " << T << " v4 = ws[(s + 4) * NOUT + o], v5 = ws[(s + 5) * NOUT + o], v6 = ws[(s + 6) * NOUT + o], v7 = ws[(s + 7) * NOUT + o];\n"
         "        acc = gr_comb0(gr_comb0(gr_comb0(gr_comb0(gr_comb0(gr_comb0(gr_comb0(gr_comb0(acc, v0), v1), v2), v3), v4), v5), v6), v7);\n"
         "      }\n"
         "      for (; s < NSPLIT; ++s) acc = gr_comb0(acc, ws[s * NOUT + o]);\n"
         "      out[o] = acc;\n    }\n"
         "  } else {\n"
         "    const long long o = blockIdx.x;\n    " << T << " acc = " << Em::identity(ph) << ";\n"
         "    for (long long s = threadIdx.x; s < NSPLIT; s += 256) acc = gr_comb0(acc, ws[s * NOUT + o]);\n"
         "    acc = gr_lanes0(acc);\n"
         "    " << T << "* sm = (" << T << "*)gr_sm;\n"
         "    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = acc;\n"
         "    __syncthreads();\n"
         "    if (threadIdx.x == 0) out[o] = gr_comb0(gr_comb0(sm[0], sm[1]), gr_comb0(sm[2], sm[3]));\n"
         "  }\n}\n";
}

// ---- SCAN (map-scan) ------------------------------------------------------------

// Inclusive scan of the mapped values along the last iteration dimension.
//   mode 0: the scanned axis is contiguous.  A workgroup walks one chunk of one line in tiles
//           of 1024 elements: four elements per lane, a shuffle scan across the wave, 32 bytes
//           of LDS across the four waves, a running carry between tiles.  Lines longer than
//           one chunk take three kernels: chunk totals, an exclusive scan of the totals, the
//           chunks again with their offsets (reduce-then-scan).
//   mode 1: a thread per line, sequential along the axis (consecutive threads touch
//           consecutive addresses when an inner dimension is contiguous).
void gen_scan(Em& e) {
  const GroupPlan& g = e.g;
  const int rank = g.rank, sd = rank - 1;
  const Phase& ph = g.phases[0];
  const char* TA = cty(ph.out_dtype);  // accumulator = output type (f32, i32 for extrema, i64 for i32 sums)
  prelude(e);
  phase_helpers(e, 0, 64);
  e.o << "static __device__ __forceinline__ float gr_up(float v, int d) { return __shfl_up(v, d, 64); }\n"
         "static __device__ __forceinline__ int gr_up(int v, int d) { return __shfl_up(v, d, 64); }\n"
         "static __device__ __forceinline__ long long gr_up(long long v, int d) {\n"
         "  int lo = __shfl_up((int)(v & 0xffffffffll), d, 64), hi = __shfl_up((int)(v >> 32), d, 64);\n"
         "  return ((long long)hi << 32) | (unsigned int)lo;\n}\n";
  const std::string ident = Em::identity(ph);
  auto conv = [&](const std::string& x) { return ph.out_dtype == GR_I64 && ph.in_dtype == GR_I32 ? "(long long)" + x : x; };
  auto load_at = [&](const std::string& col) {
    return [&e, &g, sd, col](const Instr& in, int) {
      const AccessGroup& ag = g.groups[in.group];
      std::ostringstream s;
      s << "p" << in.group << "[0";
      for (int k = 0; k < sd; ++k) if (!ag.structural_zero[k] && in.delta[k]) s << " + " << in.delta[k] << " * " << e.coef(in.group, k);
      if (!ag.structural_zero[sd]) s << " + (" << col << " + " << in.delta[sd] << ") * " << e.coef(in.group, sd);
      s << "]";
      return s.str();
    };
  };
  // common head: line index -> pointers
  auto head = [&](int per_block_line) {
    // (the chunk-count slot of a one-pass scan carries the poll limit in its upper half)
    // (one-pass scans: the chunk slot carries, in its upper half, the tag that marks a cell as published by this launch)
    if (g.scan_mode >= 2) e.o << "  const long long LINES = " << e.S(e.L.extra) << ", CH = " << e.S(e.L.extra + 1) << " & 0xffffffffll, NCHUNK = " << e.S(e.L.extra + 3) << " & 0xffffffffll;\n"
                                 "  const unsigned EPOCH = (unsigned)(" << e.slot(e.L.extra + 1) << " >> 32);\n";
    else e.o << "  const long long LINES = " << e.S(e.L.extra) << ", CH = " << e.S(e.L.extra + 1) << ", NCHUNK = " << e.S(e.L.extra + 3) << " & 0xffffffffll;\n";
    e.o << "  const long long L = " << e.dim(sd) << ";\n";
    if (per_block_line == 2) {
      // a workgroup per tile of W neighbouring lines: consecutive workgroups take neighbouring
      // column blocks, all tiles of one position along the axis before the next
      const int LX = g.BX, W = 4 * g.BX;
      e.o << "  const long long D = " << e.dim(sd - 1) << ", NCB = (D + " << W - 1 << ") / " << W << ", NCHAIN = (LINES / D) * NCB;\n"
             "  const long long chain = blockIdx.x % NCHAIN, chunk = blockIdx.x / NCHAIN;\n"
             "  const long long cb = chain % NCB;\n"
             "  const int lx = threadIdx.x % " << LX << ", ly = threadIdx.x / " << LX << ";\n"
             "  const bool colok = cb * " << W << " + lx * 4 < D;\n"
             "  const long long line = (chain / NCB) * D + (colok ? cb * " << W << " + lx * 4 : 0);\n";
    }
    else if (per_block_line) e.o << "  const long long line = blockIdx.x / NCHUNK, chunk = blockIdx.x % NCHUNK;\n";
    else if (g.scan_vec) e.o << "  const long long gt = (long long)blockIdx.x * 256 + threadIdx.x;\n  if (gt >= (LINES / 4) * NCHUNK) return;\n"
                "  const long long line = 4 * (gt % (LINES / 4)), chunk = gt / (LINES / 4);\n  (void)chunk;\n";  // four lines per thread
    else e.o << "  const long long gt = (long long)blockIdx.x * 256 + threadIdx.x;\n  if (gt >= LINES * NCHUNK) return;\n"
                "  const long long line = gt % LINES, chunk = gt / LINES;\n  (void)chunk;\n";  // neighbouring threads: neighbouring lines
    e.o << "  long long lrem = line;\n";
    for (int k = sd - 1; k >= 0; --k) {
      if (k == 0) e.o << "  const long long i0 = lrem;\n";
      else e.o << "  const long long i" << k << " = gr_peel(lrem, " << e.dim(k) << ");\n";
    }
    group_pointers(e, "  ");
    for (size_t gi = 0; gi < g.groups.size(); ++gi) {
      const AccessGroup& ag = g.groups[gi];
      e.o << "  const GM " << cty(ag.dtype) << "* const p" << gi << " = q" << gi;
      for (int k = 0; k < sd; ++k) if (!ag.structural_zero[k]) e.o << " + i" << k << " * " << e.coef((int)gi, k);
      e.o << ";\n";
    }
    e.o << "  GM " << TA << "* const po = (GM " << TA << "*)" << e.slot(e.L.out);
    for (int k = 0; k < sd; ++k) e.o << " + i" << k << " * " << e.S(e.L.ocoef + k);
    e.o << ";\n";
    e.o << "  GM " << TA << "* const ws = (GM " << TA << "*)" << e.slot(e.L.extra + 2) << ";\n  (void)ws; (void)CH; (void)po; (void)L;\n";
  };

  // mode 0: the four elements a lane owns in a tile, fetched with one dwordx4 where the tile is
  // full (the scanned axis is contiguous for every access that follows it)
  auto tile_loads = [&](const std::string& ind) {
    for (size_t i = 0; i < g.prog.size(); ++i) {
      const Instr& in = g.prog[i];
      if (in.kind != IKind::LOAD) continue;
      const AccessGroup& ag = g.groups[in.group];
      std::ostringstream base;
      base << "p" << in.group;
      for (int k = 0; k < sd; ++k) if (!ag.structural_zero[k] && in.delta[k]) base << " + " << in.delta[k] << " * " << e.coef(in.group, k);
      e.o << ind << cty(in.dtype) << " l" << i << "[4];\n";
      if (ag.structural_zero[sd]) {
        e.o << ind << "for (int j = 0; j < 4; ++j) l" << i << "[j] = (" << base.str() << ")[0];\n";
      } else if (in.dtype == GR_I64) {
        e.o << ind << "for (int j = 0; j < 4; ++j) l" << i << "[j] = (c + j < cend) ? (" << base.str() << ")[c + j + " << in.delta[sd] << "] : 0;\n";
      } else {
        e.o << ind << "if (c + 4 <= cend) { const " << vty4(in.dtype) << " w = " << e.ld(in.group, vty4(in.dtype), base.str() + " + c + " + std::to_string(in.delta[sd]))
            << "; l" << i << "[0] = w[0]; l" << i << "[1] = w[1]; l" << i << "[2] = w[2]; l" << i << "[3] = w[3]; }\n";
        e.o << ind << "else { for (int j = 0; j < 4; ++j) l" << i << "[j] = (c + j < cend) ? (" << base.str() << ")[c + j + " << in.delta[sd] << "] : " << Em::zero(in.dtype) << "; }\n";
      }
    }
  };
  auto tile_value = [](const Instr&, int id) { return "l" + std::to_string(id) + "[j]"; };

  // ---- kernel 2 of 3 (both modes): exclusive scan of each line's chunk totals, in place (at most 4096 chunks)
  auto offsets_kernel = [&]() {
    kernel_head(e, "gr_scan_offsets");
    e.o << "  const long long NCHUNK = " << e.S(e.L.extra + 3) << ";\n";
    e.o << "  GM " << TA << "* const w = (GM " << TA << "*)" << e.slot(e.L.extra + 2) << " + (long long)blockIdx.x * NCHUNK;\n";
    e.o << "  __shared__ long long gr_sm[4];\n";
    e.o << "  const int per = (int)((NCHUNK + 255) / 256);\n  const long long c0 = (long long)threadIdx.x * per;\n";
    e.o << "  " << TA << " v[16];\n  " << TA << " tot = " << ident << ";\n";
    e.o << "  for (int u = 0; u < 16; ++u) { v[u] = (u < per && c0 + u < NCHUNK) ? w[c0 + u] : " << ident << "; tot = gr_comb0(tot, v[u]); }\n";
    e.o << "  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;\n  " << TA << " x = tot;\n";
    for (int d = 1; d < 64; d <<= 1) e.o << "  { const " << TA << " y = gr_up(x, " << d << "); if (lane >= " << d << ") x = gr_comb0(y, x); }\n";
    e.o << "  " << TA << "* sm = (" << TA << "*)gr_sm;\n  if (lane == 63) sm[wave] = x;\n  __syncthreads();\n";
    e.o << "  " << TA << " off = " << ident << ";\n  for (int q = 0; q < wave; ++q) off = gr_comb0(off, sm[q]);\n";
    e.o << "  " << TA << " ex = gr_up(x, 1);\n  if (lane == 0) ex = " << ident << ";\n  off = gr_comb0(off, ex);\n";
    e.o << "  for (int u = 0; u < 16; ++u) if (u < per && c0 + u < NCHUNK) { w[c0 + u] = off; off = gr_comb0(off, v[u]); }\n}\n";
  };

  // Mode 1 walks a line sequentially; the running value makes every step depend on the one before,
  // and in the scan kernel the store of a step may alias the next load as far as the compiler
  // knows, so left alone each step waits for its own load.  The steps are therefore taken U at a
  // time: all loads of a batch first, then the U combines (and stores); a scalar loop finishes
  // the chunk.
  const int U = g.prog.size() <= 16 ? 8 : (g.prog.size() <= 48 ? 4 : 2);
  if (g.scan_mode == 1 && g.scan_vec) {
    // four neighbouring lines per thread: one dwordx4 per array and step
    const int ld = sd - 1;
    auto loads = [&](const std::string& jx, const std::string& sfx, const std::string& ind) {
      for (size_t i = 0; i < g.prog.size(); ++i) {
        const Instr& in = g.prog[i];
        if (in.kind != IKind::LOAD) continue;
        const AccessGroup& ag = g.groups[in.group];
        std::ostringstream at;
        at << "p" << in.group << " + 0";
        for (int k = 0; k < sd; ++k) if (!ag.structural_zero[k] && in.delta[k]) at << " + " << in.delta[k] << (k == ld ? std::string("") : " * " + e.coef(in.group, k));
        if (!ag.structural_zero[sd]) at << " + (" << jx << " + " << in.delta[sd] << ") * " << e.coef(in.group, sd);
        if (ag.structural_zero[ld]) e.o << ind << "const " << cty(in.dtype) << " u" << i << sfx << " = (" << at.str() << ")[0];\n";
        else e.o << ind << "const " << vty4(in.dtype) << " w" << i << sfx << " = " << e.ld(in.group, vty4(in.dtype), at.str()) << ";\n";
      }
    };
    auto step = [&](const std::string& jx, const std::string& sfx, const std::string& ind, bool store) {
      for (int c4 = 0; c4 < 4; ++c4) {
        const std::string pre = "v" + std::to_string(c4) + sfx + "_";
        emit_scalar_program(e, g.prog, {ph.value},
                            [&](const Instr& in, int id) {
                              const AccessGroup& ag = g.groups[in.group];
                              if (ag.structural_zero[ld]) return "u" + std::to_string(id) + sfx;
                              return "w" + std::to_string(id) + sfx + "[" + std::to_string(c4) + "]";
                            },
                            "0.0f", pre, ind);
        e.o << ind << "acc" << c4 << " = " << Em::combine(ph, "acc" + std::to_string(c4), pre + std::to_string(ph.value)) << ";\n";
      }
      if (store) {
        if (ph.out_dtype == GR_I64)
          e.o << ind << "po[(" << jx << ") * ostep] = acc0; po[(" << jx << ") * ostep + 1] = acc1; po[(" << jx << ") * ostep + 2] = acc2; po[(" << jx << ") * ostep + 3] = acc3;\n";
        else {
          const char* vt = ph.out_dtype == GR_F32 ? "f4u" : "i4u";
          e.o << ind << "{ " << vt << " ov; ov[0] = acc0; ov[1] = acc1; ov[2] = acc2; ov[3] = acc3; *(GM " << vt << "*)(po + (" << jx << ") * ostep) = ov; }\n";
        }
      }
    };
    auto walk = [&](bool store) {
      e.o << "  long long j = cbeg;\n  for (; j + " << U << " <= cend; j += " << U << ") {\n";
      for (int u = 0; u < U; ++u) loads("j + " + std::to_string(u), "_" + std::to_string(u), "    ");
      for (int u = 0; u < U; ++u) { e.o << "    {\n"; step("j + " + std::to_string(u), "_" + std::to_string(u), "      ", store); e.o << "    }\n"; }
      e.o << "  }\n  for (; j < cend; ++j) {\n";
      loads("j", "", "    ");
      step("j", "", "    ", store);
      e.o << "  }\n";
    };
    kernel_head(e, "gr_scan_sums");
    head(false);
    e.o << "  const long long cbeg = chunk * CH, cend = (cbeg + CH < L) ? cbeg + CH : L;\n  " << TA << " acc0 = " << ident << ", acc1 = acc0, acc2 = acc0, acc3 = acc0;\n";
    walk(false);
    e.o << "  ws[line * NCHUNK + chunk] = acc0; ws[(line + 1) * NCHUNK + chunk] = acc1; ws[(line + 2) * NCHUNK + chunk] = acc2; ws[(line + 3) * NCHUNK + chunk] = acc3;\n}\n";
    offsets_kernel();
    kernel_head(e, "gr_scan");
    head(false);
    e.o << "  const long long cbeg = chunk * CH, cend = (cbeg + CH < L) ? cbeg + CH : L;\n";
    e.o << "  const long long ostep = " << e.S(e.L.ocoef + sd) << ";\n";
    e.o << "  " << TA << " acc0 = " << ident << ", acc1 = acc0, acc2 = acc0, acc3 = acc0;\n";
    e.o << "  if (NCHUNK > 1) { acc0 = ws[line * NCHUNK + chunk]; acc1 = ws[(line + 1) * NCHUNK + chunk]; acc2 = ws[(line + 2) * NCHUNK + chunk]; acc3 = ws[(line + 3) * NCHUNK + chunk]; }\n";
    walk(true);
    e.o << "}\n";
    return;
  }
  if (g.scan_mode == 1) {
    // a thread per (line, chunk), sequential along the axis; with several chunks per line the same
    // three steps as in mode 0: chunk totals, exclusive scan of the totals, chunks with offsets
    auto walk = [&](bool store) {
      e.o << "  long long j = cbeg;\n  for (; j + " << U << " <= cend; j += " << U << ") {\n";
      // the loads of the whole batch first (a load's value is named <prefix><id>)
      for (int u = 0; u < U; ++u) {
        const std::string pre = "t" + std::to_string(u) + "_";
        for (size_t i = 0; i < g.prog.size(); ++i) {
          if (g.prog[i].kind != IKind::LOAD) continue;
          e.o << "    const " << cty(g.prog[i].dtype) << ' ' << pre << i << " = " << load_at("(j + " + std::to_string(u) + ")")(g.prog[i], (int)i) << ";\n";
        }
      }
      for (int u = 0; u < U; ++u) {
        const std::string pre = "t" + std::to_string(u) + "_";
        std::vector<char> have(g.prog.size(), 0);
        for (size_t i = 0; i < g.prog.size(); ++i) if (g.prog[i].kind == IKind::LOAD) have[i] = 1;
        e.o << "    {\n";
        emit_scalar_program(e, g.prog, {ph.value}, load_at("j"), "0.0f", pre, "      ", &have);
        e.o << "      acc = " << Em::combine(ph, "acc", pre + std::to_string(ph.value)) << ";\n";
        if (store) e.o << "      po[(j + " << u << ") * ostep] = acc;\n";
        e.o << "    }\n";
      }
      e.o << "  }\n  for (; j < cend; ++j) {\n";
      emit_scalar_program(e, g.prog, {ph.value}, load_at("j"), "0.0f", "t", "    ");
      e.o << "    acc = " << Em::combine(ph, "acc", "t" + std::to_string(ph.value)) << ";\n";
      if (store) e.o << "    po[j * ostep] = acc;\n";
      e.o << "  }\n";
    };
    kernel_head(e, "gr_scan_sums");
    head(false);
    e.o << "  const long long cbeg = chunk * CH, cend = (cbeg + CH < L) ? cbeg + CH : L;\n  " << TA << " acc = " << ident << ";\n";
    walk(false);
    e.o << "  ws[line * NCHUNK + chunk] = acc;\n}\n";
    offsets_kernel();
    kernel_head(e, "gr_scan");
    head(false);
    e.o << "  const long long cbeg = chunk * CH, cend = (cbeg + CH < L) ? cbeg + CH : L;\n";
    e.o << "  const long long ostep = " << e.S(e.L.ocoef + sd) << ";\n  " << TA << " acc = NCHUNK > 1 ? ws[line * NCHUNK + chunk] : " << ident << ";\n";
    walk(true);
    e.o << "}\n";
    return;
  }


  if (g.scan_mode == 3) {
    // ---- mode 3: a scan along a non-contiguous axis with few lines, in ONE pass over the input.
    // A workgroup owns a tile of R positions along the scanned axis by W = 4*BX neighbouring lines
    // (the innermost line dimension is contiguous): BX lanes across the lines, each with four of
    // them, LY = 256/BX lane groups along the axis, RPL consecutive positions per lane, one vector
    // load per array and position.  The tile stays in registers: every lane scans its positions,
    // the lane groups exchange their totals through LDS, the tile's totals (one per line) are
    // published, and the offsets come from the tiles before it on the same lines.  Tiles of a
    // chain (the same W lines) form groups of G; the last tile of a group also publishes the group's
    // totals.  A line's offset in tile k of group q is
    //     fold(totals of groups 0..q-1, then of the tiles of group q before k),
    // taken by 256/W lanes per line in a fixed interleaved pattern and combined in lane order, so
    // the association, and with it every float result, depends on the shape only.  Cells are
    // 8-byte words (valid bit, value) written and read with relaxed agent-scope atomics; waits are
    // bounded, and a workgroup that runs out of polls takes its offsets from the input itself, so
    // every wave terminates whatever order tiles are dispatched in.  A small kernel clears the
    // cells before every launch.
    const int LX = g.BX, W = 4 * LX, LY = 256 / LX, RPL = (int)(g.scan_chunk / LY), R = (int)g.scan_chunk, P = 256 / W;
    const int ld = sd - 1;
    const char* V4 = ph.out_dtype == GR_F32 ? "f4" : "i4";
    const std::string bits = ph.out_dtype == GR_F32 ? "__float_as_uint" : "(unsigned)";
    const std::string unbits = ph.out_dtype == GR_F32 ? "__uint_as_float" : "(int)";
    kernel_head(e, "gr_scan_clear");
    e.o << "  const long long LINES = " << e.S(e.L.extra) << ", G = " << e.S(e.L.extra + 1) << " & 0xffffffffll, NCHUNK = " << e.S(e.L.extra + 3) << " & 0xffffffffll;\n"
           "  const long long D = " << e.dim(ld) << ", NCHAIN = (LINES / D) * ((D + " << W - 1 << ") / " << W << ");\n"
           "  const long long n = NCHAIN * (NCHUNK + (NCHUNK + G - 1) / G) * " << W << ";\n"
           "  GM unsigned long long* const w = (GM unsigned long long*)" << e.slot(e.L.extra + 2) << ";\n"
           "  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;\n  if (i < n) w[i] = 0ull;\n}\n";
    e.o << "static __device__ __forceinline__ unsigned long long gr_poll(GM unsigned long long* p, unsigned& polls, const unsigned tag) {\n"
           "  unsigned long long w = __hip_atomic_load((unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n"
           "  while ((unsigned)(w >> 32) != tag && polls) { __builtin_amdgcn_s_sleep(2); --polls; w = __hip_atomic_load((unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }\n"
           "  return w;\n}\n";
    kernel_head(e, "gr_scan");
    head(2);
    e.o << "  const long long G = CH;\n";
    e.o << "  __shared__ " << V4 << " gr_sm[" << LY << "][" << LX << "];\n  __shared__ " << TA << " gr_part[256];\n  __shared__ " << TA << " gr_base[" << W << "];\n";
    e.o << "  const long long cbeg = chunk * " << R << ", j0 = cbeg + ly * " << RPL << ";\n";
    e.o << "  const long long ostep = " << e.S(e.L.ocoef + sd) << ";\n";
    e.o << "  " << TA << " v[" << RPL << "][4];\n";
    // the values of the mapped expression at position jx of the lane's four lines
    auto loads = [&](const std::string& jx, const std::string& sfx, const std::string& ind) {
      for (size_t i = 0; i < g.prog.size(); ++i) {
        const Instr& in = g.prog[i];
        if (in.kind != IKind::LOAD) continue;
        const AccessGroup& ag = g.groups[in.group];
        std::ostringstream at;
        at << "p" << in.group << " + 0";
        for (int k = 0; k < sd; ++k) if (!ag.structural_zero[k] && in.delta[k]) at << " + " << in.delta[k] << (k == ld ? std::string("") : " * " + e.coef(in.group, k));
        if (!ag.structural_zero[sd]) at << " + (" << jx << " + " << in.delta[sd] << ") * " << e.coef(in.group, sd);
        if (ag.structural_zero[ld]) e.o << ind << "const " << cty(in.dtype) << " u" << i << sfx << " = (" << at.str() << ")[0];\n";
        else e.o << ind << "const " << vty4(in.dtype) << " w" << i << sfx << " = " << e.ld(in.group, vty4(in.dtype), at.str()) << ";\n";
      }
    };
    auto values = [&](const std::string& sfx, const std::string& ind, const std::function<std::string(int)>& dst) {
      for (int c4 = 0; c4 < 4; ++c4) {
        const std::string pre = "t" + std::to_string(c4) + sfx + "_";
        emit_scalar_program(e, g.prog, {ph.value},
                            [&](const Instr& in, int id) {
                              const AccessGroup& ag = g.groups[in.group];
                              if (ag.structural_zero[ld]) return "u" + std::to_string(id) + sfx;
                              return "w" + std::to_string(id) + sfx + "[" + std::to_string(c4) + "]";
                            },
                            "0.0f", pre, ind);
        e.o << ind << dst(c4) << " = " << pre << ph.value << ";\n";
      }
    };
    // the whole tile first: RPL vector loads per array in flight per lane; a tile inside the array
    // takes straight-line code without bounds checks
    e.o << "  const bool whole = cbeg + " << R << " <= L && (cb + 1) * " << W << " <= D;\n";
    e.o << "  if (whole) {\n";
    for (int u = 0; u < RPL; ++u) loads("j0 + " + std::to_string(u), "_" + std::to_string(u), "    ");
    for (int u = 0; u < RPL; ++u) { e.o << "    {\n"; values("_" + std::to_string(u), "      ", [&](int c4) { return "v[" + std::to_string(u) + "][" + std::to_string(c4) + "]"; }); e.o << "    }\n"; }
    e.o << "  } else {\n#pragma unroll\n    for (int u = 0; u < " << RPL << "; ++u) {\n"
           "      v[u][0] = v[u][1] = v[u][2] = v[u][3] = " << ident << ";\n"
           "      if (colok && j0 + u < L) {\n";
    loads("j0 + u", "", "        ");
    values("", "        ", [&](int c4) { return "v[u][" + std::to_string(c4) + "]"; });
    e.o << "      }\n    }\n  }\n";
    // scan inside the tile: down a lane's positions, then the lane groups through LDS
    e.o << "#pragma unroll\n  for (int u = 1; u < " << RPL << "; ++u)\n#pragma unroll\n    for (int c = 0; c < 4; ++c) v[u][c] = gr_comb0(v[u - 1][c], v[u][c]);\n";
    e.o << "  { " << V4 << " t; t[0] = v[" << RPL - 1 << "][0]; t[1] = v[" << RPL - 1 << "][1]; t[2] = v[" << RPL - 1 << "][2]; t[3] = v[" << RPL - 1 << "][3]; gr_sm[ly][lx] = t; }\n"
           "  __syncthreads();\n";
    e.o << "  " << TA << " off[4] = {" << ident << ", " << ident << ", " << ident << ", " << ident << "};\n"
           "  for (int q = 0; q < ly; ++q) { const " << V4 << " t = gr_sm[q][lx];\n#pragma unroll\n    for (int c = 0; c < 4; ++c) off[c] = gr_comb0(off[c], t[c]); }\n";
    // publish the tile's totals, one cell per line
    e.o << "  const long long NGROUP = (NCHUNK + G - 1) / G, grp = chunk / G, gfirst = grp * G;\n"
           "  GM unsigned long long* const wq = (GM unsigned long long*)" << e.slot(e.L.extra + 2) << ";\n"
           "  GM unsigned long long* const wa = wq + chain * NCHUNK * " << W << ";\n"
           "  GM unsigned long long* const wg = wq + NCHAIN * NCHUNK * " << W << " + chain * NGROUP * " << W << ";\n"
           "  if (threadIdx.x < " << W << ") {\n    " << TA << " tot = " << ident << ";\n"
           "    for (int q = 0; q < " << LY << "; ++q) tot = gr_comb0(tot, ((" << TA << "*)gr_sm)[q * " << W << " + threadIdx.x]);\n"
           "    __hip_atomic_store((unsigned long long*)(wa + chunk * " << W << " + threadIdx.x), ((unsigned long long)EPOCH << 32) | " << bits << "(tot), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n  }\n"
           "  unsigned polls = (unsigned)(" << e.slot(e.L.extra + 3) << " >> 32);\n  int lost = 0;\n"
           "  if (chunk == gfirst + G - 1 && threadIdx.x < " << W << ") {\n"
           "    // last tile of a full group: the group's totals, for every later group\n"
           "    " << TA << " acc = " << ident << ";\n"
           "    for (long long q = gfirst; q < gfirst + G; q += 4) {\n      unsigned long long w[4];\n"
           "#pragma unroll\n      for (int b = 0; b < 4; ++b) w[b] = __hip_atomic_load((unsigned long long*)(wa + (q + b) * " << W << " + threadIdx.x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n"
           "#pragma unroll\n      for (int b = 0; b < 4; ++b) {\n"
           "        if ((unsigned)(w[b] >> 32) != EPOCH) w[b] = gr_poll(wa + (q + b) * " << W << " + threadIdx.x, polls, EPOCH);\n"
           "        if ((unsigned)(w[b] >> 32) == EPOCH) acc = gr_comb0(acc, " << unbits << "((unsigned)w[b])); else lost = 1;\n      }\n    }\n"
           "    if (!lost) __hip_atomic_store((unsigned long long*)(wg + grp * " << W << " + threadIdx.x), ((unsigned long long)EPOCH << 32) | " << bits << "(acc), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n"
           "  }\n"
           "  {\n    const int col = threadIdx.x % " << W << ", part = threadIdx.x / " << W << ";\n"
           "    const long long n = grp + (chunk - gfirst);\n    " << TA << " acc = " << ident << ";\n"
           "    // (four cells asked for at a time: their latencies overlap; combined in index order all the same)\n"
           "    for (long long i = part; i < n; i += " << 4 * P << ") {\n"
           "      GM unsigned long long* cell[4];\n      unsigned long long w[4];\n"
           "#pragma unroll\n      for (int b = 0; b < 4; ++b) {\n        const long long ib = i + b * " << P << ";\n"
           "        cell[b] = ib < grp ? wg + ib * " << W << " + col : wa + (gfirst + ib - grp) * " << W << " + col;\n"
           "        w[b] = ib < n ? __hip_atomic_load((unsigned long long*)cell[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;\n      }\n"
           "#pragma unroll\n      for (int b = 0; b < 4; ++b) if (i + b * " << P << " < n) {\n"
           "        if ((unsigned)(w[b] >> 32) != EPOCH) w[b] = gr_poll(cell[b], polls, EPOCH);\n"
           "        if ((unsigned)(w[b] >> 32) == EPOCH) acc = gr_comb0(acc, " << unbits << "((unsigned)w[b])); else lost = 1;\n      }\n    }\n"
           "    gr_part[threadIdx.x] = acc;\n  }\n";
    e.o << "  if (__syncthreads_or(lost)) {\n"
           "    // out of polls: the offsets straight from the input (everything before this tile on its lines)\n"
           "    " << TA << " acc[4] = {" << ident << ", " << ident << ", " << ident << ", " << ident << "};\n"
           "    if (colok) for (long long j = ly; j < cbeg; j += " << LY << ") {\n      " << TA << " x[4];\n";
    loads("j", "", "      ");
    values("", "      ", [&](int c4) { return "x[" + std::to_string(c4) + "]"; });
    e.o << "#pragma unroll\n      for (int c = 0; c < 4; ++c) acc[c] = gr_comb0(acc[c], x[c]);\n    }\n"
           "    { " << V4 << " t; t[0] = acc[0]; t[1] = acc[1]; t[2] = acc[2]; t[3] = acc[3]; gr_sm[ly][lx] = t; }\n"
           "    __syncthreads();\n"
           "    if (threadIdx.x < " << W << ") {\n      " << TA << " b = " << ident << ";\n"
           "      for (int q = 0; q < " << LY << "; ++q) b = gr_comb0(b, ((" << TA << "*)gr_sm)[q * " << W << " + threadIdx.x]);\n"
           "      gr_base[threadIdx.x] = b;\n    }\n"
           "  } else if (threadIdx.x < " << W << ") {\n    " << TA << " b = gr_part[threadIdx.x];\n";
    for (int q = 1; q < P; ++q) e.o << "    b = gr_comb0(b, gr_part[" << q * W << " + threadIdx.x]);\n";
    e.o << "    gr_base[threadIdx.x] = b;\n  }\n  __syncthreads();\n";
    e.o << "#pragma unroll\n  for (int c = 0; c < 4; ++c) off[c] = gr_comb0(gr_base[lx * 4 + c], off[c]);\n";
    {
      const char* vt = ph.out_dtype == GR_F32 ? "f4u" : "i4u";
      const std::string st = (g.nt & 8) ? "__builtin_nontemporal_store(ov, (GM " + std::string(vt) + "*)(po + (j0 + u) * ostep))" : "*(GM " + std::string(vt) + "*)(po + (j0 + u) * ostep) = ov";
      e.o << "  if (whole) {\n#pragma unroll\n    for (int u = 0; u < " << RPL << "; ++u) {\n"
             "      " << vt << " ov; for (int c = 0; c < 4; ++c) ov[c] = gr_comb0(off[c], v[u][c]); " << st << ";\n    }\n    return;\n  }\n";
      e.o << "#pragma unroll\n  for (int u = 0; u < " << RPL << "; ++u) {\n"
             "    if (colok && j0 + u < L) { " << vt << " ov; for (int c = 0; c < 4; ++c) ov[c] = gr_comb0(off[c], v[u][c]); " << st << "; }\n  }\n}\n";
    }
    return;
  }

  if (g.scan_mode == 2) {
    // ---- mode 2: long contiguous lines in ONE pass over the input.  A workgroup owns a tile of TU x 1024
    // consecutive elements of a line, keeps it in registers, scans it, publishes the tile's total and
    // needs, before it may store, the combination of everything before its tile.  Tiles form groups
    // of 128; the last tile of a group also publishes the group's total.  A tile's offset is
    //     fold(totals of the earlier groups) (+) fold(totals of the earlier tiles of its own group),
    // each fold taken lane by lane in a fixed pattern, so the association -- and with it every float
    // result -- does not depend on timing.  A published cell is one 8-byte word (valid bit, value)
    // written and read with relaxed agent-scope atomics.  Waiting is bounded: a workgroup that runs
    // out of polls computes its offset from the input itself, so every wave terminates whatever order
    // the tiles are dispatched in (in dispatch order, which is what happens, everything a tile waits
    // for is already running).  A small kernel clears the cells before every launch.
    const int TU = (int)(g.scan_chunk / 1024);  // blocks of 1024 elements per tile
    const std::string bits = ph.out_dtype == GR_F32 ? "__float_as_uint" : "(unsigned)";
    const std::string unbits = ph.out_dtype == GR_F32 ? "__uint_as_float" : "(int)";
    kernel_head(e, "gr_scan_clear");
    e.o << "  const long long LINES = " << e.S(e.L.extra) << ", NCHUNK = " << e.S(e.L.extra + 3) << " & 0xffffffffll;\n"
           "  const long long n = LINES * NCHUNK + LINES * ((NCHUNK + 127) / 128);\n"   // one cell per tile and per group
           "  GM unsigned long long* const w = (GM unsigned long long*)" << e.slot(e.L.extra + 2) << ";\n"
           "  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;\n  if (i < n) w[i] = 0ull;\n}\n";
    // wave-wide inclusive scan with row shifts inside rows of 16 lanes and two row broadcasts; lanes without a source take the identity
    e.o << "#define GR_DPP(idn, v, ctrl, rmask) " << unbits << "((unsigned)__builtin_amdgcn_update_dpp((int)" << bits << "(idn), (int)" << bits << "(v), ctrl, rmask, 0xf, false))\n";
    e.o << "static __device__ __forceinline__ " << TA << " gr_wscan(" << TA << " x) {\n  const " << TA << " idn = " << ident << ";\n"
           "  x = gr_comb0(GR_DPP(idn, x, 0x111, 0xf), x);\n  x = gr_comb0(GR_DPP(idn, x, 0x112, 0xf), x);\n"
           "  x = gr_comb0(GR_DPP(idn, x, 0x114, 0xf), x);\n  x = gr_comb0(GR_DPP(idn, x, 0x118, 0xf), x);\n"
           "  x = gr_comb0(GR_DPP(idn, x, 0x142, 0xa), x);\n  x = gr_comb0(GR_DPP(idn, x, 0x143, 0xc), x);\n  return x;\n}\n";
    e.o << "static __device__ __forceinline__ unsigned long long gr_poll(GM unsigned long long* p, unsigned& polls, const unsigned tag) {\n"
           "  unsigned long long w = __hip_atomic_load((unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n"
           "  while ((unsigned)(w >> 32) != tag && polls) { __builtin_amdgcn_s_sleep(8); --polls; w = __hip_atomic_load((unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }\n"
           "  return w;\n}\n";
    e.o << "static __device__ __forceinline__ " << TA << " gr_fold(" << TA << " x, " << TA << "* f) {\n"
           "  x = gr_lanes0(x);\n  if ((threadIdx.x & 63) == 0) f[threadIdx.x >> 6] = x;\n  __syncthreads();\n"
           "  return gr_comb0(gr_comb0(f[0], f[1]), gr_comb0(f[2], f[3]));\n}\n";
    kernel_head(e, "gr_scan");
    head(true);
    e.o << "  __shared__ " << TA << " gr_wt[" << TU << "][4];\n  __shared__ " << TA << " gr_fs[4][4];\n";
    e.o << "  const long long cbeg = chunk * CH;\n  const int clen = (int)((cbeg + CH < L) ? CH : L - cbeg);\n";
    e.o << "  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;\n";
    e.o << "  " << TA << " v[" << TU << "][4];\n";
    // positions inside the tile are 32-bit offsets from the tile's first element (one 64-bit base per array)
    for (size_t gi = 0; gi < g.groups.size(); ++gi)
      e.o << "  const GM " << cty(g.groups[gi].dtype) << "* const tp" << gi << " = p" << gi << (g.groups[gi].structural_zero[sd] ? "" : " + cbeg") << ";\n";
    e.o << "  GM " << TA << "* const tpo = po + cbeg;\n";
    // the whole tile first: TU vector loads per array in flight per lane
    // (a full tile -- every tile of a line but the last -- takes straight-line code without bounds checks)
    e.o << "  const bool whole = clen == " << TU * 1024 << ";\n";
    e.o << "  if (whole) {\n    const int cend = " << TU * 1024 << ";\n";
    for (size_t gi = 0; gi < g.groups.size(); ++gi) e.o << "    const GM " << cty(g.groups[gi].dtype) << "* const p" << gi << " = tp" << gi << ";\n";
    e.o << "#pragma unroll\n    for (int u = 0; u < " << TU << "; ++u) {\n      const int c = u * 1024 + threadIdx.x * 4;\n";
    tile_loads("      ");
    e.o << "#pragma unroll\n      for (int j = 0; j < 4; ++j) {\n";
    emit_scalar_program(e, g.prog, {ph.value}, tile_value, "0.0f", "t", "        ");
    e.o << "        v[u][j] = " << conv("t" + std::to_string(ph.value)) << ";\n      }\n    }\n  } else {\n    const int cend = clen;\n";
    for (size_t gi = 0; gi < g.groups.size(); ++gi) e.o << "    const GM " << cty(g.groups[gi].dtype) << "* const p" << gi << " = tp" << gi << ";\n";
    e.o << "#pragma unroll\n    for (int u = 0; u < " << TU << "; ++u) {\n      const int c = u * 1024 + threadIdx.x * 4;\n";
    tile_loads("      ");
    e.o << "#pragma unroll\n      for (int j = 0; j < 4; ++j) {\n        v[u][j] = " << ident << ";\n        if (c + j < cend) {\n";
    emit_scalar_program(e, g.prog, {ph.value}, tile_value, "0.0f", "t", "          ");
    e.o << "          v[u][j] = " << conv("t" + std::to_string(ph.value)) << ";\n        }\n      }\n    }\n  }\n";
    // scan inside the tile: four elements of a lane, the lanes of a wave, then waves and blocks through LDS
    e.o << "  " << TA << " xs[" << TU << "];\n";
    e.o << "#pragma unroll\n  for (int u = 0; u < " << TU << "; ++u) {\n"
           "    v[u][1] = gr_comb0(v[u][0], v[u][1]); v[u][2] = gr_comb0(v[u][1], v[u][2]); v[u][3] = gr_comb0(v[u][2], v[u][3]);\n"
           "    xs[u] = gr_wscan(v[u][3]);\n    if (lane == 63) gr_wt[u][wave] = xs[u];\n  }\n  __syncthreads();\n";
    e.o << "  " << TA << " carry = " << ident << ";\n";
    e.o << "#pragma unroll\n  for (int u = 0; u < " << TU << "; ++u) {\n    " << TA << " b = carry;\n"
           "    for (int q = 0; q < wave; ++q) b = gr_comb0(b, gr_wt[u][q]);\n"
           "    { const " << TA << " ex = GR_DPP(" << ident << ", xs[u], 0x138, 0xf); if (lane != 0) b = gr_comb0(b, ex); }\n"
           "#pragma unroll\n    for (int j = 0; j < 4; ++j) v[u][j] = gr_comb0(b, v[u][j]);\n"
           "    carry = gr_comb0(carry, gr_comb0(gr_comb0(gr_wt[u][0], gr_wt[u][1]), gr_comb0(gr_wt[u][2], gr_wt[u][3])));\n  }\n";
    // publish, then collect the offset
    e.o << "  const long long NGROUP = (NCHUNK + 127) / 128, grp = chunk / 128, gfirst = grp * 128;\n"
           "  GM unsigned long long* const wq = (GM unsigned long long*)" << e.slot(e.L.extra + 2) << ";\n"
           "  GM unsigned long long* const wa = wq + line * NCHUNK;\n"
           "  GM unsigned long long* const wg = wq + LINES * NCHUNK + line * NGROUP;\n"
           "  if (threadIdx.x == 0) __hip_atomic_store((unsigned long long*)(wa + chunk), ((unsigned long long)EPOCH << 32) | " << bits << "(carry), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n"
           "  unsigned polls = (unsigned)(" << e.slot(e.L.extra + 3) << " >> 32);\n  int lost = 0;\n"
           "  if (chunk == gfirst + 127) {\n"
           "    // last tile of a full group: the group's total, for every later group\n"
           "    " << TA << " acc = " << ident << ";\n"
           "    if (threadIdx.x < 128) { const unsigned long long w = gr_poll(wa + gfirst + threadIdx.x, polls, EPOCH); if ((unsigned)(w >> 32) == EPOCH) acc = " << unbits << "((unsigned)w); else lost = 1; }\n"
           "    const " << TA << " tot = gr_fold(acc, gr_fs[0]);\n"
           "    if (!__syncthreads_or(lost) && threadIdx.x == 0) __hip_atomic_store((unsigned long long*)(wg + grp), ((unsigned long long)EPOCH << 32) | " << bits << "(tot), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);\n"
           "  }\n"
           "  " << TA << " p1 = " << ident << ", p2 = " << ident << ";\n"
           "  // (first the earlier groups, then the earlier tiles of this group: measured faster than waiting for both at once)\n"
           "  for (long long q = threadIdx.x; q < grp; q += 256) { const unsigned long long w = gr_poll(wg + q, polls, EPOCH); if ((unsigned)(w >> 32) == EPOCH) p1 = gr_comb0(p1, " << unbits << "((unsigned)w)); else lost = 1; }\n"
           "  for (long long q = gfirst + threadIdx.x; q < chunk; q += 256) { const unsigned long long w = gr_poll(wa + q, polls, EPOCH); if ((unsigned)(w >> 32) == EPOCH) p2 = gr_comb0(p2, " << unbits << "((unsigned)w)); else lost = 1; }\n"
           "  p1 = gr_fold(p1, gr_fs[1]);\n  p2 = gr_fold(p2, gr_fs[2]);\n"
           "  " << TA << " base = gr_comb0(p1, p2);\n"
           "  if (__syncthreads_or(lost)) {\n"
           "    // out of polls: the offset straight from the input (the whole line before this tile)\n"
           "    " << TA << " acc = " << ident << ";\n    const long long cend = cbeg;\n"
           "    for (long long t0 = 0; t0 < cbeg; t0 += 1024) {\n      const long long c = t0 + threadIdx.x * 4;\n";
    tile_loads("      ");
    e.o << "#pragma unroll\n      for (int j = 0; j < 4; ++j) {\n        if (c + j < cend) {\n";
    emit_scalar_program(e, g.prog, {ph.value}, tile_value, "0.0f", "t", "          ");
    e.o << "          acc = " << Em::combine(ph, "acc", "t" + std::to_string(ph.value)) << ";\n        }\n      }\n    }\n"
           "    base = gr_fold(acc, gr_fs[3]);\n  }\n";
    {
      const char* vt = ph.out_dtype == GR_F32 ? "f4u" : "i4u";
      const std::string st = (g.nt & 8) ? "__builtin_nontemporal_store(ov, (GM " + std::string(vt) + "*)(tpo + c))" : "*(GM " + std::string(vt) + "*)(tpo + c) = ov";
      e.o << "  if (whole) {\n#pragma unroll\n    for (int u = 0; u < " << TU << "; ++u) {\n      const int c = u * 1024 + threadIdx.x * 4;\n"
             "      " << vt << " ov; for (int j = 0; j < 4; ++j) ov[j] = gr_comb0(base, v[u][j]); " << st << ";\n    }\n    return;\n  }\n";
    }
    e.o << "#pragma unroll\n  for (int u = 0; u < " << TU << "; ++u) {\n    const int c = u * 1024 + threadIdx.x * 4;\n";
    {
      const char* vt = ph.out_dtype == GR_F32 ? "f4u" : "i4u";
      e.o << "    if (c + 4 <= clen) { " << vt << " ov; for (int j = 0; j < 4; ++j) ov[j] = gr_comb0(base, v[u][j]); "
          << ((g.nt & 8) ? "__builtin_nontemporal_store(ov, (GM " + std::string(vt) + "*)(tpo + c))" : "*(GM " + std::string(vt) + "*)(tpo + c) = ov") << "; }\n"
             "    else { for (int j = 0; j < 4; ++j) if (c + j < clen) tpo[c + j] = gr_comb0(base, v[u][j]); }\n  }\n}\n";
    }
    return;
  }

  // ---- mode 0, kernel 1 of 3: chunk totals (only launched when a line has several chunks)
  kernel_head(e, "gr_scan_sums");
  head(true);
  e.o << "  __shared__ long long gr_sm[4];\n";
  e.o << "  const long long cbeg = chunk * CH, cend = (cbeg + CH < L) ? cbeg + CH : L;\n  " << TA << " acc = " << ident << ";\n";
  e.o << "  for (long long t0 = cbeg; t0 < cend; t0 += 1024) {\n    const long long c = t0 + threadIdx.x * 4;\n";
  tile_loads("    ");
  e.o << "#pragma unroll\n    for (int j = 0; j < 4; ++j) {\n      if (c + j < cend) {\n";
  emit_scalar_program(e, g.prog, {ph.value}, tile_value, "0.0f", "t", "        ");
  e.o << "        acc = " << Em::combine(ph, "acc", "t" + std::to_string(ph.value)) << ";\n      }\n    }\n  }\n";
  e.o << "  acc = gr_lanes0(acc);\n  { " << TA << "* sm = (" << TA << "*)gr_sm;\n    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = acc;\n    __syncthreads();\n"
         "    if (threadIdx.x == 0) ws[line * NCHUNK + chunk] = gr_comb0(gr_comb0(sm[0], sm[1]), gr_comb0(sm[2], sm[3])); }\n}\n";

  offsets_kernel();

  // ---- kernel 3 of 3 (the only one for single-chunk lines): scan of a chunk with its offset
  kernel_head(e, "gr_scan");
  head(true);
  e.o << "  __shared__ long long gr_sm[2][4];\n";
  e.o << "  const long long cbeg = chunk * CH, cend = (cbeg + CH < L) ? cbeg + CH : L;\n";
  e.o << "  " << TA << " carry = NCHUNK > 1 ? ws[line * NCHUNK + chunk] : " << ident << ";\n";
  e.o << "  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;\n  int buf = 0;\n";
  e.o << "  for (long long t0 = cbeg; t0 < cend; t0 += 1024) {\n    const long long c = t0 + threadIdx.x * 4;\n    " << TA << " v[4];\n";
  tile_loads("    ");
  e.o << "#pragma unroll\n    for (int j = 0; j < 4; ++j) {\n      v[j] = " << ident << ";\n      if (c + j < cend) {\n";
  emit_scalar_program(e, g.prog, {ph.value}, tile_value, "0.0f", "t", "        ");
  e.o << "        v[j] = " << conv("t" + std::to_string(ph.value)) << ";\n      }\n    }\n";
  e.o << "    v[1] = gr_comb0(v[0], v[1]); v[2] = gr_comb0(v[1], v[2]); v[3] = gr_comb0(v[2], v[3]);\n    " << TA << " x = v[3];\n";
  for (int d = 1; d < 64; d <<= 1) e.o << "    { const " << TA << " y = gr_up(x, " << d << "); if (lane >= " << d << ") x = gr_comb0(y, x); }\n";
  e.o << "    " << TA << "* sm = (" << TA << "*)gr_sm[buf];\n    if (lane == 63) sm[wave] = x;\n    __syncthreads();\n";
  e.o << "    " << TA << " base = carry;\n    for (int q = 0; q < wave; ++q) base = gr_comb0(base, sm[q]);\n";
  e.o << "    { " << TA << " ex = gr_up(x, 1); if (lane != 0) base = gr_comb0(base, ex); }\n";
  if (ph.out_dtype == GR_I64)
    e.o << "    for (int j = 0; j < 4; ++j) if (c + j < cend) po[c + j] = gr_comb0(base, v[j]);\n";
  else {
    const char* vt = ph.out_dtype == GR_F32 ? "f4u" : "i4u";
    e.o << "    if (c + 4 <= cend) { " << vt << " ov; for (int j = 0; j < 4; ++j) ov[j] = gr_comb0(base, v[j]); "
        << ((g.nt & 8) ? "__builtin_nontemporal_store(ov, (GM " + std::string(vt) + "*)(po + c))" : "*(GM " + std::string(vt) + "*)(po + c) = ov") << "; }\n"
           "    else { for (int j = 0; j < 4; ++j) if (c + j < cend) po[c + j] = gr_comb0(base, v[j]); }\n";
  }
  e.o << "    carry = gr_comb0(carry, gr_comb0(gr_comb0(sm[0], sm[1]), gr_comb0(sm[2], sm[3])));\n    buf ^= 1;\n  }\n}\n";
}

// ---- GEMV -----------------------------------------------------------------------

// Epilogue: the pointwise consumers of the dot, evaluated at output index `idx`.
void gemv_epilogue(Em& e, const std::string& idx, const std::string& acc, const std::string& indent) {
  const GroupPlan& g = e.g;
  emit_scalar_program(e, g.prog, g.results,
                      [&](const Instr& in, int) {
                        const AccessGroup& ag = g.groups[in.group];
                        if (ag.structural_zero[0]) return e.qp + std::to_string(in.group) + "[0]";
                        return e.qp + std::to_string(in.group) + "[(" + idx + " + " + std::to_string(in.delta[0]) + ") * " + e.coef(in.group, 0) + "]";
                      },
                      acc, "t", indent);
}

void gen_gemv_rowdot(Em& e) {
  const GroupPlan& g = e.g;
  const int LPR = g.LPR, KV = g.KV, RPB = 256 / LPR;
  const AccessGroup& mg = g.groups[g.mat_group];
  const AccessGroup& vg = g.groups[g.vec_group];
  const bool mat_unit = mg.coef[1] == 1, vec_unit = vg.coef[1] == 1;
  prelude(e);
  kernel_head(e, kernel_name(g));
  e.o << "  const long long M = " << e.S(e.L.extra) << ", K = " << e.S(e.L.extra + 1) << ";\n";
  group_pointers(e, "  ");
  e.o << "  const GM float* const A = q" << g.mat_group << "; const GM float* const V = q" << g.vec_group << ";\n";
  e.o << "  const long long am = " << e.coef(g.mat_group, 0) << ", ak = " << (mat_unit ? std::string("1") : e.coef(g.mat_group, 1))
      << ", vk = " << (vec_unit ? std::string("1") : e.coef(g.vec_group, 1)) << ";\n";
  e.o << "  const int lane = threadIdx.x % " << LPR << ", rib = threadIdx.x / " << LPR << ";\n";
  e.o << "  GM float* const out = (GM float*)" << e.slot(e.L.out) << ";\n";
  const int CH = LPR * 4;  // k elements per chunk of one row
  // one pass if the whole row fits KV chunks, else loop over groups of KV chunks
  e.o << "  const bool single = K <= " << (long long)CH * KV << ";\n";
  e.o << "  float wv[" << KV << "][4];\n";
  e.o << "  if (single) {\n#pragma unroll\n    for (int q = 0; q < " << KV << "; ++q) {\n      const long long k0 = (long long)q * " << CH << " + lane * 4;\n";
  e.o << "      for (int j = 0; j < 4; ++j) wv[q][j] = (k0 + j < K) ? V[(k0 + j) * vk] : 0.0f;\n    }\n  }\n";
  e.o << "  for (long long row = (long long)blockIdx.x * " << RPB << " + rib; row < M; row += (long long)gridDim.x * " << RPB << ") {\n";
  e.o << "    const GM float* const Ar = A + row * am;\n    float acc = 0.0f;\n";
  e.o << "    if (single) {\n";
  e.o << "      float xv[" << KV << "][4];\n#pragma unroll\n      for (int q = 0; q < " << KV << "; ++q) {\n        const long long k0 = (long long)q * " << CH << " + lane * 4;\n";
  if (mat_unit)
    e.o << "        if (k0 + 4 <= K) { const f4u w = " << e.ld(g.mat_group, "f4u", "Ar + k0") << "; xv[q][0] = w[0]; xv[q][1] = w[1]; xv[q][2] = w[2]; xv[q][3] = w[3]; }\n"
           "        else { for (int j = 0; j < 4; ++j) xv[q][j] = (k0 + j < K) ? Ar[k0 + j] : 0.0f; }\n";
  else
    e.o << "        for (int j = 0; j < 4; ++j) xv[q][j] = (k0 + j < K) ? Ar[(k0 + j) * ak] : 0.0f;\n";
  e.o << "      }\n#pragma unroll\n      for (int q = 0; q < " << KV << "; ++q)\n#pragma unroll\n        for (int j = 0; j < 4; ++j) acc = __builtin_fmaf(xv[q][j], wv[q][j], acc);\n";
  e.o << "    } else {\n      long long kb = 0;\n";
  if (mat_unit && vec_unit) {
    // long rows: four chunks per step, one dwordx4 of the row and of the vector per chunk and lane
    // (the vector comes from cache), four independent partial sums
    e.o << "      float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;\n";
    e.o << "      for (; kb + " << 4 * CH << " <= K; kb += " << 4 * CH << ") {\n        const long long k0 = kb + lane * 4;\n";
    for (int q = 0; q < 4; ++q)
      e.o << "        const f4u x" << q << " = " << e.ld(g.mat_group, "f4u", "Ar + k0 + " + std::to_string(q * CH)) << "; const f4u v" << q << " = *(const GM f4u*)(V + k0 + " << q * CH << ");\n";
    for (int q = 0; q < 4; ++q)
      e.o << "        for (int j = 0; j < 4; ++j) a" << q << " = __builtin_fmaf(x" << q << "[j], v" << q << "[j], a" << q << ");\n";
    e.o << "      }\n      acc = (a0 + a1) + (a2 + a3);\n";
  }
  e.o << "      for (; kb < K; kb += " << CH << ") {\n        const long long k0 = kb + lane * 4;\n";
  e.o << "        for (int j = 0; j < 4; ++j) if (k0 + j < K) acc = __builtin_fmaf(Ar[(k0 + j) * ak], V[(k0 + j) * vk], acc);\n      }\n    }\n";
  for (int m = LPR / 2; m > 0; m >>= 1) e.o << "    acc += gr_xor(acc, " << m << ");\n";
  e.o << "    if (lane == 0) {\n";
  gemv_epilogue(e, "row", "acc", "      ");
  e.o << "      out[row] = t" << g.results[0] << ";\n    }\n  }\n}\n";
}

// Second stage of the column-accumulate contraction: combines the slab partial vectors in a
// fixed order (deterministic; the two-kernel reduction of Section 3.2) and applies the epilogue.
void emit_colacc_combine(Em& e, const std::string& kname) {
  const GroupPlan& g = e.g;
  kernel_head(e, kname);
  e.o << "  const long long M = " << e.S(e.L.extra) << ", SLABS = " << e.S(e.L.extra + 3) << ";\n";
  e.o << "  const GM float* const ws = (const GM float*)" << e.slot(e.L.extra + 2) << ";\n";
  group_pointers(e, "  ", {g.mat_group, g.vec_group});
  e.o << "  const int tx = threadIdx.x % 16, sg = threadIdx.x / 16;\n";
  e.o << "  const long long m = (long long)blockIdx.x * 16 + tx;\n";
  e.o << "  __shared__ float sm[16][17];\n  float part = 0.0f;\n";
  e.o << "  if (m < M) {\n    long long s = sg;\n"
         "    for (; s + 112 < SLABS; s += 128) {\n      float v[8];\n"
         "#pragma unroll\n      for (int u = 0; u < 8; ++u) v[u] = ws[(s + 16 * u) * M + m];\n"
         "#pragma unroll\n      for (int u = 0; u < 8; ++u) part += v[u];\n    }\n"
         "    for (; s < SLABS; s += 16) part += ws[s * M + m];\n  }\n";
  e.o << "  sm[sg][tx] = part;\n  __syncthreads();\n";
  e.o << "  if (sg == 0 && m < M) {\n    float acc = sm[0][tx];\n    for (int y = 1; y < 16; ++y) acc += sm[y][tx];\n";
  gemv_epilogue(e, "m", "acc", "    ");
  e.o << "    ((GM float*)" << e.slot(e.L.out) << ")[m] = t" << g.results[0] << ";\n  }\n}\n";
}

void gen_gemv_colacc(Em& e) {
  const GroupPlan& g = e.g;
  const int BX = g.BX, BY = g.BY, UN = g.unroll;
  const AccessGroup& vg = g.groups[g.vec_group];
  const bool vec_unit = vg.coef[1] == 1;
  prelude(e);
  // stage 1: per-slab partial vectors
  kernel_head(e, kernel_name(g));
  e.o << "  const long long M = " << e.S(e.L.extra) << ", K = " << e.S(e.L.extra + 1) << ", SLABS = " << e.S(e.L.extra + 3) << ";\n";
  e.o << "  GM float* const ws = (GM float*)" << e.slot(e.L.extra + 2) << ";\n";
  group_pointers(e, "  ");
  e.o << "  const GM float* const A = q" << g.mat_group << "; const GM float* const V = q" << g.vec_group << ";\n";
  e.o << "  const long long ak = " << e.coef(g.mat_group, 1) << ", vk = " << (vec_unit ? std::string("1") : e.coef(g.vec_group, 1)) << ";\n";
  e.o << "  const int tx = threadIdx.x % " << BX << ", ty = threadIdx.x / " << BX << ";\n";
  e.o << "  const long long ncb = (M + " << BX * 4 - 1 << ") / " << BX * 4 << ";\n";
  e.o << "  const long long cb = blockIdx.x % ncb, slab = blockIdx.x / ncb;\n";
  e.o << "  const long long m0 = cb * " << BX * 4 << " + tx * 4;\n";
  e.o << "  const long long ks = (K + SLABS - 1) / SLABS, kbeg = slab * ks, kend = (kbeg + ks < K) ? kbeg + ks : K;\n";
  e.o << "  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};\n";
  e.o << "  if (m0 + 4 <= M) {\n"
         "    long long k = kbeg + ty;\n"
         "    for (; k + " << (UN - 1) * BY << " < kend; k += " << UN * BY << ") {\n"
         "      f4u x[" << UN << "]; float s[" << UN << "];\n"
         "#pragma unroll\n      for (int u = 0; u < " << UN << "; ++u) { x[u] = " << e.ld(g.mat_group, "f4u", "A + (k + u * " + std::to_string(BY) + ") * ak + m0") << "; s[u] = V[(k + u * " << BY << ") * vk]; }\n"
         "#pragma unroll\n      for (int u = 0; u < " << UN << "; ++u) { acc[0] = __builtin_fmaf(x[u][0], s[u], acc[0]); acc[1] = __builtin_fmaf(x[u][1], s[u], acc[1]); acc[2] = __builtin_fmaf(x[u][2], s[u], acc[2]); acc[3] = __builtin_fmaf(x[u][3], s[u], acc[3]); }\n"
         "    }\n"
         "    for (; k < kend; k += " << BY << ") { const f4u x = *(const GM f4u*)(A + k * ak + m0); const float s = V[k * vk];\n"
         "      acc[0] = __builtin_fmaf(x[0], s, acc[0]); acc[1] = __builtin_fmaf(x[1], s, acc[1]); acc[2] = __builtin_fmaf(x[2], s, acc[2]); acc[3] = __builtin_fmaf(x[3], s, acc[3]); }\n"
         "  } else {\n"
         "    for (long long k = kbeg + ty; k < kend; k += " << BY << ") { const float s = V[k * vk];\n"
         "      for (int j = 0; j < 4; ++j) if (m0 + j < M) acc[j] = __builtin_fmaf(A[k * ak + m0 + j], s, acc[j]); }\n"
         "  }\n";
  e.o << "  __shared__ float sm[" << BY << "][" << BX * 4 << "];\n";
  e.o << "  for (int j = 0; j < 4; ++j) sm[ty][tx * 4 + j] = acc[j];\n  __syncthreads();\n";
  e.o << "  if (ty == 0) {\n    for (int j = 0; j < 4; ++j) {\n      float t = sm[0][tx * 4 + j];\n      for (int y = 1; y < " << BY << "; ++y) t += sm[y][tx * 4 + j];\n"
         "      if (m0 + j < M) ws[slab * M + m0 + j] = t;\n    }\n  }\n}\n";
  emit_colacc_combine(e, kernel_name(g) + "_combine");
}

// Row-dot contraction, its epilogue, and the column-accumulate contraction that consumes the
// epilogue's result, in one pass over the matrix: a row stays in registers between
// z = X[i,:].w, r_i = epilogue(z) and g += X[i,:] * r_i.
void gen_gemv_pair(Em& e, Em& e2) {
  const GroupPlan& g = e.g;
  const int LPR = g.LPR, KV = g.KV, RPB = 256 / LPR, CH = LPR * 4;
  const AccessGroup& mg = g.groups[g.mat_group];
  const AccessGroup& vg = g.groups[g.vec_group];
  (void)mg;
  const bool vec_unit = vg.coef[1] == 1;
  prelude(e);
  kernel_head(e, "gr_gemv_pair");
  e.o << "  const long long M = " << e.S(e.L.extra) << ", K = " << e.S(e.L.extra + 1) << ", SLABS = " << e.S(e.L.extra + 3) << ";\n";
  e.o << "  GM float* const ws = (GM float*)" << e.slot(e.L.extra + 2) << ";\n";
  group_pointers(e, "  ");
  e.o << "  const GM float* const A = q" << g.mat_group << "; const GM float* const V = q" << g.vec_group << ";\n";
  e.o << "  const long long am = " << e.coef(g.mat_group, 0) << ", vk = " << (vec_unit ? std::string("1") : e.coef(g.vec_group, 1)) << ";\n";
  e.o << "  const int lane = threadIdx.x % " << LPR << ", rib = threadIdx.x / " << LPR << ";\n";
  e.o << "  GM float* const out = (GM float*)" << e.slot(e.L.out) << ";\n";
  e.o << "  const long long rs = ((M + SLABS - 1) / SLABS + " << RPB - 1 << ") / " << RPB << " * " << RPB << ";\n";
  e.o << "  const long long rbeg = (long long)blockIdx.x * rs, rend = (rbeg + rs < M) ? rbeg + rs : M;\n";
  e.o << "  float wv[" << KV << "][4], acc[" << KV << "][4];\n";
  e.o << "#pragma unroll\n  for (int q = 0; q < " << KV << "; ++q) {\n    const long long k0 = (long long)q * " << CH << " + lane * 4;\n"
         "    for (int j = 0; j < 4; ++j) { wv[q][j] = (k0 + j < K) ? V[(k0 + j) * vk] : 0.0f; acc[q][j] = 0.0f; }\n  }\n";
  e.o << "  for (long long row = rbeg + rib; row < rend; row += " << RPB << ") {\n";
  e.o << "    const GM float* const Ar = A + row * am;\n    float xv[" << KV << "][4];\n";
  e.o << "#pragma unroll\n    for (int q = 0; q < " << KV << "; ++q) {\n      const long long k0 = (long long)q * " << CH << " + lane * 4;\n"
         "      if (k0 + 4 <= K) { const f4u w = " << e.ld(g.mat_group, "f4u", "Ar + k0") << "; xv[q][0] = w[0]; xv[q][1] = w[1]; xv[q][2] = w[2]; xv[q][3] = w[3]; }\n"
         "      else { for (int j = 0; j < 4; ++j) xv[q][j] = (k0 + j < K) ? Ar[k0 + j] : 0.0f; }\n    }\n";
  e.o << "    float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};\n"
         "#pragma unroll\n    for (int q = 0; q < " << KV << "; ++q)\n#pragma unroll\n      for (int j = 0; j < 4; ++j) z[j] = __builtin_fmaf(xv[q][j], wv[q][j], z[j]);\n"
         "    float zz = (z[0] + z[1]) + (z[2] + z[3]);\n";
  for (int m = LPR / 2; m > 0; m >>= 1) e.o << "    zz += gr_xor(zz, " << m << ");\n";
  gemv_epilogue(e, "row", "zz", "    ");
  e.o << "    const float rr = t" << g.results[0] << ";\n    if (lane == 0) out[row] = rr;\n";
  e.o << "#pragma unroll\n    for (int q = 0; q < " << KV << "; ++q)\n#pragma unroll\n      for (int j = 0; j < 4; ++j) acc[q][j] = __builtin_fmaf(xv[q][j], rr, acc[q][j]);\n  }\n";
  // lanes with the same position in different row groups of a wave own the same columns
  e.o << "#pragma unroll\n  for (int q = 0; q < " << KV << "; ++q)\n#pragma unroll\n    for (int j = 0; j < 4; ++j) {\n";
  for (int m = LPR; m < 64; m <<= 1) e.o << "      acc[q][j] += gr_xor(acc[q][j], " << m << ");\n";
  e.o << "    }\n";
  e.o << "  __shared__ float sm[4][" << CH * KV << "];\n";
  e.o << "  if ((threadIdx.x & 63) < " << LPR << ") {\n#pragma unroll\n    for (int q = 0; q < " << KV << "; ++q)\n      for (int j = 0; j < 4; ++j) sm[threadIdx.x >> 6][q * " << CH << " + lane * 4 + j] = acc[q][j];\n  }\n";
  e.o << "  __syncthreads();\n";
  e.o << "  for (int k = threadIdx.x; k < " << CH * KV << "; k += 256)\n    if (k < K) ws[(long long)blockIdx.x * K + k] = ((sm[0][k] + sm[1][k]) + sm[2][k]) + sm[3][k];\n}\n";
  // second stage with the second sub-graph's epilogue; its argument block follows the first one
  emit_colacc_combine(e2, "gr_gemv_pair_combine");
  e.o << e2.o.str();
}

// ---- GEMM (matrix cores) ----------------------------------------------------------

// The text fn writes to e.o, taken back out of the stream.
template <class F>
std::string captured(Em& e, F fn) {
  const std::string before = e.o.str();
  e.o.str("");
  fn();
  const std::string body = e.o.str();
  e.o.str(before);
  e.o.seekp(0, std::ios::end);
  return body;
}

// body once per combination of the loop variables, each a constant of its block.  Accumulators are register
// arrays, so every index into them has to be a constant or the array moves to scratch memory; the loops over them
// are unrolled here, in the text, because the compiler drops "#pragma unroll" once the unrolled size passes a
// threshold, which a long epilogue (tanh, erf, exp and log on 256 accumulators) does.
void emit_unrolled(std::ostream& o, const std::vector<std::pair<const char*, int>>& loops, const std::string& body, const char* ind) {
  std::vector<int> at(loops.size(), 0);
  for (;;) {
    o << ind << "{ constexpr int";
    for (size_t k = 0; k < loops.size(); ++k) o << (k ? ", " : " ") << loops[k].first << " = " << at[k];
    o << ";\n" << body << ind << "}\n";
    size_t k = loops.size();
    while (k > 0 && ++at[k - 1] == loops[k - 1].second) at[--k] = 0;
    if (k == 0) return;
  }
}

using EpiLoad = std::function<std::string(const Instr&, int)>;
void gemm_combine(Em& e, const EpiLoad& epi_load);

// Matrix product of large operands, each contiguous along one of its dimensions (K a multiple of 16; M and N need
// not be multiples of 256: edge tiles load clamped rows and store only what exists): one workgroup per 256 x 256 tile of the result and
// per compute unit, four waves with a 128 x 128 quarter each as 4 x 4 matrix-core blocks (256 accumulator
// registers per lane).
//   * Tiles of 16 values of k go from global memory straight into LDS (global_load_lds_dwordx4: lane L of a
//     wave deposits its 16 bytes at M0 + 16 L, whatever address it loaded them from), two steps ahead, into a
//     ring of three stages, so a step has one barrier, no staging registers and no LDS write instructions.
//   * Left tile: 256 rows of 16 floats; the four 16-byte chunks of row m sit at chunk position c ^ (m / 4 % 4),
//     which lets both the depositing wave (16 lanes = 4 rows x 4 chunks) and the reading one (16 lanes = 16
//     rows, one chunk) touch every bank once.  A lane reads the four k values of a chunk with one ds_read_b128
//     and feeds them to four matrix instructions: the instruction for element t of the chunks takes k = 4 h + t
//     (+ 8 in the second half of the step) in half-wave h instead of k = 2 s + h.  Both operands use the same
//     assignment, so every product is formed once; only the order of the additions differs.
//   * Right tile: 16 rows of 256 floats with a pitch of 264 (rows 4 apart lie 32 banks apart).  Block j of a
//     lane's four column blocks is column 4 r + j of the wave's 128 (r = lane % 32), so the four operands of a
//     k come with one ds_read_b128 and a lane's results are four neighbouring columns (16-byte stores).
//   * Per step and wave: 128 matrix instructions, 16 LDS reads, 8 direct loads, one barrier, each placed
//     behind a fixed matrix instruction (scheduling barriers pin the order): with one wave per SIMD every
//     instruction between two matrix instructions delays the second one, which is what bounds this kernel
//     (measured on 4096^3, one variant each: staging through registers 137 TFLOP/s, direct loads 143, the
//     same with addresses precomputed and 16-byte reads of the right operand 151; a loop of nothing but
//     matrix instructions 154).
// The direct loads are written as assembly: the compiler's own form of them makes it wait for every outstanding
// LDS read before each use (it counts them as LDS traffic that may return out of order).  Their completion is
// tracked by hand: vmcnt(8) before a step's barrier leaves only the eight loads of the newest tile in flight.
void gemm_big_body(Em& e, const EpiLoad& epi_load) {
  const GroupPlan& g = e.g;
  const int NB = g.BX / 64;          // matrix-core blocks per wave along each dimension: 4 (256 x 256 tiles) or 2 (128 x 128)
  const int T = 64 * NB, G = NB * NB, P = 2 * NB;   // tile edge, matrix instructions per group, direct loads per wave and step
  // An operand is either "k-contiguous" (kc: its tile is T rows of 16 k values, 16-byte chunks swizzled, a lane's
  // 16-byte read holds four k of one row and serves four matrix instructions) or "row-contiguous" (its tile is 16 k
  // rows of T values, a lane's read holds one k of NB neighbouring rows = its NB blocks).  Row-contiguous tiles of 256
  // values have a pitch of 264 floats (one row per load instruction); those of 128 values lie in pairs of rows (one
  // pair per load instruction) at a pitch of 272 per pair: rows four apart are 32 banks apart either way.
  struct Op { bool kc; const char* n; const char* ld; const char* org; const char* lim; int part; int size; };
  const bool akc = g.groups[g.mat_group].coef[1] == 1, bkc = g.groups[g.vec_group].coef[1] != 1;
  const int KC = T * 16, RC = NB == 4 ? 16 * 264 : 8 * 272;
  Op ops[2] = {{akc, "a", akc ? "am" : "ak", "bm0", "M", 0, akc ? KC : RC}, {bkc, "b", bkc ? "bn" : "bk", "bn0", "N", akc ? KC : RC, bkc ? KC : RC}};
  const int STAGE = ops[0].size + ops[1].size;   // floats
  auto rc_row = [&](int k) { return NB == 4 ? k * 264 : (k >> 1) * 272 + (k & 1) * 128; };   // offset of k row k of a row-contiguous tile (k without the half-wave's 4 h)
  const char* RV = NB == 4 ? "f4" : "gr_f2";      // what a lane reads of a row-contiguous tile per k
  std::ostream& o = e.o;
  const bool split = g.slabs > 1;
  o << "  __shared__ __attribute__((aligned(16))) float gr_lds[" << 3 * STAGE << "];\n"
       "  typedef __attribute__((address_space(3))) float lfloat;\n"
       "  typedef __attribute__((address_space(3))) f4 lf4;\n"
       "  typedef float gr_f2 __attribute__((ext_vector_type(2)));\n"
       "  typedef gr_f2 gr_f2u __attribute__((aligned(4)));\n"
       "  typedef __attribute__((address_space(3))) gr_f2 lgr_f2;\n"
       "  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;\n"
       "  const int wm = (wave >> 1) * " << 32 * NB << ", wn = (wave & 1) * " << 32 * NB << ";\n"
       "  const long long tiles_n = (N + " << T - 1 << ") / " << T << ";\n";
  // split K (few output tiles, a long contraction): workgroup (tile, split) accumulates the steps of k in [kbeg, KE),
  // a whole number of steps and at least two by the planner's choice, and leaves its partial tile in a workspace
  if (split) o << "  const long long tiles = tiles_n * ((M + " << T - 1 << ") / " << T << "), tile = blockIdx.x % tiles, split = blockIdx.x / tiles;\n"
                  "  const long long kbeg = split * " << e.S(e.L.ocoef + 1) << ", KE = kbeg + " << e.S(e.L.ocoef + 1) << " < K ? kbeg + " << e.S(e.L.ocoef + 1) << " : K;\n";
  else o << "  const long long tile = blockIdx.x, kbeg = 0, KE = K;\n";
  o << "  const long long bm0 = (tile / tiles_n) * " << T << ", bn0 = (tile % tiles_n) * " << T << ";\n"
       "  f16v acc[" << NB << "][" << NB << "];\n"
       "  for (int i = 0; i < " << NB << "; ++i) for (int j = 0; j < " << NB << "; ++j) for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;\n"
       "  const unsigned wv = __builtin_amdgcn_readfirstlane(wave);\n"
       "  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) void*)gr_lds;\n";
  for (const Op& x : ops) {
    const std::string n = x.n, w0 = x.n[0] == 'a' ? "wm" : "wn", X = x.n[0] == 'a' ? "A" : "B";
    // direct loads: a uniform base (advanced every step; made visibly uniform, the operands of the loads must be scalar
    // registers) plus a 32-bit byte offset per lane and piece
    o << "  unsigned " << n << "off[" << NB << "];\n#pragma unroll\n";
    if (x.kc)
      // (rows beyond the operand's edge read its last row: their results are never stored)
      o << "  for (int p = 0; p < " << NB << "; ++p) { const int m = 16 * (" << NB << " * wave + p) + lane / 4, c = (lane % 4) ^ ((m >> 2) & 3); const long long last = " << x.lim << " - 1 - " << x.org
        << "; " << n << "off[p] = 4u * (unsigned)((m < last ? m : last) * " << x.ld << " + 4 * c); }\n"
           "  const unsigned long long " << n << "64 = (unsigned long long)(" << X << " + " << x.org << " * " << x.ld << " + kbeg);\n"
           "  const unsigned long long " << n << "step = 64ull;\n";
    else {
      // (groups of four beyond the operand's edge, whose extent is a multiple of four, read its last group)
      if (NB == 4) o << "  for (int p = 0; p < 4; ++p) { const long long last = " << x.lim << " - 4 - " << x.org << "; " << n << "off[p] = 4u * (unsigned)((4 * wave + p) * " << x.ld << " + (4 * lane < last ? 4 * lane : last)); }\n";
      else o << "  for (int p = 0; p < 2; ++p) { const long long last = " << x.lim << " - 4 - " << x.org << "; " << n << "off[p] = 4u * (unsigned)((2 * (2 * wave + p) + lane / 32) * " << x.ld << " + (4 * l32 < last ? 4 * l32 : last)); }\n";
      o << "  const unsigned long long " << n << "64 = (unsigned long long)(" << X << " + " << x.org << " + kbeg * " << x.ld << ");\n"
           "  const unsigned long long " << n << "step = 64ull * (unsigned long long)__builtin_amdgcn_readfirstlane((int)" << x.ld << ");\n";
    }
    const int wave_bytes = x.kc ? 1024 * NB : (NB == 4 ? 4 * 264 * 4 : 4 * 272 * 2);
    o << "  unsigned long long " << n << "base = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(" << n << "64 >> 32)) << 32) | (unsigned)__builtin_amdgcn_readfirstlane((int)" << n << "64);\n"
         "  unsigned " << n << "lds[3];\n#pragma unroll\n  for (int st = 0; st < 3; ++st) " << n << "lds[st] = lds0 + " << 4 * STAGE << "u * st + " << 4 * x.part << "u + " << wave_bytes << "u * wv;\n";
    // LDS read bases of this lane, per stage
    if (x.kc)
      o << "  const lfloat* " << n << "p[3][2];\n#pragma unroll\n  for (int st = 0; st < 3; ++st)\n#pragma unroll\n"
           "    for (int hf = 0; hf < 2; ++hf) " << n << "p[st][hf] = (const lfloat*)gr_lds + st * " << STAGE << " + " << x.part << " + (" << w0 << " + l32) * 16 + 4 * ((2 * hf + lh) ^ ((l32 >> 2) & 3));\n"
           "  f4 " << n << "F[2][" << NB << "];\n";
    else
      o << "  const lfloat* " << n << "p[3];\n#pragma unroll\n  for (int st = 0; st < 3; ++st) " << n << "p[st] = (const lfloat*)gr_lds + st * " << STAGE << " + " << x.part << " + " << rc_row(4) << " * lh + " << w0 << " + " << NB << " * l32;\n"
           "  " << RV << " " << n << "F[2];\n";
  }
  o << "  const long long nkt = (KE - kbeg) / 16;\n";
  // piece p (0 .. NB - 1: the left tile, NB .. 2 NB - 1: the right tile) of the tile at the bases into the stage in role st
  auto piece = [&](int st, int p, const char* ind) {
    const Op& x = ops[p / NB];
    const int imm = (x.kc ? 1024 : (NB == 4 ? 4 * 264 : 4 * 272)) * (p % NB);
    // The statement must not touch the scalar condition code: the compiler splits its own 64-bit additions (s_add_u32 ..
    // s_addc_u32) around it, so M0 is set with a move of a sum the compiler formed (an s_add_i32 here once corrupted the
    // carry of a base address: a memory fault).  The wait states cover what the compiler's hazard handling does not see
    // inside an asm statement: M0 written by a scalar instruction needs one before the load, a base address that a vector
    // instruction such as v_readfirstlane wrote needs five.
    o << ind << "asm volatile(\"s_mov_b32 m0, %2\\n\\ts_nop 4\\n\\tglobal_load_lds_dwordx4 %0, %1\" : : \"v\"("
      << x.n << "off[" << p % NB << "]), \"s\"(" << x.n << "base), \"s\"(" << x.n << "lds[" << st << "] + " << imm << "u) : \"memory\", \"m0\");\n";
  };
  // (Starting every workgroup's walk along k at a different step, so that workgroups running together read
  // different columns, was measured on 2048^3, whose rows of 8 KiB cost the 128 x 128-tile kernel a tenth against rows
  // padded by 64 bytes: no change, so the walk starts at zero everywhere.)
  const char* ADV = "abase += astep; bbase += bstep;\n";
  const char* SB = "__builtin_amdgcn_sched_barrier(0);\n";
  // operand of a matrix instruction (group s of the step, block blk) and the LDS reads that provide it
  auto val = [&](const Op& x, int s, int blk) {
    std::ostringstream v;
    if (x.kc) v << x.n << "F[" << (s >> 2) << "][" << blk << "][" << (s & 3) << "]";
    else v << x.n << "F[" << (s & 1) << "][" << blk << "]";
    return v.str();
  };
  auto read_kc = [&](const Op& x, int st, int hf, int blk, const char* ind) {
    o << ind << x.n << "F[" << hf << "][" << blk << "] = *(const lf4*)(" << x.n << "p[" << st << "][" << hf << "] + " << blk * 512 << ");\n";
  };
  auto read_rc = [&](const Op& x, int st, int s, const char* ind) {
    o << ind << x.n << "F[" << (s & 1) << "] = *(const l" << RV << "*)(" << x.n << "p[" << st << "] + " << rc_row(8 * (s >> 2) + (s & 3)) << ");\n";
  };
  // One step.  Role 0 is the stage that holds the current tile; the tile two steps on goes to the stage in role 2 if more2;
  // the first operands of the next step are read (from role 1) behind the barrier if more1.  Every load and LDS read
  // sits behind a fixed matrix instruction of a fixed group.
  auto step = [&](bool more2, bool more1, const char* ind) {
    for (int s = 0; s < 8; ++s) {
      if (s == 7)
        // the next tile has landed (all but the newest P loads are complete) and this wave's reads of the current one are done
        o << ind << "__builtin_amdgcn_s_waitcnt(" << (more2 ? 0x0070 | P : 0x0070) << ");\n" << ind << "__builtin_amdgcn_s_barrier();\n";
      for (int q = 0; q < G; ++q) {
        const int i = q / NB, j = q % NB;
        o << ind << SB << ind << "acc[" << i << "][" << j << "] = __builtin_amdgcn_mfma_f32_32x32x2f32(" << val(ops[0], s, i) << ", " << val(ops[1], s, j)
          << ", acc[" << i << "][" << j << "], 0, 0, 0);\n" << ind << SB;
        if (more2 && q == 1 && s < P && s < 7) piece(2, s, ind);
        if (more2 && NB == 4 && s == 6 && q == 9) piece(2, 7, ind);
        if (more2 && s == (NB == 4 ? 6 : 3) && q == (NB == 4 ? 9 : 1)) o << ind << ADV;
        for (int k = 0; k < 2; ++k) {
          const Op& x = ops[k];
          if (x.kc) {
            // second half of the step: behind the last NB matrix instructions of group 1 (left) / 2 (right);
            // first half of the next step: behind the first 2 NB of group 7
            if (s == 1 + k && q >= G - NB) read_kc(x, 0, 1, q - (G - NB), ind);
            if (s == 7 && more1 && q >= NB * k && q < NB + NB * k) read_kc(x, 1, 0, q - NB * k, ind);
          } else {
            if (s < 7 && q == NB + k) read_rc(x, 0, s + 1, ind);
            if (s == 7 && more1 && q == NB + k) read_rc(x, 1, 0, ind);
          }
        }
      }
    }
  };
  // prologue: tiles 0 and 1 (K >= 32)
  for (int t = 0; t < 2; ++t) {
    for (int p = 0; p < P; ++p) piece(t, p, "  ");
    o << "  " << ADV;
  }
  o << "  __builtin_amdgcn_s_waitcnt(" << (0x0F70 | P) << ");\n  __builtin_amdgcn_s_barrier();\n";
  for (const Op& x : ops) {
    if (x.kc) for (int blk = 0; blk < NB; ++blk) read_kc(x, 0, 0, blk, "  ");
    else read_rc(x, 0, 0, "  ");
  }
  // the stages rotate through three roles (0: the tile of this step, 1: of the next one, 2: the target of this step's
  // loads): the addresses are exchanged after every step, a handful of register moves per step
  std::ostringstream rot;
  for (const Op& x : ops) {
    rot << "{ const unsigned t = " << x.n << "lds[0]; " << x.n << "lds[0] = " << x.n << "lds[1]; " << x.n << "lds[1] = " << x.n << "lds[2]; " << x.n << "lds[2] = t; }\n";
    if (x.kc) rot << "    { const lfloat* const t0 = " << x.n << "p[0][0]; const lfloat* const t1 = " << x.n << "p[0][1]; " << x.n << "p[0][0] = " << x.n << "p[1][0]; " << x.n << "p[0][1] = " << x.n << "p[1][1]; "
                  << x.n << "p[1][0] = " << x.n << "p[2][0]; " << x.n << "p[1][1] = " << x.n << "p[2][1]; " << x.n << "p[2][0] = t0; " << x.n << "p[2][1] = t1; }\n";
    else rot << "    { const lfloat* const t0 = " << x.n << "p[0]; " << x.n << "p[0] = " << x.n << "p[1]; " << x.n << "p[1] = " << x.n << "p[2]; " << x.n << "p[2] = t0; }\n";
    if (&x == &ops[0]) rot << "    ";
  }
  o << "  long long kt = 0;\n"
       "  for (; kt + 2 < nkt; ++kt) {\n";
  step(true, true, "    ");
  o << "    " << rot.str() << "  }\n"
       "  // the last two steps load nothing\n";
  step(false, true, "  ");
  o << "  " << rot.str();
  step(false, false, "  ");
  // epilogue on the accumulators: element q of a block is its row rr = 8 (q / 4) + 4 (lane / 32) + q % 4 and column lane % 32;
  // block i of a k-contiguous left operand holds rows wm + 32 i + rr, of a row-contiguous one rows wm + NB rr + i; block j
  // of a row-contiguous right operand holds column wn + NB (lane % 32) + j (a lane's NB results are neighbours: one
  // vector store), of a k-contiguous one column wn + 32 j + lane % 32.
  // Results beyond the edges of the matrix are computed like the others, from operands read at the clamped position,
  // and not stored (no branch around the epilogue: sixty-four guarded copies of a large one made the register
  // allocator spill).
  if (split) o << "  GM float* const out = (GM float*)" << e.slot(e.L.ocoef) << " + split * M * N;\n";   // the partial tile; gr_gemm_combine applies the epilogue
  else o << "  GM float* const out = (GM float*)" << e.slot(e.L.out) << ";\n";
  const std::string body = captured(e, [&] {
    o << "      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);\n"
         "      const long long row_at = bm0 + wm + " << (ops[0].kc ? "32 * i + rr" : std::to_string(NB) + " * rr + i") << ", row = row_at < M ? row_at : M - 1;\n"
         "      " << RV << " ov;\n"
         "#pragma unroll\n      for (int j = 0; j < " << NB << "; ++j) {\n"
         "        const long long col_at = bn0 + wn + " << (ops[1].kc ? "32 * j + l32" : std::to_string(NB) + " * l32 + j") << ", col = col_at < N ? col_at : N - 1;\n"
         "        const float cacc = acc[i][j][q];\n";
    std::string res = "cacc";
    if (!split) { emit_scalar_program(e, g.prog, g.results, epi_load, "cacc", "t", "        "); res = "t" + std::to_string(g.results[0]); }
    if (ops[1].kc) o << "        if (row_at < M && col_at < N) out[row * N + col] = " << res << ";\n      }\n      (void)ov;\n";
    else o << "        ov[j] = " << res << ";\n      }\n"
              "      if (row_at < M && bn0 + wn + " << NB << " * l32 < N) *(GM " << RV << "u*)(out + row * N + bn0 + wn + " << NB << " * l32) = ov;\n";
  });
  emit_unrolled(o, {{"i", NB}, {"q", 16}}, body, "    ");
  o << "}\n";
}


// C = A.B for f32 on MFMA (v_mfma_f32_32x32x2_f32: f32 inputs, f32 accumulation), the one place
// on this path that is a dense contraction.  A workgroup of four waves owns a 128x128 tile of
// C; each wave a 64x64 quarter as 2x2 MFMA blocks (64 accumulator VGPRs).  K advances in steps
// of 16: the next A and B tiles are fetched from global memory into registers (dwordx4 along
// whichever dimension of the operand is contiguous, so transposed views cost nothing) while the
// current tiles are consumed from LDS, k-major so that the 32 lanes of an MFMA operand read 32
// consecutive words.  The pointwise consumers of the dot run on the accumulators (epilogue).
void gen_gemm(Em& e) {
  const GroupPlan& g = e.g;
  const AccessGroup& ag = g.groups[g.mat_group];
  const AccessGroup& bg = g.groups[g.vec_group];
  const int a_mode = ag.coef[1] == 1 ? 0 : (ag.coef[0] == 1 ? 1 : 2);  // 0: k contiguous, 1: m contiguous, 2: neither
  const int b_mode = bg.coef[1] == 1 ? 0 : (bg.coef[0] == 1 ? 1 : 2);  // 0: n contiguous, 1: k contiguous, 2: neither
  // Tile of C per workgroup: 128 x 128 (four waves, each a 64 x 64 quarter as 2 x 2 matrix-core
  // blocks), or 128 x 32 for products with at most 32 columns (each wave one 32 x 32 block of its
  // own 32 rows): a 128-wide tile would spend the matrix cores on columns that do not exist.
  const int BN = g.BX == 32 ? 32 : 128;
  const int IB = BN == 128 ? 2 : 1, JB = IB;   // 32 x 32 blocks per wave along m and n
  // padded LDS rows: k-major tiles of 128 (B: BN) floats.  An operand that is contiguous along k is
  // transposed on its way into LDS by scalar writes, four k rows apart within a wave: a row pitch of
  // 130 puts those rows eight banks apart (pitch 132: only two distinct bank offsets, every write a
  // two-way conflict); an operand copied row by row with 16-byte writes needs a multiple of four.
  // K advances in steps of KS = 16 (one barrier per step), or 32 on request (option "gemm_kstep";
  // measured slower: 127 against 134 TFLOP/s on 4096^3).
  const int KS = BN == 128 && g.UC == 2 ? 32 : 16;
  const int TK = KS / 4;        // threads along k of an operand that is contiguous along k (four floats each)
  const int NI = KS / 8;        // vector loads per thread and operand tile
  const int AP = a_mode == 0 ? (KS == 32 ? 129 : 130) : 132;
  const int BP = BN == 128 && b_mode == 1 ? (KS == 32 ? 129 : 130) : BN + 4;
  prelude(e);
  e.o << "typedef float f16v __attribute__((ext_vector_type(16)));\n";
  kernel_head(e, "gr_gemm");
  e.o << "  const long long M = " << e.S(e.L.extra) << ", N = " << e.S(e.L.extra + 1) << ", K = " << e.S(e.L.extra + 2) << ";\n";
  group_pointers(e, "  ");
  e.o << "  const GM float* const A = q" << g.mat_group << "; const GM float* const B = q" << g.vec_group << ";\n";
  e.o << "  const long long am = " << e.coef(g.mat_group, 0) << ", ak = " << e.coef(g.mat_group, 1) << ", bk = " << e.coef(g.vec_group, 0)
      << ", bn = " << e.coef(g.vec_group, 1) << ";\n  (void)am; (void)ak; (void)bk; (void)bn;\n";
  const EpiLoad epi_load = [&](const Instr& in, int) {
    const AccessGroup& eg = g.groups[in.group];
    std::ostringstream s2;
    s2 << e.qp << in.group << "[0";
    if (!eg.structural_zero[0]) s2 << " + (row + " << in.delta[0] << ") * " << e.coef(in.group, 0);
    if (!eg.structural_zero[1]) s2 << " + (col + " << in.delta[1] << ") * " << e.coef(in.group, 1);
    s2 << "]";
    return s2.str();
  };
  auto emit_combine = [&]() { gemm_combine(e, epi_load); };
  if (g.VR == 2) {   // tiles loaded straight into LDS
    gemm_big_body(e, epi_load);
    emit_combine();
    return;
  }
  e.o << "  __shared__ float As[2][" << KS << "][" << AP << "];\n  __shared__ float Bs[2][" << KS << "][" << BP << "];\n";
  e.o << "  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;\n";
  if (BN == 128) e.o << "  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64, l32 = lane & 31, lh = lane >> 5;\n";
  else e.o << "  const int wm = wave * 32, wn = 0, l32 = lane & 31, lh = lane >> 5;\n";
  // split-K for products with few output tiles: workgroup (tile, split) accumulates k in
  // [kbeg, KE) and leaves its partial tile in a workspace; gr_gemm_combine adds the partial tiles
  // in a fixed order and applies the epilogue (the two-kernel reduction of Section 3.2)
  e.o << "  const long long NSPLIT = " << e.S(e.L.extra + 3) << ", KCH = " << e.S(e.L.ocoef + 1) << ";\n";
  e.o << "  const long long tiles_n = (N + " << BN - 1 << ") / " << BN << ", tiles = tiles_n * ((M + 127) / 128);\n";
  e.o << "  const long long tile = blockIdx.x % tiles, split = blockIdx.x / tiles;\n";
  e.o << "  const long long bm0 = (tile / tiles_n) * 128, bn0 = (tile % tiles_n) * " << BN << ";\n";
  e.o << "  const long long kbeg = split * KCH, KE = (kbeg + KCH < K) ? kbeg + KCH : K;\n";
  e.o << "  f16v acc[" << IB << "][" << JB << "];\n  for (int i = 0; i < " << IB << "; ++i) for (int j = 0; j < " << JB << "; ++j) for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;\n";
  e.o << "  float ra[" << 4 * NI << "], rb[" << 4 * NI << "];\n  (void)rb;\n";
  // --- global -> registers, per operand a guarded version (edge tiles, K tail) and an unguarded
  // one for tiles that lie inside the operand: straight-line loads that the compiler keeps in
  // flight under the matrix instructions of the previous step
  for (int guarded = 1; guarded >= 0; --guarded) {
    e.o << "  auto fetchA" << (guarded ? "_g" : "_u") << " = [&](long long k0) {\n";
    if (a_mode == 0) {
      e.o << "    for (int i = 0; i < " << NI << "; ++i) {\n      const long long row = bm0 + tid / " << TK << " + " << 256 / TK << " * i, kk = k0 + (tid % " << TK << ") * 4;\n";
      if (guarded) e.o << "      if (row < M && kk + 4 <= KE) { const f4u w = *(const GM f4u*)(A + row * am + kk); ra[4*i] = w[0]; ra[4*i+1] = w[1]; ra[4*i+2] = w[2]; ra[4*i+3] = w[3]; }\n"
                          "      else { for (int j = 0; j < 4; ++j) ra[4*i+j] = (row < M && kk + j < KE) ? A[row * am + kk + j] : 0.0f; }\n    }\n";
      else e.o << "      const f4u w = *(const GM f4u*)(A + row * am + kk); ra[4*i] = w[0]; ra[4*i+1] = w[1]; ra[4*i+2] = w[2]; ra[4*i+3] = w[3];\n    }\n";
    } else if (a_mode == 1) {
      e.o << "    for (int i = 0; i < " << NI << "; ++i) {\n      const long long kk = k0 + tid / 32 + 8 * i, row = bm0 + (tid % 32) * 4;\n";
      if (guarded) e.o << "      if (kk < KE && row + 4 <= M) { const f4u w = *(const GM f4u*)(A + kk * ak + row); ra[4*i] = w[0]; ra[4*i+1] = w[1]; ra[4*i+2] = w[2]; ra[4*i+3] = w[3]; }\n"
                          "      else { for (int j = 0; j < 4; ++j) ra[4*i+j] = (kk < KE && row + j < M) ? A[kk * ak + row + j] : 0.0f; }\n    }\n";
      else e.o << "      const f4u w = *(const GM f4u*)(A + kk * ak + row); ra[4*i] = w[0]; ra[4*i+1] = w[1]; ra[4*i+2] = w[2]; ra[4*i+3] = w[3];\n    }\n";
    } else {
      e.o << "    for (int i = 0; i < " << 4 * NI << "; ++i) { const int el = tid + 256 * i; const long long row = bm0 + el % 128, kk = k0 + el / 128;\n";
      if (guarded) e.o << "      ra[i] = (row < M && kk < KE) ? A[row * am + kk * ak] : 0.0f; }\n";
      else e.o << "      ra[i] = A[row * am + kk * ak]; }\n";
    }
    e.o << "  };\n";
    e.o << "  auto fetchB" << (guarded ? "_g" : "_u") << " = [&](long long k0) {\n";
    if (BN == 32) {
      // 16 x 32 tile: two elements per thread, always guarded (the operand is small)
      e.o << "    for (int i = 0; i < 2; ++i) { const int el = tid + 256 * i; const long long col = bn0 + el % 32, kk = k0 + el / 32;\n"
             "      rb[i] = (col < N && kk < KE) ? B[kk * bk + col * bn] : 0.0f; }\n";
    } else if (b_mode == 0) {
      e.o << "    for (int i = 0; i < " << NI << "; ++i) {\n      const long long kk = k0 + tid / 32 + 8 * i, col = bn0 + (tid % 32) * 4;\n";
      if (guarded) e.o << "      if (kk < KE && col + 4 <= N) { const f4u w = *(const GM f4u*)(B + kk * bk + col); rb[4*i] = w[0]; rb[4*i+1] = w[1]; rb[4*i+2] = w[2]; rb[4*i+3] = w[3]; }\n"
                          "      else { for (int j = 0; j < 4; ++j) rb[4*i+j] = (kk < KE && col + j < N) ? B[kk * bk + col + j] : 0.0f; }\n    }\n";
      else e.o << "      const f4u w = *(const GM f4u*)(B + kk * bk + col); rb[4*i] = w[0]; rb[4*i+1] = w[1]; rb[4*i+2] = w[2]; rb[4*i+3] = w[3];\n    }\n";
    } else if (b_mode == 1) {
      e.o << "    for (int i = 0; i < " << NI << "; ++i) {\n      const long long col = bn0 + tid / " << TK << " + " << 256 / TK << " * i, kk = k0 + (tid % " << TK << ") * 4;\n";
      if (guarded) e.o << "      if (col < N && kk + 4 <= KE) { const f4u w = *(const GM f4u*)(B + col * bn + kk); rb[4*i] = w[0]; rb[4*i+1] = w[1]; rb[4*i+2] = w[2]; rb[4*i+3] = w[3]; }\n"
                          "      else { for (int j = 0; j < 4; ++j) rb[4*i+j] = (col < N && kk + j < KE) ? B[col * bn + kk + j] : 0.0f; }\n    }\n";
      else e.o << "      const f4u w = *(const GM f4u*)(B + col * bn + kk); rb[4*i] = w[0]; rb[4*i+1] = w[1]; rb[4*i+2] = w[2]; rb[4*i+3] = w[3];\n    }\n";
    } else {
      e.o << "    for (int i = 0; i < " << 4 * NI << "; ++i) { const int el = tid + 256 * i; const long long col = bn0 + el % 128, kk = k0 + el / 128;\n";
      if (guarded) e.o << "      rb[i] = (col < N && kk < KE) ? B[kk * bk + col * bn] : 0.0f; }\n";
      else e.o << "      rb[i] = B[kk * bk + col * bn]; }\n";
    }
    e.o << "  };\n";
  }
  // --- registers -> LDS (k-major tiles), in pieces: a piece is what one of a thread's vector loads brought
  // (four floats of A or of B).  The main loop puts one piece behind each of the last matrix
  // instructions of a step, so that the LDS writes are issued while the matrix cores work; all of
  // them in a row after the last matrix instruction cost a tenth of the kernel's time (measured).
  std::vector<std::string> pieces;
  for (int i = 0; i < NI; ++i) {
    const std::string I = std::to_string(i);
    if (a_mode == 0) pieces.push_back("for (int j = 0; j < 4; ++j) As[buf][(tid % " + std::to_string(TK) + ") * 4 + j][tid / " + std::to_string(TK) + " + " + std::to_string(256 / TK) + " * " + I + "] = ra[4*" + I + "+j];");
    else if (a_mode == 1) pieces.push_back("for (int j = 0; j < 4; ++j) As[buf][tid / 32 + 8 * " + I + "][(tid % 32) * 4 + j] = ra[4*" + I + "+j];");
    else pieces.push_back("for (int i = " + std::to_string(4 * i) + "; i < " + std::to_string(4 * i + 4) + "; ++i) { const int el = tid + 256 * i; As[buf][el / 128][el % 128] = ra[i]; }");
  }
  if (BN == 32) pieces.push_back("for (int i = 0; i < 2; ++i) { const int el = tid + 256 * i; Bs[buf][el / 32][el % 32] = rb[i]; }");
  else for (int i = 0; i < NI; ++i) {
    const std::string I = std::to_string(i);
    if (b_mode == 0) pieces.push_back("for (int j = 0; j < 4; ++j) Bs[buf][tid / 32 + 8 * " + I + "][(tid % 32) * 4 + j] = rb[4*" + I + "+j];");
    else if (b_mode == 1) pieces.push_back("for (int j = 0; j < 4; ++j) Bs[buf][(tid % " + std::to_string(TK) + ") * 4 + j][tid / " + std::to_string(TK) + " + " + std::to_string(256 / TK) + " * " + I + "] = rb[4*" + I + "+j];");
    else pieces.push_back("for (int i = " + std::to_string(4 * i) + "; i < " + std::to_string(4 * i + 4) + "; ++i) { const int el = tid + 256 * i; Bs[buf][el / 128][el % 128] = rb[i]; }");
  }
  e.o << "  auto stash = [&](int buf) {\n";
  for (const std::string& pc : pieces) e.o << "    " << pc << "\n";
  e.o << "  };\n";
  if (BN == 128) {
    // The operands of matrix-instruction group ks + 1 are read from LDS before the four matrix
    // instructions of group ks are issued: the reads complete under 256 cycles of matrix work
    // (measured on 4096^3: 127 -> 133.7 TFLOP/s), and one piece of the next tile goes to LDS behind
    // each of the last matrix instructions of the step.  Scheduling barriers keep the order written
    // here: the compiler's scheduler would sink the reads below the matrix instructions and gather
    // the LDS writes at the end.  (A pure matrix-instruction loop reaches 155.6 TFLOP/s on this
    // device.  Measured and not adopted: steps of 32 values of k, 127 TFLOP/s; two barriers per
    // step with the LDS writes in the first half and the first operands of the next step read
    // before the second barrier, 132.6; a second or third resident workgroup per compute unit,
    // workgroups started half a step apart: no change.)
    const int G = KS / 2;                                   // groups of four matrix instructions per step
    const int first = G * 4 - 1 - (int)pieces.size();       // matrix instruction (0-based, of 4G) after which the first piece goes; none after the last
    e.o << "  auto step = [&](int cur, bool more) {\n"
           "    const int buf = cur ^ 1;\n"
           "    float a0 = As[cur][lh][wm + l32], a1 = As[cur][lh][wm + 32 + l32];\n"
           "    float b0 = Bs[cur][lh][wn + l32], b1 = Bs[cur][lh][wn + 32 + l32];\n";
    for (int ks = 0; ks < G; ++ks) {
      e.o << "    {\n      float na0 = 0.0f, na1 = 0.0f, nb0 = 0.0f, nb1 = 0.0f;\n";
      if (ks < G - 1)
        e.o << "      na0 = As[cur][" << 2 * ks + 2 << " + lh][wm + l32]; na1 = As[cur][" << 2 * ks + 2 << " + lh][wm + 32 + l32];\n"
               "      nb0 = Bs[cur][" << 2 * ks + 2 << " + lh][wn + l32]; nb1 = Bs[cur][" << 2 * ks + 2 << " + lh][wn + 32 + l32];\n";
      e.o << "      __builtin_amdgcn_sched_barrier(0);\n";
      const char* mm[4] = {"acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);", "acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);",
                           "acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);", "acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);"};
      for (int m = 0; m < 4; ++m) {
        e.o << "      " << mm[m] << "\n";
        const int pi = ks * 4 + m - first;
        if (pi >= 0 && pi < (int)pieces.size())
          e.o << "      __builtin_amdgcn_sched_barrier(0);\n      if (more) { " << pieces[pi] << " }\n      __builtin_amdgcn_sched_barrier(0);\n";
      }
      e.o << "      a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;\n    }\n";
    }
    e.o << "  };\n";
  } else
    e.o << "  auto step = [&](int cur, bool more) {\n#pragma unroll\n    for (int ks = 0; ks < 8; ++ks) {\n"
           "      const float a0 = As[cur][2 * ks + lh][wm + l32];\n"
           "      const float b0 = Bs[cur][2 * ks + lh][l32];\n"
           "      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);\n    }\n"
           "    if (more) stash(cur ^ 1);\n  };\n";
  e.o << "  const long long nkt = KE > kbeg ? (KE - kbeg + " << KS - 1 << ") / " << KS << " : 0;\n  int cur = 0;\n";
  // workgroup-uniform choice between four loops: each operand unguarded where its tile is interior
  e.o << "  const bool kfull = (KE - kbeg) % " << KS << " == 0, a_in = kfull && bm0 + 128 <= M, b_in = kfull && bn0 + " << BN << " <= N;\n";
  auto loop = [&](const char* fa, const char* fb, const char* ind) {
    e.o << ind << "if (nkt > 0) { " << fa << "(kbeg); " << fb << "(kbeg); stash(0); }\n" << ind << "__syncthreads();\n"
        << ind << "for (long long kt = 0; kt < nkt; ++kt) {\n"
        << ind << "  if (kt + 1 < nkt) { " << fa << "(kbeg + (kt + 1) * " << KS << "); " << fb << "(kbeg + (kt + 1) * " << KS << "); }\n"
        << ind << "  step(cur, kt + 1 < nkt);\n"
        << ind << "  __syncthreads();\n" << ind << "  cur ^= 1;\n" << ind << "}\n";
  };
  e.o << "  if (a_in && b_in) {\n";
  loop("fetchA_u", "fetchB_u", "    ");
  e.o << "  } else if (a_in) {\n";
  loop("fetchA_u", "fetchB_g", "    ");
  e.o << "  } else if (b_in) {\n";
  loop("fetchA_g", "fetchB_u", "    ");
  e.o << "  } else {\n";
  loop("fetchA_g", "fetchB_g", "    ");
  e.o << "  }\n";
  // --- epilogue on the accumulators: element q of a 32x32 block sits at row 8*(q/4) + 4*(lane/32) + q%4, column lane%32
  e.o << "  GM float* const out = (GM float*)" << e.slot(e.L.out) << ";\n";
  e.o << "  if (NSPLIT > 1) {\n    GM float* const ws = (GM float*)" << e.slot(e.L.ocoef) << " + split * M * N;\n"
         "#pragma unroll\n    for (int i = 0; i < " << IB << "; ++i)\n#pragma unroll\n    for (int j = 0; j < " << JB << "; ++j)\n#pragma unroll\n      for (int q = 0; q < 16; ++q) {\n"
         "        const long long row = bm0 + wm + 32 * i + 8 * (q / 4) + 4 * lh + (q % 4), col = bn0 + wn + 32 * j + l32;\n"
         "        if (row < M && col < N) ws[row * N + col] = acc[i][j][q];\n      }\n    return;\n  }\n";
  // (an index of acc that is not a constant would move the accumulators to scratch memory: the loops over blocks
  // and over groups of four elements are unrolled in the text, the four elements of a group by the compiler)
  const std::string body = captured(e, [&] {
    e.o << "#pragma unroll\n      for (int ql = 0; ql < 4; ++ql) {\n"
           "      const int q = 4 * qh + ql;\n"
           "      const long long row = bm0 + wm + 32 * i + 8 * qh + 4 * lh + ql, col = bn0 + wn + 32 * j + l32;\n"
           "      if (row < M && col < N) {\n        const float cacc = acc[i][j][q];\n";
    emit_scalar_program(e, g.prog, g.results, epi_load, "cacc", "t", "        ");
    e.o << "        out[row * N + col] = t" << g.results[0] << ";\n      }\n      }\n";
  });
  emit_unrolled(e.o, {{"i", IB}, {"j", JB}, {"qh", 4}}, body, "    ");
  e.o << "}\n";
  emit_combine();
}

// The second kernel of a matrix product whose K range is split over workgroups.
void gemm_combine(Em& e, const EpiLoad& epi_load) {
  const GroupPlan& g = e.g;
  // second stage of a split product: partial tiles added in split order, then the epilogue
  kernel_head(e, "gr_gemm_combine");
  e.o << "  const long long M = " << e.S(e.L.extra) << ", N = " << e.S(e.L.extra + 1) << ", NSPLIT = " << e.S(e.L.extra + 3) << ";\n";
  e.o << "  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;\n  if (idx >= M * N) return;\n";
  e.o << "  const long long row = idx / N, col = idx % N;\n";
  e.o << "  const GM float* const ws = (const GM float*)" << e.slot(e.L.ocoef) << ";\n";
  e.o << "  GM float* const out = (GM float*)" << e.slot(e.L.out) << ";\n";
  group_pointers(e, "  ", {g.mat_group, g.vec_group});
  e.o << "  float cacc = ws[idx];\n  long long s = 1;\n"
         "  for (; s + 4 <= NSPLIT; s += 4) {\n"
         "    const float v0 = ws[s * M * N + idx], v1 = ws[(s + 1) * M * N + idx], v2 = ws[(s + 2) * M * N + idx], v3 = ws[(s + 3) * M * N + idx];\n"
         "    cacc = (((cacc + v0) + v1) + v2) + v3;\n  }\n"
         "  for (; s < NSPLIT; ++s) cacc += ws[s * M * N + idx];\n";
  emit_scalar_program(e, g.prog, g.results, epi_load, "cacc", "t", "  ");
  e.o << "  out[idx] = t" << g.results[0] << ";\n}\n";
}

}  // namespace

std::string generate_source(const GroupPlan& g) {
  Em e(g);
  switch (g.kind) {
    case GroupKind::MAP: gen_map(e); break;
    case GroupKind::ROWRED: gen_rowred(e); break;
    case GroupKind::REDUCE: gen_reduce(e); break;
    case GroupKind::SCAN: gen_scan(e); break;
    case GroupKind::GEMM: gen_gemm(e); break;
    case GroupKind::GEMV:
      if (g.gemv_mode == 2) {
        Em e2(*g.pair);
        e2.slot_base = e.L.total;
        e.total_slots = e2.total_slots = e.L.total + e2.L.total;
        gen_gemv_pair(e, e2);
      } else if (g.gemv_mode == 1) gen_gemv_colacc(e);
      else gen_gemv_rowdot(e);
      break;
  }
  return e.o.str();
}

}  // namespace gr
