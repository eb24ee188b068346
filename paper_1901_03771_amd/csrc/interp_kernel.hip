// Point-program interpreter: evaluates a fused map sub-graph from byte code
// while its generated kernel is still in the run-time compiler.  Same
// arithmetic as the generated code (one IEEE operation per recorded op, no
// contraction; the same device math functions), one iteration point per lane.
//
// A workgroup covers 256 consecutive positions of the innermost iteration
// dimension at one index of the outer dimensions, so the outer index is found
// once per workgroup with 32-bit divisions.  Values live in LDS, slot-major
// (lane l of slot s at s*256+l: conflict-free, and no private-memory arrays).
#include <hip/hip_runtime.h>

#include "interp.h"

#define GM __attribute__((address_space(1)))

// gr_erff (and gr_divc, which agrees with the division below bit for bit): the text the generated kernels carry
#define GR_ANY_LANE(c) (__builtin_amdgcn_ballot_w64(c) != 0ull)
#define GR_KEEP_BRANCH __builtin_amdgcn_sched_barrier(0)
#define GR_DEVICE_MATH_SOURCE(...) __VA_ARGS__
#include "device_math.h"
#undef GR_DEVICE_MATH_SOURCE

static __device__ __forceinline__ float gi_maxf(float a, float b) { return (a >= b || a != a) ? a : b; }
static __device__ __forceinline__ float gi_minf(float a, float b) { return (a <= b || a != a) ? a : b; }

__global__ __launch_bounds__(256) void gr_interp_map_kernel(GrInterpArgs a) {
  __shared__ unsigned vals[GR_INTERP_SLOTS * 256];
  constexpr int CD = GR_INTERP_RANK - 1;
  const long long C = a.dims[CD];
  const unsigned ntc = (unsigned)((C + 255) / 256);
  const unsigned ct = blockIdx.x % ntc;
  unsigned rem = blockIdx.x / ntc;
  unsigned idx[CD];
#pragma unroll
  for (int k = CD - 1; k >= 0; --k) {
    const unsigned d = (unsigned)a.dims[k];  // the host checked that the grid, hence every outer extent, fits 31 bits
    idx[k] = rem % d;
    rem /= d;
  }
  const long long c = (long long)ct * 256 + threadIdx.x;
  if (c >= C) return;  // no barrier below: every lane touches only its own LDS column
  unsigned* const my = vals + threadIdx.x;
  const int n = a.n_instr;
  for (int pc = 0; pc < n; ++pc) {
    const unsigned w = a.code[pc];
    const unsigned op = w & 0xffu, dst = (w >> 8) & 0xffu, xa = (w >> 16) & 0xffu, xb = w >> 24;
    unsigned r;
    if (op == GI_LOAD) {
      long long off = a.ldoff[xb] + a.gcoef[xa][CD] * c;
#pragma unroll
      for (int k = 0; k < CD; ++k) off += a.gcoef[xa][k] * (long long)idx[k];
      r = *(const GM unsigned*)(a.gptr[xa] + 4ull * (unsigned long long)off);
    } else if (op == GI_CONST) {
      r = a.consts[xa];
    } else {
      const unsigned ux = my[xa * 256];
      const unsigned uy = my[xb * 256];  // unary ops encode b = a
      const float fx = __uint_as_float(ux), fy = __uint_as_float(uy);
      const int ix = (int)ux, iy = (int)uy;
      switch (op) {
        case GI_FNEG: r = __float_as_uint(-fx); break;
        case GI_FABS: r = __float_as_uint(__builtin_fabsf(fx)); break;
        case GI_FEXP: r = __float_as_uint(gr_expf(fx)); break;
        case GI_FLOG: r = __float_as_uint(gr_logf(fx)); break;
        case GI_FSQRT: r = __float_as_uint(sqrtf(fx)); break;
        case GI_FSQUARE: r = __float_as_uint(fx * fx); break;
        case GI_FTANH: r = __float_as_uint(tanhf(fx)); break;
        case GI_FERF: r = __float_as_uint(gr_erff(fx)); break;
        case GI_FADD: r = __float_as_uint(fx + fy); break;
        case GI_FSUB: r = __float_as_uint(fx - fy); break;
        case GI_FMUL: r = __float_as_uint(fx * fy); break;
        case GI_FDIV: r = __float_as_uint(fx / fy); break;
        case GI_FMAX: r = __float_as_uint(gi_maxf(fx, fy)); break;
        case GI_FMIN: r = __float_as_uint(gi_minf(fx, fy)); break;
        // i32: two's-complement wrap-around through unsigned arithmetic
        case GI_INEG: r = 0u - ux; break;
        case GI_IABS: r = ix < 0 ? 0u - ux : ux; break;
        case GI_ISQUARE: r = ux * ux; break;
        case GI_IADD: r = ux + uy; break;
        case GI_ISUB: r = ux - uy; break;
        case GI_IMUL: r = ux * uy; break;
        case GI_IMAX: r = ix >= iy ? ux : uy; break;
        case GI_IMIN: r = ix <= iy ? ux : uy; break;
        default: r = 0u; break;
      }
    }
    my[dst * 256] = r;
  }
  long long oo = a.ocoef[CD] * c;
#pragma unroll
  for (int k = 0; k < CD; ++k) oo += a.ocoef[k] * (long long)idx[k];
  *(GM unsigned*)(a.out + 4ull * (unsigned long long)oo) = my[a.result_slot * 256];
}

// One segment of byte code at element `c` of the row whose outer indices are `idx`.
static __device__ __forceinline__ void gi_run(const GrInterpArgs& a, int pc, const int end, const long long c, const unsigned* idx,
                                              unsigned* const my, const unsigned* red) {
  constexpr int CD = GR_INTERP_RANK - 1;
  for (; pc < end; ++pc) {
    const unsigned w = a.code[pc];
    const unsigned op = w & 0xffu, dst = (w >> 8) & 0xffu, xa = (w >> 16) & 0xffu, xb = w >> 24;
    unsigned r;
    if (op == GI_LOAD) {
      long long off = a.ldoff[xb] + a.gcoef[xa][CD] * c;
#pragma unroll
      for (int k = 0; k < CD; ++k) off += a.gcoef[xa][k] * (long long)idx[k];
      r = *(const GM unsigned*)(a.gptr[xa] + 4ull * (unsigned long long)off);
    } else if (op == GI_CONST) {
      r = a.consts[xa];
    } else if (op == GI_RED) {
      r = red[xa];
    } else {
      const unsigned ux = my[xa * 256];
      const unsigned uy = my[xb * 256];
      const float fx = __uint_as_float(ux), fy = __uint_as_float(uy);
      const int ix = (int)ux, iy = (int)uy;
      switch (op) {
        case GI_FNEG: r = __float_as_uint(-fx); break;
        case GI_FABS: r = __float_as_uint(__builtin_fabsf(fx)); break;
        case GI_FEXP: r = __float_as_uint(gr_expf(fx)); break;
        case GI_FLOG: r = __float_as_uint(gr_logf(fx)); break;
        case GI_FSQRT: r = __float_as_uint(sqrtf(fx)); break;
        case GI_FSQUARE: r = __float_as_uint(fx * fx); break;
        case GI_FTANH: r = __float_as_uint(tanhf(fx)); break;
        case GI_FERF: r = __float_as_uint(gr_erff(fx)); break;
        case GI_FADD: r = __float_as_uint(fx + fy); break;
        case GI_FSUB: r = __float_as_uint(fx - fy); break;
        case GI_FMUL: r = __float_as_uint(fx * fy); break;
        case GI_FDIV: r = __float_as_uint(fx / fy); break;
        case GI_FMAX: r = __float_as_uint(gi_maxf(fx, fy)); break;
        case GI_FMIN: r = __float_as_uint(gi_minf(fx, fy)); break;
        case GI_INEG: r = 0u - ux; break;
        case GI_IABS: r = ix < 0 ? 0u - ux : ux; break;
        case GI_ISQUARE: r = ux * ux; break;
        case GI_IADD: r = ux + uy; break;
        case GI_ISUB: r = ux - uy; break;
        case GI_IMUL: r = ux * uy; break;
        case GI_IMAX: r = ix >= iy ? ux : uy; break;
        case GI_IMIN: r = ix <= iy ? ux : uy; break;
        default: r = 0u; break;
      }
    }
    my[dst * 256] = r;
  }
}

static __device__ __forceinline__ unsigned gi_combine(int op, int is_int, unsigned x, unsigned y) {
  if (is_int) {
    const int ix = (int)x, iy = (int)y;
    return op == 0 ? x + y : (op == 1 ? (ix >= iy ? x : y) : (ix <= iy ? x : y));
  }
  const float fx = __uint_as_float(x), fy = __uint_as_float(y);
  return __float_as_uint(op == 0 ? fx + fy : (op == 1 ? gi_maxf(fx, fy) : gi_minf(fx, fy)));
}

// Row-resident reductions: 256 / lanes rows per workgroup; every segment walks the row once.  The
// elements of a row go to the lanes, and the partial results are combined, exactly as in the
// generated kernel of the same sub-graph (lane l takes the elements 4 * (p * lanes + l) + j for
// p = 0, 1, ... in that order; butterfly over the lanes of a wave from the widest distance down;
// then the waves of a row in pairs), so both give the same bits, sums included.  All lanes reach
// every barrier: rows past the end repeat the last row and skip the stores.
__global__ __launch_bounds__(256) void gr_interp_rowred_kernel(GrInterpRowArgs A) {
  __shared__ unsigned vals[GR_INTERP_SLOTS * 256];
  __shared__ unsigned red[256][GR_INTERP_PHASES];
  __shared__ unsigned part[4];
  constexpr int CD = GR_INTERP_RANK - 1;
  const GrInterpArgs& a = A.m;
  const int RT = A.lanes, NP = A.positions, lane = threadIdx.x % RT, rslot = threadIdx.x / RT;
  const long long C = a.dims[CD];
  unsigned long long rows = 1;
#pragma unroll
  for (int k = 0; k < CD; ++k) rows *= (unsigned long long)a.dims[k];
  const unsigned long long row_raw = (unsigned long long)blockIdx.x * (256 / RT) + rslot;
  const bool row_ok = row_raw < rows;
  const unsigned row = (unsigned)(row_ok ? row_raw : rows - 1);   // the host checked that rows fit 31 bits
  unsigned idx[CD];
  {
    unsigned rem = row;
#pragma unroll
    for (int k = CD - 1; k >= 0; --k) {
      const unsigned d = (unsigned)a.dims[k];
      idx[k] = rem % d;
      rem /= d;
    }
  }
  unsigned* const my = vals + threadIdx.x;
  for (int s = 0; s <= A.n_phase; ++s) {
    const bool final = s == A.n_phase;
    if (final) {
      if (A.per_row) {
        if (lane == 0) {
          gi_run(a, A.seg_begin[s], A.seg_end[s], 0, idx, my, red[rslot]);
          if (row_ok) *(GM unsigned*)(a.out + 4ull * (unsigned long long)row) = my[A.seg_slot[s] * 256];
        }
        break;
      }
      for (int p = 0; p < NP; ++p)
        for (int j = 0; j < 4; ++j) {
          const long long c = ((long long)p * RT + lane) * 4 + j;
          if (c >= C) continue;
          gi_run(a, A.seg_begin[s], A.seg_end[s], c, idx, my, red[rslot]);
          if (row_ok) *(GM unsigned*)(a.out + 4ull * ((unsigned long long)row * (unsigned long long)C + (unsigned long long)c)) = my[A.seg_slot[s] * 256];
        }
      break;
    }
    const int op = A.phase_op[s], is_int = A.phase_int[s];
    unsigned acc = is_int ? (op == 0 ? 0u : (op == 1 ? 0x80000000u : 0x7fffffffu))
                          : (op == 0 ? 0u : (op == 1 ? 0xff800000u : 0x7f800000u));   // 0, -inf / INT_MIN, +inf / INT_MAX
    for (int p = 0; p < NP; ++p)
      for (int j = 0; j < 4; ++j) {
        const long long c = ((long long)p * RT + lane) * 4 + j;
        if (c >= C) continue;
        gi_run(a, A.seg_begin[s], A.seg_end[s], c, idx, my, red[rslot]);
        acc = gi_combine(op, is_int, acc, my[A.seg_slot[s] * 256]);
      }
    for (int m = (RT < 64 ? RT : 64) / 2; m > 0; m >>= 1) acc = gi_combine(op, is_int, acc, (unsigned)__shfl_xor((int)acc, m, 64));
    if (RT > 64) {
      if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
      __syncthreads();
      if (RT == 256) acc = gi_combine(op, is_int, gi_combine(op, is_int, part[0], part[1]), gi_combine(op, is_int, part[2], part[3]));
      else { const int w0 = (threadIdx.x >> 7) * 2; acc = gi_combine(op, is_int, part[w0], part[w0 + 1]); }
    }
    if (lane == 0) red[rslot][s] = acc;
    __syncthreads();
  }
}

// ---- reductions over any axes, scans and contractions -------------------------------------------

static __device__ __forceinline__ unsigned long long gi_identity64(int op, int is_int, int out_i64) {
  if (out_i64) return op == 0 ? 0ull : (op == 1 ? 0x8000000000000000ull : 0x7fffffffffffffffull);
  if (is_int) return op == 0 ? 0u : (op == 1 ? 0x80000000u : 0x7fffffffu);
  return op == 0 ? 0u : (op == 1 ? 0xff800000u : 0x7f800000u);
}

// combine(x, y) on running values: 64-bit integers where the result is one (an i32 value entering
// a sum is widened before), else 32-bit values in the low word
static __device__ __forceinline__ unsigned long long gi_combine64(int op, int is_int, int out_i64, unsigned long long x, unsigned long long y) {
  if (out_i64) {
    const long long ix = (long long)x, iy = (long long)y;
    return op == 0 ? x + y : (op == 1 ? (ix >= iy ? x : y) : (ix <= iy ? x : y));
  }
  return gi_combine(op, is_int, (unsigned)x, (unsigned)y);
}

static __device__ __forceinline__ unsigned long long gi_widen(int out_i64, unsigned v) {
  return out_i64 ? (unsigned long long)(long long)(int)v : (unsigned long long)v;
}

// folds the 256 running values of a workgroup in a fixed tree; every lane returns the result
static __device__ __forceinline__ unsigned long long gi_fold256(unsigned long long* sm, int op, int is_int, int out_i64, unsigned long long v) {
  sm[threadIdx.x] = v;
  __syncthreads();
  for (int d = 128; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) sm[threadIdx.x] = gi_combine64(op, is_int, out_i64, sm[threadIdx.x], sm[threadIdx.x + d]);
    __syncthreads();
  }
  const unsigned long long r = sm[0];
  __syncthreads();
  return r;
}

// Reduction: a workgroup per output; its lanes take the reduced range 256 elements at a time.
__global__ __launch_bounds__(256) void gr_interp_reduce_kernel(GrInterpGenArgs A) {
  __shared__ unsigned vals[GR_INTERP_SLOTS * 256];
  __shared__ unsigned long long sm[256];
  constexpr int R = GR_INTERP_RANK, CD = R - 1;
  const GrInterpArgs& a = A.m;
  unsigned full[R];
  const unsigned long long o = blockIdx.x / (unsigned long long)A.nsplit, sl = blockIdx.x % (unsigned long long)A.nsplit;
  {
    unsigned long long rem = o;
    for (int k = A.first_reduced - 1; k >= 0; --k) { const unsigned long long d = (unsigned long long)a.dims[k]; full[k] = (unsigned)(rem % d); rem /= d; }
  }
  unsigned* const my = vals + threadIdx.x;
  const int op = A.op, is_int = A.is_int, w64 = A.out_i64;
  unsigned long long acc = gi_identity64(op, is_int, w64);
  const long long chunk = (A.red_len + A.nsplit - 1) / A.nsplit;
  const long long rbeg = (long long)sl * chunk, rend = rbeg + chunk < A.red_len ? rbeg + chunk : A.red_len;
  for (long long r = rbeg + threadIdx.x; r < rend; r += 256) {
    unsigned long long rem = (unsigned long long)r;
    for (int k = CD; k >= A.first_reduced; --k) { const unsigned long long d = (unsigned long long)a.dims[k]; full[k] = (unsigned)(rem % d); rem /= d; }
    gi_run(a, 0, a.n_instr, (long long)full[CD], full, my, nullptr);
    acc = gi_combine64(op, is_int, w64, acc, gi_widen(w64, my[A.slot * 256]));
  }
  acc = gi_fold256(sm, op, is_int, w64, acc);
  if (threadIdx.x == 0) {
    if (A.nsplit > 1) *(GM unsigned long long*)(A.partial + 8ull * blockIdx.x) = acc;
    else if (w64) *(GM unsigned long long*)(a.out + 8ull * o) = acc;
    else *(GM unsigned*)(a.out + 4ull * o) = (unsigned)acc;
  }
}

// Second stage of a split reduction: the slices' partial results of one output, folded in slice order.
__global__ __launch_bounds__(256) void gr_interp_combine_kernel(GrInterpGenArgs A) {
  __shared__ unsigned long long sm[256];
  const int op = A.op, is_int = A.is_int, w64 = A.out_i64;
  const unsigned long long o = blockIdx.x;
  unsigned long long acc = gi_identity64(op, is_int, w64);
  // lane l folds slices l * per .. l * per + per - 1 in order; the tree then joins neighbouring lanes
  const long long per = (A.nsplit + 255) / 256;
  for (long long q = 0; q < per; ++q) {
    const long long sl = (long long)threadIdx.x * per + q;
    if (sl < A.nsplit) acc = gi_combine64(op, is_int, w64, acc, *(const GM unsigned long long*)(A.partial + 8ull * (o * (unsigned long long)A.nsplit + (unsigned long long)sl)));
  }
  acc = gi_fold256(sm, op, is_int, w64, acc);
  if (threadIdx.x == 0) {
    if (w64) *(GM unsigned long long*)(A.m.out + 8ull * o) = acc;
    else *(GM unsigned*)(A.m.out + 4ull * o) = (unsigned)acc;
  }
}

// Inclusive scan along the last dimension: a workgroup per line, 256 elements at a time with a
// running carry (a log-step scan of the 256 values in LDS).
__global__ __launch_bounds__(256) void gr_interp_scan_kernel(GrInterpGenArgs A) {
  __shared__ unsigned vals[GR_INTERP_SLOTS * 256];
  __shared__ unsigned long long sm[2][256];
  constexpr int R = GR_INTERP_RANK, CD = R - 1;
  const GrInterpArgs& a = A.m;
  unsigned idx[R];
  {
    unsigned long long rem = blockIdx.x;
    for (int k = CD - 1; k >= 0; --k) { const unsigned long long d = (unsigned long long)a.dims[k]; idx[k] = (unsigned)(rem % d); rem /= d; }
  }
  long long obase = 0;
  for (int k = 0; k < CD; ++k) obase += a.ocoef[k] * (long long)idx[k];
  unsigned* const my = vals + threadIdx.x;
  const int op = A.op, is_int = A.is_int, w64 = A.out_i64;
  const unsigned long long idn = gi_identity64(op, is_int, w64);
  unsigned long long carry = idn;
  const long long L = A.red_len;
  for (long long t0 = 0; t0 < L; t0 += 256) {
    const long long c = t0 + threadIdx.x;
    unsigned long long v = idn;
    if (c < L) {
      gi_run(a, 0, a.n_instr, c, idx, my, nullptr);
      v = gi_widen(w64, my[A.slot * 256]);
    }
    int cur = 0;
    sm[0][threadIdx.x] = v;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {
      unsigned long long x = sm[cur][threadIdx.x];
      if ((int)threadIdx.x >= d) x = gi_combine64(op, is_int, w64, sm[cur][threadIdx.x - d], x);
      sm[cur ^ 1][threadIdx.x] = x;
      cur ^= 1;
      __syncthreads();
    }
    const unsigned long long incl = gi_combine64(op, is_int, w64, carry, sm[cur][threadIdx.x]);
    const unsigned long long total = sm[cur][255];
    if (c < L) {
      const long long oo = obase + a.ocoef[CD] * c;
      if (w64) *(GM unsigned long long*)(a.out + 8ull * (unsigned long long)oo) = incl;
      else *(GM unsigned*)(a.out + 4ull * (unsigned long long)oo) = (unsigned)incl;
    }
    carry = gi_combine64(op, is_int, w64, carry, total);
    __syncthreads();
  }
}

// Matrix-vector contraction with epilogue: a workgroup per output row.
__global__ __launch_bounds__(256) void gr_interp_gemv_kernel(GrInterpGenArgs A) {
  __shared__ unsigned vals[GR_INTERP_SLOTS * 256];
  __shared__ unsigned long long sm[256];
  constexpr int R = GR_INTERP_RANK, CD = R - 1;
  const GrInterpArgs& a = A.m;
  const long long row = blockIdx.x;
  const GM float* const Ar = (const GM float*)A.mat + row * A.am;
  const GM float* const V = (const GM float*)A.vec;
  float acc = 0.0f;
  for (long long k = threadIdx.x; k < A.K; k += 256) acc = __builtin_fmaf(Ar[k * A.ak], V[k * A.bk], acc);
  const unsigned sum = (unsigned)gi_fold256(sm, 0, 0, 0, (unsigned long long)__float_as_uint(acc));
  if (threadIdx.x == 0) {
    unsigned idx[R];
    for (int k = 0; k < R; ++k) idx[k] = 0;
    gi_run(a, 0, a.n_instr, row, idx, vals, &sum);
    *(GM unsigned*)(a.out + 4ull * (unsigned long long)row) = vals[A.slot * 256];
  }
}

// Matrix-matrix contraction with epilogue: a thread per element of the result, lanes along its rows' columns.
__global__ __launch_bounds__(256) void gr_interp_gemm_kernel(GrInterpGenArgs A) {
  __shared__ unsigned vals[GR_INTERP_SLOTS * 256];
  constexpr int R = GR_INTERP_RANK, CD = R - 1;
  const GrInterpArgs& a = A.m;
  const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
  if (o >= A.M * A.N) return;   // no barrier below
  const long long row = o / A.N, col = o % A.N;
  const GM float* const Ar = (const GM float*)A.mat + row * A.am;
  const GM float* const Bc = (const GM float*)A.vec + col * A.bn;
  float acc = 0.0f;
  for (long long k = 0; k < A.K; ++k) acc = __builtin_fmaf(Ar[k * A.ak], Bc[k * A.bk], acc);
  const unsigned sum = __float_as_uint(acc);
  unsigned idx[R];
  for (int k = 0; k < R; ++k) idx[k] = 0;
  idx[CD - 1] = (unsigned)row;
  unsigned* const my = vals + threadIdx.x;
  gi_run(a, 0, a.n_instr, col, idx, my, &sum);
  *(GM unsigned*)(a.out + 4ull * (unsigned long long)o) = my[A.slot * 256];
}

extern "C" int gr_launch_interp_gen(void* stream, const GrInterpGenArgs* args, unsigned grid) {
  switch (args->kind) {
    case GI_KIND_REDUCE: hipLaunchKernelGGL(gr_interp_reduce_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, *args); break;
    case GI_KIND_SCAN: hipLaunchKernelGGL(gr_interp_scan_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, *args); break;
    case GI_KIND_COMBINE: hipLaunchKernelGGL(gr_interp_combine_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, *args); break;
    case GI_KIND_GEMV: hipLaunchKernelGGL(gr_interp_gemv_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, *args); break;
    default: hipLaunchKernelGGL(gr_interp_gemm_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, *args); break;
  }
  return (int)hipGetLastError();
}

extern "C" int gr_launch_interp_rowred(void* stream, const GrInterpRowArgs* args, unsigned grid) {
  hipLaunchKernelGGL(gr_interp_rowred_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, *args);
  return (int)hipGetLastError();
}

extern "C" int gr_launch_interp_map(void* stream, const GrInterpArgs* args, unsigned grid) {
  hipLaunchKernelGGL(gr_interp_map_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, *args);
  return (int)hipGetLastError();
}
