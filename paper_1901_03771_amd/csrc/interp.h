// Argument block of the point-program interpreter, shared by the host encoder
// and the device kernel.  A map sub-graph whose kernel is still being compiled
// runs through this one precompiled kernel instead of waiting (Section 6 of
// the paper names JIT time as the main bottleneck and overlapping compilation
// with execution as the remedy): the point function of Section 3.1 is executed
// as byte code, one iteration point per lane.
#pragma once

#define GR_INTERP_RANK 6       // iteration dimensions, right-aligned (leading ones pad)
#define GR_INTERP_GROUPS 12    // operand access patterns
#define GR_INTERP_LOADS 48
#define GR_INTERP_CONSTS 32
#define GR_INTERP_INSTR 192
#define GR_INTERP_SLOTS 40     // live 32-bit values per lane (kept in LDS, slot-major)

enum {
  GI_LOAD = 0, GI_CONST,
  GI_FNEG, GI_FABS, GI_FEXP, GI_FLOG, GI_FSQRT, GI_FSQUARE, GI_FTANH, GI_FERF,
  GI_FADD, GI_FSUB, GI_FMUL, GI_FDIV, GI_FMAX, GI_FMIN,
  GI_INEG, GI_IABS, GI_ISQUARE, GI_IADD, GI_ISUB, GI_IMUL, GI_IMAX, GI_IMIN,
  GI_RED   // row-resident reductions: the value of an earlier reduction phase of this row (a = phase)
};

struct GrInterpArgs {
  int n_instr;
  int result_slot;
  long long dims[GR_INTERP_RANK];
  unsigned long long gptr[GR_INTERP_GROUPS];               // byte address read at iteration point 0 with no shift
  long long gcoef[GR_INTERP_GROUPS][GR_INTERP_RANK];       // elements per unit step of each iteration dimension
  unsigned long long out;                                  // byte address of the output element of point 0
  long long ocoef[GR_INTERP_RANK];
  long long ldoff[GR_INTERP_LOADS];                        // element offset of each load's static shift
  unsigned consts[GR_INTERP_CONSTS];                       // bit patterns
  unsigned code[GR_INTERP_INSTR];                          // op | dst << 8 | a << 16 | b << 24
                                                           // LOAD: a = group, b = index into ldoff; CONST: a = index into consts
};

// Row-resident reductions (a softmax: row maximum, sum of exponentials, final map) through the
// interpreter: the code holds one segment per reduction phase and one for the final map; a row
// is walked once per segment by the lanes the generated kernel would give it.
#define GR_INTERP_PHASES 4

struct GrInterpRowArgs {
  GrInterpArgs m;                            // dims (last: row length), operands, constants, all segments' code; out = first output element
  int n_phase;                               // reduction phases before the final segment
  int seg_begin[GR_INTERP_PHASES + 1];       // code range and value slot of each segment (phases, then the final one)
  int seg_end[GR_INTERP_PHASES + 1];
  int seg_slot[GR_INTERP_PHASES + 1];
  int phase_op[GR_INTERP_PHASES];            // 0 sum, 1 max, 2 min
  int phase_int[GR_INTERP_PHASES];           // the phase combines i32 values (else f32)
  int per_row;                               // one output value per row (else one per element)
  int lanes;                                 // lanes per row and vec4 positions per lane: those of the generated kernel
  int positions;                             // (1, 2, 4, 8, 16, 64, 128 or 256 lanes)
};

// Sub-graphs that are cuts of their own -- a reduction over any axes, a scan, a contraction with
// its pointwise epilogue -- through the interpreter: the value program (for a contraction: the
// epilogue, which reads the accumulated sum as phase value 0) is byte code as above; the kernel
// around it is chosen by `kind`.  Plain schedules (a workgroup per output, per line or per row, a
// thread per element of a matrix product): they bridge the fraction of a second a compilation
// takes.  Integer and max/min results are exact; a float sum is associated differently from the
// generated kernel's (both are deterministic and within the same bound of the exact sum).
enum { GI_KIND_REDUCE = 0, GI_KIND_SCAN, GI_KIND_GEMV, GI_KIND_GEMM, GI_KIND_COMBINE };

struct GrInterpGenArgs {
  GrInterpArgs m;              // dims (right-aligned), operands, constants, code; out = first output element
  int kind;
  int slot;                    // LDS slot of the program's value
  int op;                      // 0 sum, 1 max, 2 min
  int is_int;                  // values are i32 (else f32)
  int out_i64;                 // the running value / result is a 64-bit integer (sums of i32)
  int first_reduced;           // reduce: dims [0, first_reduced) are kept, the rest is reduced (index into the right-aligned dims)
  long long nout, red_len;     // reduce: outputs and reduced elements per output; scan: lines and line length
  long long nsplit;            // reduce: workgroups per output (each takes a slice of the reduced range); > 1: partial results go to `partial`
  unsigned long long partial;  // and a second launch (kind GI_KIND_COMBINE) folds them in slice order
  unsigned long long mat, vec; // contractions: byte addresses of element (0, 0) of both operands
  long long am, ak, bk, bn;    // A[row * am + k * ak], B[k * bk + col * bn] (a vector operand: bn = 0)
  long long M, N, K;
};
