// Device math functions shared, as one text, by the generated kernels (the code generator pastes it
// into every kernel source) and by the precompiled byte-code interpreter (which includes it as
// code): a value never depends on which of the two produced it.
//
// The including file defines GR_DEVICE_MATH_SOURCE(...) either as its arguments (code) or as their
// stringification (text).  No preprocessor directives, comments or string literals inside the
// macro argument.
//
// gr_erff(x): error function in binary32, within 2 ulp of the exact value (1.5 ulp measured against
// a binary64 reference over four million arguments per interval, all 2^30 arguments of magnitude
// below 4 on the device by the test suite).  Two polynomial pieces, both evaluated, one selected:
//   |x| <  0.75: erf(x) = x + x * W(x^2), W of degree 5 (starts at 2/sqrt(pi) - 1)
//   |x| >= 0.75: erf(x) = sign(x) * (1 - 2^(a * Q(a))), a = min(|x|, 4), Q of degree 5 fitted to
//                log2(erfc(a)) / a; the power of two is the hardware's v_exp_f32 (its error of one
//                ulp is scaled by erfc(a) <= 0.29).  From |x| = 4 on the result is 1 exactly.
// Coefficients: weighted minimax fits (Lawson iteration) of the relative error of erf, rounded to
// binary32.  NaN compares false against the threshold and takes the first piece, which returns NaN.
// The device library's erff evaluates two longer pieces plus a full-range expf in most waves.
//
// gr_divc(x, c): x / c for a divisor that is the same in every lane (a scalar constant of the
// recorded program).  The compiler's IEEE division spends two scaling instructions, a reciprocal
// with two refinement steps and a fix-up on every quotient; with a uniform divisor the refined
// reciprocal is common to all quotients of a thread (the compiler merges the identical
// computations), and where neither scaling nor fix-up can matter -- 2^-40 <= |c| <= 2^40 and
// 2^-80 <= |x| <= 2^80 in every lane of the wave, so that quotient and residuals are normal
// numbers far from overflow -- the remaining steps are the same multiply and four fused
// multiply-adds, hence the same correctly rounded quotient.  Any other wave takes x / c.
//
// gr_expf(x), gr_logf(x): exponential and natural logarithm in binary32 on the hardware's power of
// two and binary logarithm (v_exp_f32, v_log_f32, one ulp each), within 2 ulp of the exact value.
//   exp: x log2(e) as an unevaluated sum p + e (log2(e) split into a binary32 head and tail, the
//        product's rounding error recovered with a fused multiply-add), n = round(p),
//        result = 2^((p - n) + e) scaled by 2^n (denormal results come out of the scaling);
//        0 below ln(2^-150), infinity from ln(2^128 (1 - 2^-25)) on.
//   log: log2(x) ln(2) with ln(2) as head and tail the same way; denormal arguments are scaled by
//        2^32 first (the instruction flushes them) and 32 is taken off the binary logarithm;
//        log(0) = -inf, log(x < 0) = NaN, log(inf) = inf.
// The selects that serve the rare arguments (a huge |x|, a denormal, zero, a negative number) run
// only in a wave that holds such an argument: they leave every other lane's value as it is, so a
// value never depends on its neighbours.  The device library's versions run them for every element.
// The including file defines the test and the branch: GR_ANY_LANE(c) as "c holds in some lane of
// the wave" (a ballot) and GR_KEEP_BRANCH as a scheduling barrier, which emits nothing and keeps
// the compiler from turning a short conditional block back into unconditional selects; a kernel
// that wants straight-line code (the epilogue of a matrix product over hundreds of accumulators,
// where branches cost registers; an epilogue inside a loop that the compiler should pipeline)
// defines them as true and as nothing.
GR_DEVICE_MATH_SOURCE(
static __device__ __forceinline__ float gr_erff(float x) {
  const float a = __builtin_fabsf(x);
  const float z = x * x;
  float w = -0x1.61dfd2p-11f;
  w = __builtin_fmaf(w, z, 0x1.4f2ccp-8f);
  w = __builtin_fmaf(w, z, -0x1.b7a89cp-6f);
  w = __builtin_fmaf(w, z, 0x1.ce2ac8p-4f);
  w = __builtin_fmaf(w, z, -0x1.81273ap-2f);
  w = __builtin_fmaf(w, z, 0x1.06eba8p-3f);
  const float small = __builtin_fmaf(x, w, x);
  const float ac = __builtin_fminf(a, 4.0f);
  float q = 0x1.475524p-12f;
  q = __builtin_fmaf(q, ac, -0x1.31cfcap-8f);
  q = __builtin_fmaf(q, ac, 0x1.0f413ap-5f);
  q = __builtin_fmaf(q, ac, -0x1.374a6p-3f);
  q = __builtin_fmaf(q, ac, -0x1.d58704p-1f);
  q = __builtin_fmaf(q, ac, -0x1.a0cd3cp+0f);
  const float large = __builtin_copysignf(1.0f - __builtin_amdgcn_exp2f(q * ac), x);
  return a >= 0.75f ? large : small;
}
static __device__ __forceinline__ float gr_expf(float x) {
  const float p = x * 0x1.715476p+0f;
  const float e = __builtin_fmaf(x, 0x1.4ae0cp-26f, __builtin_fmaf(x, 0x1.715476p+0f, -p));
  const float n = __builtin_rintf(p);
  float r = __builtin_ldexpf(__builtin_amdgcn_exp2f((p - n) + e), (int)n);
  if (GR_ANY_LANE(!(__builtin_fabsf(x) <= 87.0f))) {
    GR_KEEP_BRANCH;
    r = x < -0x1.9fe368p+6f ? 0.0f : r;
    r = x > 0x1.62e42ep+6f ? __builtin_inff() : r;
  }
  return r;
}
static __device__ __forceinline__ float gr_logf(float x) {
  if (!GR_ANY_LANE(!__builtin_amdgcn_classf(x, 0x100))) {
    const float y = __builtin_amdgcn_logf(x);
    const float p = y * 0x1.62e43p-1f;
    return p + __builtin_fmaf(y, -0x1.05c61p-29f, __builtin_fmaf(y, 0x1.62e43p-1f, -p));
  }
  const bool tiny = x < 0x1p-126f;
  const float y0 = __builtin_amdgcn_logf(tiny ? x * 0x1p+32f : x);
  const float y = tiny ? y0 - 32.0f : y0;
  const float p = y * 0x1.62e43p-1f;
  const float r = p + __builtin_fmaf(y, -0x1.05c61p-29f, __builtin_fmaf(y, 0x1.62e43p-1f, -p));
  return __builtin_fabsf(y0) < __builtin_inff() ? r : y0;
}
static __device__ __forceinline__ float gr_divc(float x, float c) {
  const unsigned cb = __float_as_uint(c) & 0x7fffffffu;
  const unsigned xb = __float_as_uint(x) & 0x7fffffffu;
  const bool plain = cb - 0x2b800000u <= 0x28000000u && xb - 0x17800000u <= 0x50000000u;
  if (GR_ANY_LANE(!plain)) return x / c;
  const float y0 = __builtin_amdgcn_rcpf(c);
  const float y = __builtin_fmaf(__builtin_fmaf(-c, y0, 1.0f), y0, y0);
  const float q0 = x * y;
  const float q1 = __builtin_fmaf(__builtin_fmaf(-c, q0, x), y, q0);
  return __builtin_fmaf(__builtin_fmaf(-c, q1, x), y, q1);
}
)
