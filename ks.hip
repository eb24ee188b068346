#include <hip/hip_runtime.h>
#define GM __attribute__((address_space(1)))
typedef float f4 __attribute__((ext_vector_type(4)));
typedef f4 f4u __attribute__((aligned(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef f2 f2u __attribute__((aligned(4)));
typedef int i4 __attribute__((ext_vector_type(4)));
typedef i4 i4u __attribute__((aligned(4)));
typedef int i2 __attribute__((ext_vector_type(2)));
typedef i2 i2u __attribute__((aligned(4)));
struct Args { unsigned long long s[21]; };
static __device__ __forceinline__ long long gr_peel(long long& rem, long long d) {
  if ((((unsigned long long)rem) | ((unsigned long long)d)) >> 32) { const long long i = rem % d; rem /= d; return i; }
  const unsigned r = (unsigned)rem, dd = (unsigned)d, q = r / dd;
  rem = q;
  return r - q * dd;
}
#define GR_ANY_LANE(c) true
#define GR_KEEP_BRANCH
static __device__ __forceinline__ float gr_maxf(float a, float b) { return (a >= b || a != a) ? a : b; }
static __device__ __forceinline__ float gr_minf(float a, float b) { return (a <= b || a != a) ? a : b; }
static __device__ __forceinline__ float gr_sqrtf(float x) {
  const float y = __builtin_amdgcn_rsqf(x);
  const float s = x * y, h = 0.5f * y;
  float t = __builtin_fmaf(__builtin_fmaf(-s, s, x), h, s);
  if (GR_ANY_LANE(!(x >= 0x1p-96f && x < __builtin_inff()))) {
    GR_KEEP_BRANCH;
    const bool tiny = __builtin_fabsf(x) < 0x1p-96f && x != 0.0f;
    if (GR_ANY_LANE(tiny)) return sqrtf(x);
    t = (x == 0.0f || x == __builtin_inff()) ? x : t;
  }
  return t;
}
static __device__ __forceinline__ float gr_erff(float x) { const float a = __builtin_fabsf(x); const float z = x * x; float w = -0x1.61dfd2p-11f; w = __builtin_fmaf(w, z, 0x1.4f2ccp-8f); w = __builtin_fmaf(w, z, -0x1.b7a89cp-6f); w = __builtin_fmaf(w, z, 0x1.ce2ac8p-4f); w = __builtin_fmaf(w, z, -0x1.81273ap-2f); w = __builtin_fmaf(w, z, 0x1.06eba8p-3f); const float small = __builtin_fmaf(x, w, x); const float ac = __builtin_fminf(a, 4.0f); float q = 0x1.475524p-12f; q = __builtin_fmaf(q, ac, -0x1.31cfcap-8f); q = __builtin_fmaf(q, ac, 0x1.0f413ap-5f); q = __builtin_fmaf(q, ac, -0x1.374a6p-3f); q = __builtin_fmaf(q, ac, -0x1.d58704p-1f); q = __builtin_fmaf(q, ac, -0x1.a0cd3cp+0f); const float large = __builtin_copysignf(1.0f - __builtin_amdgcn_exp2f(q * ac), x); return a >= 0.75f ? large : small; } static __device__ __forceinline__ float gr_expf(float x) { const float p = x * 0x1.715476p+0f; const float e = __builtin_fmaf(x, 0x1.4ae0cp-26f, __builtin_fmaf(x, 0x1.715476p+0f, -p)); const float n = __builtin_rintf(p); float r = __builtin_ldexpf(__builtin_amdgcn_exp2f((p - n) + e), (int)n); if (GR_ANY_LANE(!(__builtin_fabsf(x) <= 87.0f))) { GR_KEEP_BRANCH; r = x < -0x1.9fe368p+6f ? 0.0f : r; r = x > 0x1.62e42ep+6f ? __builtin_inff() : r; } return r; } static __device__ __forceinline__ float gr_logf(float x) { if (!GR_ANY_LANE(!__builtin_amdgcn_classf(x, 0x100))) { const float y = __builtin_amdgcn_logf(x); const float p = y * 0x1.62e43p-1f; return p + __builtin_fmaf(y, -0x1.05c61p-29f, __builtin_fmaf(y, 0x1.62e43p-1f, -p)); } const bool tiny = x < 0x1p-126f; const float y0 = __builtin_amdgcn_logf(tiny ? x * 0x1p+32f : x); const float y = tiny ? y0 - 32.0f : y0; const float p = y * 0x1.62e43p-1f; const float r = p + __builtin_fmaf(y, -0x1.05c61p-29f, __builtin_fmaf(y, 0x1.62e43p-1f, -p)); return __builtin_fabsf(y0) < __builtin_inff() ? r : y0; } static __device__ __forceinline__ float gr_divc(float x, float c) { const unsigned cb = __float_as_uint(c) & 0x7fffffffu; const unsigned xb = __float_as_uint(x) & 0x7fffffffu; const bool plain = cb - 0x2b800000u <= 0x28000000u && xb - 0x17800000u <= 0x50000000u; if (__builtin_amdgcn_ballot_w64(!plain) != 0ull) return x / c; const float y0 = __builtin_amdgcn_rcpf(c); const float y = __builtin_fmaf(__builtin_fmaf(-c, y0, 1.0f), y0, y0); const float q0 = x * y; const float q1 = __builtin_fmaf(__builtin_fmaf(-c, q0, x), y, q0); return __builtin_fmaf(__builtin_fmaf(-c, q1, x), y, q1); }
static __device__ __forceinline__ float gr_xor(float v, int m) { return __shfl_xor(v, m, 64); }
static __device__ __forceinline__ int gr_xor(int v, int m) { return __shfl_xor(v, m, 64); }
static __device__ __forceinline__ long long gr_xor(long long v, int m) {
  int lo = __shfl_xor((int)(v & 0xffffffffll), m, 64), hi = __shfl_xor((int)(v >> 32), m, 64);
  return ((long long)hi << 32) | (unsigned int)lo;
}
typedef float f16v __attribute__((ext_vector_type(16)));
extern "C" __global__ __launch_bounds__(256) void gr_gemm(Args a) {
  const long long M = ((long long)a.s[15]), N = ((long long)a.s[16]), K = ((long long)a.s[17]);
  const GM float* const q0 = (const GM float*)a.s[0] + ((long long)a.s[1]);
  const GM float* const q1 = (const GM float*)a.s[4] + ((long long)a.s[5]);
  const GM float* const q2 = (const GM float*)a.s[8] + ((long long)a.s[9]);
  const GM float* const A = q1; const GM float* const B = q2;
  const long long am = ((long long)a.s[6]), ak = ((long long)a.s[7]), bk = ((long long)a.s[10]), bn = ((long long)a.s[11]);
  (void)am; (void)ak; (void)bk; (void)bn;
  __shared__ __attribute__((aligned(16))) float gr_lds[12288];
  typedef __attribute__((address_space(3))) float lfloat;
  typedef __attribute__((address_space(3))) f4 lf4;
  typedef float gr_f2 __attribute__((ext_vector_type(2)));
  typedef gr_f2 gr_f2u __attribute__((aligned(4)));
  typedef __attribute__((address_space(3))) gr_f2 lgr_f2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const long long tiles_n = (N + 127) / 128;
  const long long tiles = tiles_n * ((M + 127) / 128), tile = blockIdx.x % tiles, split = blockIdx.x / tiles;
  const long long kbeg = split * ((long long)a.s[20]), KE = kbeg + ((long long)a.s[20]) < K ? kbeg + ((long long)a.s[20]) : K;
  const long long bm0 = (tile / tiles_n) * 128, bn0 = (tile % tiles_n) * 128;
  f16v acc[2][2];
  for (int i = 0; i < 2; ++i) for (int j = 0; j < 2; ++j) for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;
  const unsigned wv = __builtin_amdgcn_readfirstlane(wave);
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) void*)gr_lds;
  unsigned aoff[2];
#pragma unroll
  for (int p = 0; p < 2; ++p) { const int m = 16 * (2 * wave + p) + lane / 4, c = (lane % 4) ^ ((m >> 2) & 3); const long long last = M - 1 - bm0; aoff[p] = 4u * (unsigned)((m < last ? m : last) * am + 4 * c); }
  const unsigned long long a64 = (unsigned long long)(A + bm0 * am + kbeg);
  const unsigned long long astep = 64ull;
  unsigned long long abase = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(a64 >> 32)) << 32) | (unsigned)__builtin_amdgcn_readfirstlane((int)a64);
  unsigned alds[3];
#pragma unroll
  for (int st = 0; st < 3; ++st) alds[st] = lds0 + 16384u * st + 0u + 2048u * wv;
  const lfloat* ap[3][2];
#pragma unroll
  for (int st = 0; st < 3; ++st)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) ap[st][hf] = (const lfloat*)gr_lds + st * 4096 + 0 + (wm + l32) * 16 + 4 * ((2 * hf + lh) ^ ((l32 >> 2) & 3));
  f4 aF[2][2];
  unsigned boff[2];
#pragma unroll
  for (int p = 0; p < 2; ++p) { const int m = 16 * (2 * wave + p) + lane / 4, c = (lane % 4) ^ ((m >> 2) & 3); const long long last = N - 1 - bn0; boff[p] = 4u * (unsigned)((m < last ? m : last) * bn + 4 * c); }
  const unsigned long long b64 = (unsigned long long)(B + bn0 * bn + kbeg);
  const unsigned long long bstep = 64ull;
  unsigned long long bbase = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(b64 >> 32)) << 32) | (unsigned)__builtin_amdgcn_readfirstlane((int)b64);
  unsigned blds[3];
#pragma unroll
  for (int st = 0; st < 3; ++st) blds[st] = lds0 + 16384u * st + 8192u + 2048u * wv;
  const lfloat* bp[3][2];
#pragma unroll
  for (int st = 0; st < 3; ++st)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) bp[st][hf] = (const lfloat*)gr_lds + st * 4096 + 2048 + (wn + l32) * 16 + 4 * ((2 * hf + lh) ^ ((l32 >> 2) & 3));
  f4 bF[2][2];
  const long long nkt = (KE - kbeg) / 16;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(aoff[0]), "s"(abase), "s"(alds[0] + 0u) : "memory", "m0");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(aoff[1]), "s"(abase), "s"(alds[0] + 1024u) : "memory", "m0");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(boff[0]), "s"(bbase), "s"(blds[0] + 0u) : "memory", "m0");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(boff[1]), "s"(bbase), "s"(blds[0] + 1024u) : "memory", "m0");
  abase += astep; bbase += bstep;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(aoff[0]), "s"(abase), "s"(alds[1] + 0u) : "memory", "m0");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(aoff[1]), "s"(abase), "s"(alds[1] + 1024u) : "memory", "m0");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(boff[0]), "s"(bbase), "s"(blds[1] + 0u) : "memory", "m0");
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(boff[1]), "s"(bbase), "s"(blds[1] + 1024u) : "memory", "m0");
  abase += astep; bbase += bstep;
  __builtin_amdgcn_s_waitcnt(3956);
  __builtin_amdgcn_s_barrier();
  aF[0][0] = *(const lf4*)(ap[0][0] + 0);
  aF[0][1] = *(const lf4*)(ap[0][0] + 512);
  bF[0][0] = *(const lf4*)(bp[0][0] + 0);
  bF[0][1] = *(const lf4*)(bp[0][0] + 512);
  long long kt = 0;
  for (; kt + 2 < nkt; ++kt) {
    __builtin_amdgcn_sched_barrier(0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][0], bF[0][0][0], acc[0][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][0], bF[0][1][0], acc[0][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(aoff[0]), "s"(abase), "s"(alds[2] + 0u) : "memory", "m0");
    __builtin_amdgcn_sched_barrier(0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][0], bF[0][0][0], acc[1][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][0], bF[0][1][0], acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][1], bF[0][0][1], acc[0][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][1], bF[0][1][1], acc[0][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(aoff[1]), "s"(abase), "s"(alds[2] + 1024u) : "memory", "m0");
    __builtin_amdgcn_sched_barrier(0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][1], bF[0][0][1], acc[1][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    aF[1][0] = *(const lf4*)(ap[0][1] + 0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][1], bF[0][1][1], acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    aF[1][1] = *(const lf4*)(ap[0][1] + 512);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][2], bF[0][0][2], acc[0][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][2], bF[0][1][2], acc[0][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(boff[0]), "s"(bbase), "s"(blds[2] + 0u) : "memory", "m0");
    __builtin_amdgcn_sched_barrier(0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][2], bF[0][0][2], acc[1][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    bF[1][0] = *(const lf4*)(bp[0][1] + 0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][2], bF[0][1][2], acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    bF[1][1] = *(const lf4*)(bp[0][1] + 512);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][3], bF[0][0][3], acc[0][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][3], bF[0][1][3], acc[0][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(boff[1]), "s"(bbase), "s"(blds[2] + 1024u) : "memory", "m0");
    abase += astep; bbase += bstep;
    __builtin_amdgcn_sched_barrier(0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][3], bF[0][0][3], acc[1][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][3], bF[0][1][3], acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][0], bF[1][0][0], acc[0][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][0], bF[1][1][0], acc[0][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][0], bF[1][0][0], acc[1][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][0], bF[1][1][0], acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][1], bF[1][0][1], acc[0][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][1], bF[1][1][1], acc[0][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][1], bF[1][0][1], acc[1][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][1], bF[1][1][1], acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][2], bF[1][0][2], acc[0][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][2], bF[1][1][2], acc[0][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][2], bF[1][0][2], acc[1][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][2], bF[1][1][2], acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(116);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][3], bF[1][0][3], acc[0][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    aF[0][0] = *(const lf4*)(ap[1][0] + 0);
    __builtin_amdgcn_sched_barrier(0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][3], bF[1][1][3], acc[0][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    aF[0][1] = *(const lf4*)(ap[1][0] + 512);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][3], bF[1][0][3], acc[1][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    bF[0][0] = *(const lf4*)(bp[1][0] + 0);
    __builtin_amdgcn_sched_barrier(0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][3], bF[1][1][3], acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    bF[0][1] = *(const lf4*)(bp[1][0] + 512);
    { const unsigned t = alds[0]; alds[0] = alds[1]; alds[1] = alds[2]; alds[2] = t; }
    { const lfloat* const t0 = ap[0][0]; const lfloat* const t1 = ap[0][1]; ap[0][0] = ap[1][0]; ap[0][1] = ap[1][1]; ap[1][0] = ap[2][0]; ap[1][1] = ap[2][1]; ap[2][0] = t0; ap[2][1] = t1; }
    { const unsigned t = blds[0]; blds[0] = blds[1]; blds[1] = blds[2]; blds[2] = t; }
    { const lfloat* const t0 = bp[0][0]; const lfloat* const t1 = bp[0][1]; bp[0][0] = bp[1][0]; bp[0][1] = bp[1][1]; bp[1][0] = bp[2][0]; bp[1][1] = bp[2][1]; bp[2][0] = t0; bp[2][1] = t1; }
  }
  // the last two steps load nothing
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][0], bF[0][0][0], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][0], bF[0][1][0], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][0], bF[0][0][0], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][0], bF[0][1][0], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][1], bF[0][0][1], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][1], bF[0][1][1], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][1], bF[0][0][1], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  aF[1][0] = *(const lf4*)(ap[0][1] + 0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][1], bF[0][1][1], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  aF[1][1] = *(const lf4*)(ap[0][1] + 512);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][2], bF[0][0][2], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][2], bF[0][1][2], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][2], bF[0][0][2], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  bF[1][0] = *(const lf4*)(bp[0][1] + 0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][2], bF[0][1][2], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  bF[1][1] = *(const lf4*)(bp[0][1] + 512);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][3], bF[0][0][3], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][3], bF[0][1][3], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][3], bF[0][0][3], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][3], bF[0][1][3], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][0], bF[1][0][0], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][0], bF[1][1][0], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][0], bF[1][0][0], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][0], bF[1][1][0], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][1], bF[1][0][1], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][1], bF[1][1][1], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][1], bF[1][0][1], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][1], bF[1][1][1], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][2], bF[1][0][2], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][2], bF[1][1][2], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][2], bF[1][0][2], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][2], bF[1][1][2], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(112);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][3], bF[1][0][3], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  aF[0][0] = *(const lf4*)(ap[1][0] + 0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][3], bF[1][1][3], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  aF[0][1] = *(const lf4*)(ap[1][0] + 512);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][3], bF[1][0][3], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  bF[0][0] = *(const lf4*)(bp[1][0] + 0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][3], bF[1][1][3], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  bF[0][1] = *(const lf4*)(bp[1][0] + 512);
  { const unsigned t = alds[0]; alds[0] = alds[1]; alds[1] = alds[2]; alds[2] = t; }
    { const lfloat* const t0 = ap[0][0]; const lfloat* const t1 = ap[0][1]; ap[0][0] = ap[1][0]; ap[0][1] = ap[1][1]; ap[1][0] = ap[2][0]; ap[1][1] = ap[2][1]; ap[2][0] = t0; ap[2][1] = t1; }
    { const unsigned t = blds[0]; blds[0] = blds[1]; blds[1] = blds[2]; blds[2] = t; }
    { const lfloat* const t0 = bp[0][0]; const lfloat* const t1 = bp[0][1]; bp[0][0] = bp[1][0]; bp[0][1] = bp[1][1]; bp[1][0] = bp[2][0]; bp[1][1] = bp[2][1]; bp[2][0] = t0; bp[2][1] = t1; }
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][0], bF[0][0][0], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][0], bF[0][1][0], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][0], bF[0][0][0], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][0], bF[0][1][0], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][1], bF[0][0][1], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][1], bF[0][1][1], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][1], bF[0][0][1], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  aF[1][0] = *(const lf4*)(ap[0][1] + 0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][1], bF[0][1][1], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  aF[1][1] = *(const lf4*)(ap[0][1] + 512);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][2], bF[0][0][2], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][2], bF[0][1][2], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][2], bF[0][0][2], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  bF[1][0] = *(const lf4*)(bp[0][1] + 0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][2], bF[0][1][2], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  bF[1][1] = *(const lf4*)(bp[0][1] + 512);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][3], bF[0][0][3], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][0][3], bF[0][1][3], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][3], bF[0][0][3], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[0][1][3], bF[0][1][3], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][0], bF[1][0][0], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][0], bF[1][1][0], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][0], bF[1][0][0], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][0], bF[1][1][0], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][1], bF[1][0][1], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][1], bF[1][1][1], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][1], bF[1][0][1], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][1], bF[1][1][1], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][2], bF[1][0][2], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][2], bF[1][1][2], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][2], bF[1][0][2], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][2], bF[1][1][2], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(112);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][3], bF[1][0][3], acc[0][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][0][3], bF[1][1][3], acc[0][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][3], bF[1][0][3], acc[1][0], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_sched_barrier(0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(aF[1][1][3], bF[1][1][3], acc[1][1], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
  GM float* const out = (GM float*)a.s[19] + split * M * N;
    { constexpr int i = 0, q = 0;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 1;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 2;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 3;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 4;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 5;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 6;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 7;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 8;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 9;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 10;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 11;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 12;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 13;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 14;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 0, q = 15;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 0;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 1;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 2;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 3;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 4;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 5;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 6;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 7;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 8;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 9;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 10;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 11;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 12;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 13;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 14;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
    { constexpr int i = 1, q = 15;
      const int rr = 8 * (q / 4) + 4 * lh + (q % 4);
      const long long row_at = bm0 + wm + 32 * i + rr, row = row_at < M ? row_at : M - 1;
      gr_f2 ov;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const long long col_at = bn0 + wn + 32 * j + l32, col = col_at < N ? col_at : N - 1;
        const float cacc = acc[i][j][q];
        if (row_at < M && col_at < N) out[row * N + col] = cacc;
      }
      (void)ov;
    }
}
extern "C" __global__ __launch_bounds__(256) void gr_gemm_combine(Args a) {
  const long long M = ((long long)a.s[15]), N = ((long long)a.s[16]), NSPLIT = ((long long)a.s[18]);
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= M * N) return;
  const long long row = idx / N, col = idx % N;
  const GM float* const ws = (const GM float*)a.s[19];
  GM float* const out = (GM float*)a.s[12];
  const GM float* const q0 = (const GM float*)a.s[0] + ((long long)a.s[1]);
  float cacc = ws[idx];
  long long s = 1;
  for (; s + 4 <= NSPLIT; s += 4) {
    const float v0 = ws[s * M * N + idx], v1 = ws[(s + 1) * M * N + idx], v2 = ws[(s + 2) * M * N + idx], v3 = ws[(s + 3) * M * N + idx];
    cacc = (((cacc + v0) + v1) + v2) + v3;
  }
  for (; s < NSPLIT; ++s) cacc += ws[s * M * N + idx];
  const float t0 = cacc;
  const float t1 = q0[0 + (col + 0) * ((long long)a.s[3])];
  const float t2 = (t0 + t1);
  const float t3 = tanhf(t2);
  out[idx] = t3;
}
