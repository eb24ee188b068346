// Plain streaming kernels: a copy and a read-only pass over a buffer, used to
// measure the HBM bandwidth a kernel on this device can actually reach, the
// context for every "fraction of peak" figure of the fused kernels.
#include <hip/hip_runtime.h>

typedef float f4 __attribute__((ext_vector_type(4)));

// Each workgroup of 256 lanes moves 4 consecutive 4 KiB segments per step, so
// every load and store instruction of a wave covers 1 KiB of contiguous memory.
__global__ __launch_bounds__(256) void gr_stream_copy_kernel(f4* __restrict__ dst, const f4* __restrict__ src, size_t n16) {
  size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  if (i + 768 < n16) {
    // non-temporal loads and stores measured fastest on MI355X
    f4 a = __builtin_nontemporal_load(&src[i]), b = __builtin_nontemporal_load(&src[i + 256]);
    f4 c = __builtin_nontemporal_load(&src[i + 512]), d = __builtin_nontemporal_load(&src[i + 768]);
    __builtin_nontemporal_store(a, &dst[i]); __builtin_nontemporal_store(b, &dst[i + 256]);
    __builtin_nontemporal_store(c, &dst[i + 512]); __builtin_nontemporal_store(d, &dst[i + 768]);
  } else {
    for (int u = 0; u < 4; ++u) if (i + 256 * u < n16) dst[i + 256 * u] = src[i + 256 * u];
  }
}

__global__ __launch_bounds__(256) void gr_stream_read_kernel(const f4* __restrict__ src, size_t n16, float* __restrict__ sink) {
  size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  f4 acc = {0.f, 0.f, 0.f, 0.f};
  if (i + 768 < n16) {
    f4 a = __builtin_nontemporal_load(&src[i]), b = __builtin_nontemporal_load(&src[i + 256]);
    f4 c = __builtin_nontemporal_load(&src[i + 512]), d = __builtin_nontemporal_load(&src[i + 768]);
    acc = (a + b) + (c + d);
  } else {
    for (int u = 0; u < 4; ++u) if (i + 256 * u < n16) acc += src[i + 256 * u];
  }
  float s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  // data-dependent store that (for finite inputs) is almost never taken keeps the loads alive
  if (s == 1.2345678e-30f) sink[blockIdx.x % 4096] = s;
}

extern "C" void gr_launch_stream_copy(void* stream, void* dst, const void* src, size_t n16) {
  unsigned grid = (unsigned)((n16 + 1023) / 1024);
  hipLaunchKernelGGL(gr_stream_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (f4*)dst, (const f4*)src, n16);
}

extern "C" void gr_launch_stream_read(void* stream, const void* src, size_t n16, void* sink) {
  unsigned grid = (unsigned)((n16 + 1023) / 1024);
  hipLaunchKernelGGL(gr_stream_read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const f4*)src, n16, (float*)sink);
}
