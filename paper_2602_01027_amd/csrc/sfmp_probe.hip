// Streaming-read probe of the benchmark (libsfmp_probe.so): see sfmp_probe.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sfmp_probe.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kGrid = 512;  // workgroups = check words written

__global__ __launch_bounds__(1024) void stream_read_kernel(const u32x4* __restrict__ src, int64_t n16, uint32_t* out) {
  const int64_t stride = (int64_t)gridDim.x * 1024;
  uint32_t acc = 0;
  int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride),
                c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
    const u32x4 x = a ^ b ^ c ^ d;
    acc ^= x[0] ^ x[1] ^ x[2] ^ x[3];
  }
  for (; i < n16; i += stride) {
    const u32x4 a = __builtin_nontemporal_load(src + i);
    acc ^= a[0] ^ a[1] ^ a[2] ^ a[3];
  }
  __shared__ uint32_t red[1024];
  red[threadIdx.x] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t r = 0;
    for (int t = 0; t < 1024; ++t) r ^= red[t];
    out[blockIdx.x] = r;
  }
}

}  // namespace

extern "C" int sfmp_probe_stream_read(const void* src_dev, int64_t bytes, void* out_dev, void* hip_stream) {
  if (!src_dev || !out_dev) return -1;
  if (bytes < 16 || (bytes % 16) != 0 || (reinterpret_cast<uintptr_t>(src_dev) % 16) != 0 ||
      (reinterpret_cast<uintptr_t>(out_dev) % 4) != 0)
    return -2;
  hipLaunchKernelGGL(stream_read_kernel, dim3(kGrid), dim3(1024), 0, (hipStream_t)hip_stream, (const u32x4*)src_dev,
                     bytes / 16, (uint32_t*)out_dev);
  return hipGetLastError() == hipSuccess ? 0 : -6;
}
