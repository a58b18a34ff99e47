// Streaming-read probe of the benchmark (libsfmp_probe.so): see sfmp_probe.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sfmp_probe.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kGrid = 256;   // one workgroup of 16 wavefronts per compute unit: the launch shape of the decode kernels
constexpr int kWaves = kGrid * 16;

// Every wavefront reads whole 1 KiB pieces (16 bytes per lane), piece w, w + 4096, ... for wavefront w, four
// independent loads in flight per lane, and writes one check word: no LDS, no barrier, nothing computed.
__global__ __launch_bounds__(1024) void stream_read_kernel(const u32x4* __restrict__ src, int64_t n16, uint32_t* out) {
  const int64_t wave = (int64_t)blockIdx.x * 16 + threadIdx.x / 64;
  const int lane = threadIdx.x % 64;
  const int64_t stride = (int64_t)kWaves * 64;
  u32x4 acc0 = {0u, 0u, 0u, 0u}, acc1 = acc0, acc2 = acc0, acc3 = acc0;
  int64_t i = wave * 64 + lane;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    acc0 ^= __builtin_nontemporal_load(src + i);
    acc1 ^= __builtin_nontemporal_load(src + i + stride);
    acc2 ^= __builtin_nontemporal_load(src + i + 2 * stride);
    acc3 ^= __builtin_nontemporal_load(src + i + 3 * stride);
  }
  for (; i < n16; i += stride) acc0 ^= __builtin_nontemporal_load(src + i);
  const u32x4 x = acc0 ^ acc1 ^ acc2 ^ acc3;
  uint32_t r = x[0] ^ x[1] ^ x[2] ^ x[3];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) r ^= __shfl_xor(r, o, 64);
  if (lane == 0 && wave < 512) out[wave] = r;  // 2048 bytes of check words
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
