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

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
// One v_mfma_f32_16x16x32_f16 per workgroup (one wavefront): A row 0 = a[32], B column 0 = b[32], everything else
// zero, C = 0; the result element (0, 0).  Lane kb * 16 holds the products k = 8 kb .. 8 kb + 7.
__global__ __launch_bounds__(64) void mfma_dot_kernel(const _Float16* __restrict__ a, const _Float16* __restrict__ b,
                                                      float* __restrict__ out) {
  const int t = blockIdx.x, lane = threadIdx.x, i16 = lane % 16, kb = lane / 16;
  half8 av, bv;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    av[j] = i16 == 0 ? a[(size_t)t * 32 + 8 * kb + j] : (_Float16)0;
    bv[j] = i16 == 0 ? b[(size_t)t * 32 + 8 * kb + j] : (_Float16)0;
  }
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
  acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc, 0, 0, 0);
  if (lane == 0) out[t] = acc[0];
}

}  // namespace

extern "C" int sfmp_probe_mfma_dot(const void* a_dev, const void* b_dev, int32_t count, void* out_dev, void* hip_stream) {
  if (!a_dev || !b_dev || !out_dev) return -1;
  if (count < 1 || (reinterpret_cast<uintptr_t>(a_dev) % 2) != 0 || (reinterpret_cast<uintptr_t>(b_dev) % 2) != 0 ||
      (reinterpret_cast<uintptr_t>(out_dev) % 4) != 0)
    return -2;
  hipLaunchKernelGGL(mfma_dot_kernel, dim3((unsigned)count), dim3(64), 0, (hipStream_t)hip_stream, (const _Float16*)a_dev,
                     (const _Float16*)b_dev, (float*)out_dev);
  return hipGetLastError() == hipSuccess ? 0 : -6;
}

extern "C" int sfmp_probe_stream_read(const void* src_dev, int64_t bytes, void* out_dev, void* hip_stream) {
  if (!src_dev || !out_dev) return -1;
  if (bytes < 16 || (bytes % 16) != 0 || (reinterpret_cast<uintptr_t>(src_dev) % 16) != 0 ||
      (reinterpret_cast<uintptr_t>(out_dev) % 4) != 0)
    return -2;
  hipLaunchKernelGGL(stream_read_kernel, dim3(kGrid), dim3(1024), 0, (hipStream_t)hip_stream, (const u32x4*)src_dev,
                     bytes / 16, (uint32_t*)out_dev);
  return hipGetLastError() == hipSuccess ? 0 : -6;
}
