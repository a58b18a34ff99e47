// sfmp_unpack: packed streams -> uint8 codes, with the device unpack routines of the GEMM
// kernels; and the zero-fill kernel used to initialise workspaces.
#include "sfmp_device.h"
#include "sfmp_internal.h"

namespace sfmp {

template <int B>
__device__ __forceinline__ void unpack_tile_to_codes(const uint8_t* tile, int lane, uint8_t* dst, int64_t ld) {
  const int i = lane % 16, kb = lane / 16;
#pragma unroll
  for (int sigma = 0; sigma < 8; ++sigma) {
    uint32_t w[B];
    load_slab_words<B>(tile, sigma, lane, w);
    uint32_t op[4][4];
    unpack_slab<B>(w, op);
    uint8_t* row = dst + (int64_t)(8 * i + sigma) * ld + 8 * kb;
#pragma unroll
    for (int kappa = 0; kappa < 4; ++kappa) {
      const int p = step_pos<B>(kappa);
      uint32_t lo = 0, hi = 0;  // 8 codes of this lane and k-step as two little-endian words
#pragma unroll
      for (int reg = 0; reg < 4; ++reg) {
        const uint32_t f = op[kappa][reg];
        const uint32_t q0 = (f >> p) & ((1u << B) - 1u);
        const uint32_t q1 = (f >> (16 + p)) & ((1u << B) - 1u);
        const uint32_t two = q0 | (q1 << 8);
        if (reg < 2) lo |= two << (16 * reg); else hi |= two << (16 * (reg - 2));
      }
      uint2 v;
      v.x = lo;
      v.y = hi;
      *reinterpret_cast<uint2*>(row + 32 * kappa) = v;
    }
  }
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t* __restrict__ s2, const uint8_t* __restrict__ s3,
                                                     const uint8_t* __restrict__ s4,
                                                     const int32_t* __restrict__ tile_desc, uint8_t* __restrict__ codes,
                                                     int ntr, int ntc, int64_t K) {
  const int lane = threadIdx.x % kWave;
  const int64_t t = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave;
  if (t >= (int64_t)ntr * ntc) return;
  const int tr = (int)(t / ntc), tc = (int)(t % ntc);
  const int32_t desc = __builtin_amdgcn_readfirstlane(tile_desc[t]);
  const int b = (desc & 3) + 2;
  const int64_t slot = desc >> 2;
  uint8_t* dst = codes + (int64_t)tr * kTile * K + (int64_t)tc * kTile;
  if (b == 2) unpack_tile_to_codes<2>(s2 + slot * 4096, lane, dst, K);
  else if (b == 3) unpack_tile_to_codes<3>(s3 + slot * 6144, lane, dst, K);
  else unpack_tile_to_codes<4>(s4 + slot * 8192, lane, dst, K);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* __restrict__ p, int64_t n16) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const uint4 z = make_uint4(0, 0, 0, 0);
  for (; i < n16; i += stride) p[i] = z;
}

static int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error(what, hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return SFMP_OK;
}

int launch_unpack(const sfmp_layout_t* L, const uint8_t* s2, const uint8_t* s3, const uint8_t* s4,
                  const int32_t* index, uint8_t* codes, void* stream) {
  const int ntr = L->N / kTile, ntc = L->K / kTile;
  const int64_t nt = (int64_t)ntr * ntc;
  const unsigned grid = (unsigned)((nt + 3) / 4);
  hipLaunchKernelGGL(unpack_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, s2, s3, s4, index + 3, codes, ntr,
                     ntc, (int64_t)L->K);
  return check_launch("sfmp_unpack launch");
}

int launch_fill_zero(void* ptr, int64_t bytes, void* stream) {
  const int64_t n16 = bytes / 16;
  if (n16 == 0) return SFMP_OK;
  const unsigned grid = (unsigned)((n16 + 255) / 256 > 4096 ? 4096 : (n16 + 255) / 256);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (uint4*)ptr, n16);
  return check_launch("sfmp_workspace_init launch");
}

}  // namespace sfmp
