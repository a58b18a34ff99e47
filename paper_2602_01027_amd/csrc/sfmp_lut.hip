// One-bit lookup-table GEMV (M = 1) on the bit-plane format: the paper's own kernel scheme (Appendix B, Eq. 10-13;
// Appendix F) carried to gfx950, as a measured alternative to the MFMA path of sfmp_gemm.
//
// The weights are b one-bit matrices per 128 x 128 tile (b = the tile's width), in the +-1 form of Appendix B:
//   w = sum_i 2^i s^ W^_i + z^,   s^ = s/2,  W^_i = 2 W_i - 1,  z^ = z + (2^b - 1) s / 2.
// A workgroup of 256 threads owns 256 output features (two tile rows) and a range of tile columns.  Per tile column
// it builds, in LDS, the 16 tables of the column's 16 groups of 8 activations: 128 entries each (fp32, or fp16 as
// in Appendix F: 2 bytes per entry, the fp32 sum rounded once), entry p =
// sum_t (+-) x_t with the sign of x_t given by bit t of p and x_7 always negative; an index with its top bit set is
// served by the complemented index with the sign flipped (mirror storage: half the table).  Each thread then walks
// its feature's 16 bytes per bit plane, one lookup per byte, adds the looked-up values over the groups, weights the
// planes by 2^i, applies s^ and adds z^ times the sum of the column's activations.  The partial sums of the K
// ranges (fp32 [ksplit, N]) are added in a fixed order by a second small kernel, which also undoes the row
// permutation, so results repeat bit for bit.
#include <type_traits>

#include "sfmp_device.h"
#include "sfmp_internal.h"

namespace sfmp {

constexpr int kLutThreads = 256;      // = output features per workgroup
constexpr int kLutPlaneBytes = 2048;  // one bit plane of a 128 x 128 tile
// workgroups aimed at: K is cut into ranges until there are about this many (512, 1024 and 2048 were measured)
constexpr int kLutTargetGroups = 2048;

struct LutParams {
  const _Float16* X;
  const int32_t* col_perm;
  const uint8_t* planes;
  const uint32_t* tile_off;
  const _Float16* scales;
  const _Float16* zeros;
  float* partial;  // [ksplit, N]
  int32_t N, K, ntc, ksplit;
};

// H16: table entries stored as fp16 (the accumulation stays in fp32)
template <bool H16>
__global__ __launch_bounds__(kLutThreads) void lut_gemv_kernel(const LutParams p) {
  typedef typename std::conditional<H16, _Float16, float>::type entry_t;
  __shared__ __align__(16) entry_t lut[2][16][128];  // double-buffered over tile columns
  const int tid = threadIdx.x;
  const int rb = (int)blockIdx.x / p.ksplit, ks = (int)blockIdx.x % p.ksplit;
  const int n = rb * kLutThreads + tid;                                   // output feature (reordered coordinates)
  const bool active = n < p.N;                                            // uniform per wavefront: N is a multiple of 128
  const int tr = __builtin_amdgcn_readfirstlane(min(n, p.N - 1) / kTile);  // tile row of this wavefront
  const int r = n % kTile;
  const int tc_begin = (int)((int64_t)ks * p.ntc / p.ksplit), tc_end = (int)((int64_t)(ks + 1) * p.ntc / p.ksplit);

  // Everything a tile column needs from memory is requested one column ahead (this thread's 16 bytes of each bit
  // plane, its scale and zero, and the 8 activations of the table entries it builds), so that the lookups of a
  // column run while the next column's data is on its way.
  struct Column {
    u32x4 w[4];
    float s, z, x[8];
    int b;
  };
  const int g_build = tid / 16, sub = tid % 16;  // this thread builds entries 8 sub .. 8 sub + 7 of group g_build
  auto request = [&](int tc, Column& c) {
    const uint32_t t0 = p.tile_off[tr * p.ntc + tc], t1 = p.tile_off[tr * p.ntc + tc + 1];
    c.b = (int)(t1 - t0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (active && i < c.b)
        c.w[i] = *reinterpret_cast<const u32x4*>(p.planes + ((size_t)t0 + i) * kLutPlaneBytes + (size_t)r * 16);
    c.s = 0.f, c.z = 0.f;
    if (active) {
      c.s = (float)p.scales[(size_t)tc * p.N + n];
      c.z = (float)p.zeros[(size_t)tc * p.N + n];
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int k = tc * kTile + 8 * g_build + t;
      c.x[t] = (float)p.X[p.col_perm ? p.col_perm[k] : k];
    }
  };

  float y = 0.f;
  Column cur, nxt;
  if (tc_begin < tc_end) request(tc_begin, cur);
  for (int tc = tc_begin; tc < tc_end; ++tc) {
    const int buf = (tc - tc_begin) & 1;
    if (tc + 1 < tc_end) request(tc + 1, nxt);
    // ---- tables of this tile column
    {
      const float* x = cur.x;
      // bits 3..6 of the index come from sub, bit 7 is 0, bits 0..2 are filled in below
      float base = -x[0] - x[1] - x[2] - x[7];
#pragma unroll
      for (int t = 3; t < 7; ++t) base += ((sub >> (t - 3)) & 1) ? x[t] : -x[t];
      float e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        e[j] = base + 2.f * (((j & 1) ? x[0] : 0.f) + ((j & 2) ? x[1] : 0.f) + ((j & 4) ? x[2] : 0.f));
      entry_t* dst = &lut[buf][g_build][sub * 8];
      if constexpr (H16) {
        half8 h;
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = (_Float16)e[j];  // round to nearest even, once per entry
        *reinterpret_cast<half8*>(dst) = h;
      } else {
        *reinterpret_cast<floatx4*>(dst) = floatx4{e[0], e[1], e[2], e[3]};
        *reinterpret_cast<floatx4*>(dst + 4) = floatx4{e[4], e[5], e[6], e[7]};
      }
    }
    __syncthreads();  // (the other buffer is still being read by slower wavefronts: hence two buffers)
    if (active) {
      // sum of the column's activations = minus the sum of the entries with every sign negative
      float sum_x = 0.f;
#pragma unroll
      for (int g = 0; g < 16; ++g) sum_x -= (float)lut[buf][g][0];
      float total = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (i < cur.b) {
          float plane_sum = 0.f;
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const uint32_t word = cur.w[i][d];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int g = 4 * d + q;
              const int32_t top = (int32_t)(word << (24 - 8 * q)) >> 31;  // all ones if the byte's top bit is set
              const uint32_t idx = ((word >> (8 * q)) ^ (uint32_t)top) & 0x7Fu;
              const float v = (float)lut[buf][g][idx];  // (fp16 -> fp32 is exact)
              plane_sum += __uint_as_float(__float_as_uint(v) ^ ((uint32_t)top & 0x80000000u));
            }
          }
          total += (float)(1 << i) * plane_sum;
        }
      }
      const float s_hat = 0.5f * cur.s;
      const float z_hat = cur.z + 0.5f * (float)((1 << cur.b) - 1) * cur.s;
      y += s_hat * total + z_hat * sum_x;
    }
    cur = nxt;
  }
  if (active) p.partial[(size_t)ks * p.N + n] = y;
}

// fixed-order sum of the K ranges; the loads of 8 ranges are in flight together (one thread per output feature
// would otherwise wait for up to ksplit dependent trips to memory)
__global__ __launch_bounds__(64) void lut_reduce_kernel(const float* __restrict__ partial, const int32_t* __restrict__ row_perm,
                                                       _Float16* __restrict__ Y, int N, int ksplit) {
  const int n = (int)blockIdx.x * 64 + (int)threadIdx.x;
  if (n >= N) return;
  const int32_t col = row_perm ? row_perm[n] : n;
  float sum = 0.f;
  for (int k0 = 0; k0 < ksplit; k0 += 8) {
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = k0 + j < ksplit ? partial[(size_t)(k0 + j) * N + n] : 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) sum += v[j];
  }
  Y[col] = (_Float16)sum;
}

static int lut_ksplit(int32_t N, int32_t K) {
  const int nrb = (N + kLutThreads - 1) / kLutThreads, ntc = K / kTile;
  int ks = (kLutTargetGroups + nrb - 1) / nrb;
  return ks < 1 ? 1 : ks > ntc ? ntc : ks;
}

}  // namespace sfmp

extern "C" {

int sfmp_lut_gemv_workspace(int32_t N, int32_t K, int64_t* bytes) {
  if (!bytes) return SFMP_ERR_NULL;
  if (int e = sfmp::check_shape(N, K)) return e;
  *bytes = sfmp::round_up_256((int64_t)sfmp::lut_ksplit(N, K) * N * 4);
  return SFMP_OK;
}

int sfmp_lut_gemv(const void* X_dev, const int32_t* col_perm_dev, int32_t N, int32_t K, const void* planes_dev,
                  const uint32_t* tile_off_dev, const void* scales_dev, const void* zeros_dev,
                  const int32_t* row_perm_dev, void* Y_dev, int32_t table_format, void* workspace_dev,
                  int64_t workspace_bytes, void* hip_stream) {
  using namespace sfmp;
  if (!X_dev || !planes_dev || !tile_off_dev || !scales_dev || !zeros_dev || !Y_dev) return SFMP_ERR_NULL;
  if (int e = check_shape(N, K)) return e;
  if (table_format != SFMP_LUT_TABLE_FP32 && table_format != SFMP_LUT_TABLE_FP16) return SFMP_ERR_LAYOUT;
  const int ks = lut_ksplit(N, K);
  const int64_t need = round_up_256((int64_t)ks * N * 4);
  if (!workspace_dev || ((uintptr_t)workspace_dev & 255) != 0 || workspace_bytes < need) return SFMP_ERR_WORKSPACE;
  LutParams p;
  p.X = (const _Float16*)X_dev;
  p.col_perm = col_perm_dev;
  p.planes = (const uint8_t*)planes_dev;
  p.tile_off = tile_off_dev;
  p.scales = (const _Float16*)scales_dev;
  p.zeros = (const _Float16*)zeros_dev;
  p.partial = (float*)workspace_dev;
  p.N = N;
  p.K = K;
  p.ntc = K / kTile;
  p.ksplit = ks;
  const unsigned nrb = (unsigned)((N + kLutThreads - 1) / kLutThreads);
  if (table_format == SFMP_LUT_TABLE_FP16)
    hipLaunchKernelGGL(lut_gemv_kernel<true>, dim3(nrb * (unsigned)ks), dim3(kLutThreads), 0, (hipStream_t)hip_stream, p);
  else
    hipLaunchKernelGGL(lut_gemv_kernel<false>, dim3(nrb * (unsigned)ks), dim3(kLutThreads), 0, (hipStream_t)hip_stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error("sfmp_lut_gemv launch", hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  hipLaunchKernelGGL(lut_reduce_kernel, dim3((unsigned)((N + 63) / 64)), dim3(64), 0, (hipStream_t)hip_stream,
                     (const float*)workspace_dev, row_perm_dev, (_Float16*)Y_dev, (int)N, ks);
  e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error("sfmp_lut_gemv reduction launch", hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return SFMP_OK;
}

}  // extern "C"
