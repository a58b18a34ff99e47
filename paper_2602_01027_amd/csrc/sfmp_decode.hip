// Decode path (M <= 16): bandwidth-bound mixed-precision GEMV / skinny GEMM for gfx950.
//
// Work split.  A workgroup is 4 wavefronts; wavefront w owns tile row 4*rowgroup + w and
// walks `tiles_per_chunk` consecutive 128x128 tiles of that row (one K chunk).  The tile's
// bit-width is read from the block-index table and selects, wavefront-uniformly, one of
// three specialised bodies: there is no divergence inside a wavefront.  The four tile rows
// of a workgroup share the K chunk, so the activation slice X[:, col_perm[chunk]] is
// gathered once per workgroup into LDS (the permutation is fused into this load).
//
// Per tile and lane: 2*B 16-byte loads (1 KiB contiguous per wavefront per load), one
// v_and_b32 per code pair (codes become fp16 denormals q*2^(p-24)), and 32 MFMA
// 16x16x32 instructions that contract the tile against the LDS-resident activations, whose
// slots were pre-multiplied by 2^(h-p).  The matrix pipe is used as the MAC engine of a
// memory-bound kernel: the VALU budget per weight at HBM speed (2-4 lane-ops) is spent on
// the unpack, and the MFMA cost does not grow with M up to 16.  Per 128-column group the
// fp32 MFMA result is scaled: acc += s*2^(24-h) * sum(q*x) + z * sum(x)   (Appendix B Eq. 11,
// re-associated per group), sum(x) coming from one extra MFMA against a vector of ones.
//
// K reduction.  Each wavefront stores its 128 x M fp32 partial; an arrival counter per tile
// row lets the last wavefront of a row add the partials in chunk order (deterministic),
// convert to fp16 (RNE) and scatter the row through row_perm.  Counters are left at zero.
#include "sfmp_device.h"
#include "sfmp_internal.h"

namespace sfmp {

struct DecodeParams {
  const _Float16* X;
  const int32_t* col_perm;
  const uint8_t* s2;
  const uint8_t* s3;
  const uint8_t* s4;
  const int32_t* tile_desc;
  const _Float16* scales;
  const _Float16* zeros;
  const int32_t* row_perm;
  _Float16* Y;
  float* partial;
  int32_t* counters;
  int32_t M, N, K, ntr, ntc, tiles_per_chunk, nchunk;
};

__host__ __device__ constexpr float pow2f(int e) {
  float v = 1.0f;
  for (int i = 0; i < e; ++i) v *= 2.0f;
  for (int i = 0; i < -e; ++i) v *= 0.5f;
  return v;
}

// Activation pre-scale for k-step kappa: slot v gets 2^(h - p(kappa, v/2)).
template <int B>
__device__ __forceinline__ half8 prescale(int kappa) {
  half8 f;
#pragma unroll
  for (int v = 0; v < 8; ++v) f[v] = (_Float16)pow2f(prescale_exp<B>() - field_pos<B>(kappa, v / 2));
  return f;
}

template <int B>
__device__ __forceinline__ void issue_tile_loads(const uint8_t* tile, int lane, uint32_t (&w)[32]) {
  const u32x4* src = reinterpret_cast<const u32x4*>(tile) + lane;
#pragma unroll
  for (int c = 0; c < 2 * B; ++c) {
    const u32x4 v = __builtin_nontemporal_load(src + c * 64);
    w[4 * c + 0] = v[0];
    w[4 * c + 1] = v[1];
    w[4 * c + 2] = v[2];
    w[4 * c + 3] = v[3];
  }
}

template <int B, int MR>
__device__ __forceinline__ void contract_tile(const uint32_t (&w)[32], const half8 (&a)[4], const floatx4& sx,
                                              const u32x4& sraw, const u32x4& zraw, float (&acc)[8][MR]) {
  half8 ap[4];
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa) ap[kappa] = a[kappa] * prescale<B>(kappa);
  union {
    u32x4 u;
    half8 h;
  } sc, zr;
  sc.u = sraw;
  zr.u = zraw;
  constexpr float kFix = pow2f(24 - prescale_exp<B>());
#pragma unroll
  for (int sigma = 0; sigma < 8; ++sigma) {
    uint32_t op[4][4];
    unpack_slab<B>(&w[sigma * B], op);
    floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kappa = 0; kappa < 4; ++kappa)
      c = __builtin_amdgcn_mfma_f32_16x16x32_f16(ap[kappa], as_half8(op[kappa][0], op[kappa][1], op[kappa][2], op[kappa][3]),
                                                 c, 0, 0, 0);
    const float s = (float)sc.h[sigma] * kFix;
    const float z = (float)zr.h[sigma];
#pragma unroll
    for (int r = 0; r < MR; ++r) acc[sigma][r] += s * c[r] + z * sx[r];
  }
}

template <int MR>
__global__ __launch_bounds__(256) void decode_kernel(const DecodeParams p) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  _Float16* Xs = reinterpret_cast<_Float16*>(lds_raw);  // [tile*16 + kblock][M][8]

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = tid / kWave;
  const int chunk = blockIdx.x % p.nchunk;
  const int rowgroup = blockIdx.x / p.nchunk;
  const int tr = rowgroup * 4 + wave;
  const bool active = tr < p.ntr;
  const int tc0 = chunk * p.tiles_per_chunk;
  const int ntile = min(p.tiles_per_chunk, p.ntc - tc0);
  const int M = p.M;

  // ---- first tile: descriptor, packed words, scales and zeros are requested before anything else
  uint32_t w[32];
  u32x4 sraw = {0, 0, 0, 0}, zraw = {0, 0, 0, 0};
  int32_t desc = 0;
  const int64_t sz_lane_off = (int64_t)(active ? tr : 0) * kTile + 8 * (lane % 16);
  if (active) {
    desc = __builtin_amdgcn_readfirstlane(p.tile_desc[(int64_t)tr * p.ntc + tc0]);
    const int64_t slot = desc >> 2;
    switch (desc & 3) {
      case 0: issue_tile_loads<2>(p.s2 + slot * 4096, lane, w); break;
      case 1: issue_tile_loads<3>(p.s3 + slot * 6144, lane, w); break;
      default: issue_tile_loads<4>(p.s4 + slot * 8192, lane, w); break;
    }
    sraw = *reinterpret_cast<const u32x4*>(p.scales + (int64_t)tc0 * p.N + sz_lane_off);
    zraw = *reinterpret_cast<const u32x4*>(p.zeros + (int64_t)tc0 * p.N + sz_lane_off);
  }

  // ---- gather the activation slice of this K chunk into LDS (column permutation fused here)
  {
    const int kspan = ntile * kTile;
    const int total = kspan * M;
    for (int idx = tid; idx < total; idx += 256) {
      const int m = idx / kspan;
      const int kl = idx - m * kspan;
      const int k = tc0 * kTile + kl;
      const int src = p.col_perm ? p.col_perm[k] : k;
      Xs[((kl >> 3) * M + m) * 8 + (kl & 7)] = p.X[(int64_t)m * p.K + src];
    }
  }
  __syncthreads();
  if (!active) return;

  float acc[8][MR];
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int r = 0; r < MR; ++r) acc[s][r] = 0.f;

  const int mrow = lane % 16;  // activation row this lane feeds to the MFMA A operand
  half8 ones;
#pragma unroll
  for (int v = 0; v < 8; ++v) ones[v] = (_Float16)1.0f;

  for (int t = 0; t < ntile; ++t) {
    if (t > 0) {
      desc = __builtin_amdgcn_readfirstlane(p.tile_desc[(int64_t)tr * p.ntc + tc0 + t]);
      const int64_t slot = desc >> 2;
      switch (desc & 3) {
        case 0: issue_tile_loads<2>(p.s2 + slot * 4096, lane, w); break;
        case 1: issue_tile_loads<3>(p.s3 + slot * 6144, lane, w); break;
        default: issue_tile_loads<4>(p.s4 + slot * 8192, lane, w); break;
      }
      sraw = *reinterpret_cast<const u32x4*>(p.scales + (int64_t)(tc0 + t) * p.N + sz_lane_off);
      zraw = *reinterpret_cast<const u32x4*>(p.zeros + (int64_t)(tc0 + t) * p.N + sz_lane_off);
    }
    // activation operand of the 4 k-steps of this tile and the per-row sums of x over the group
    half8 a[4];
    floatx4 sx = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kappa = 0; kappa < 4; ++kappa) {
      half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (mrow < M) v = *reinterpret_cast<const half8*>(Xs + ((t * 16 + kappa * 4 + lane / 16) * M + mrow) * 8);
      a[kappa] = v;
      sx = __builtin_amdgcn_mfma_f32_16x16x32_f16(v, ones, sx, 0, 0, 0);
    }
    switch (desc & 3) {
      case 0: contract_tile<2, MR>(w, a, sx, sraw, zraw, acc); break;
      case 1: contract_tile<3, MR>(w, a, sx, sraw, zraw, acc); break;
      default: contract_tile<4, MR>(w, a, sx, sraw, zraw, acc); break;
    }
  }

  // ---- K reduction and epilogue.  Lane (j = lane%16, g = lane/16) holds, for r < MR, the outputs
  // of activation row m = 4g + r and weight rows n = 128*tr + 8j + sigma.
  const int j = lane % 16, g = lane / 16;
  const int64_t n0 = (int64_t)tr * kTile + 8 * j;
  if (p.nchunk == 1) {
#pragma unroll
    for (int r = 0; r < MR; ++r) {
      const int m = 4 * g + r;
      if (m < M) {
#pragma unroll
        for (int sigma = 0; sigma < 8; ++sigma) {
          const int64_t n = n0 + sigma;
          const int64_t col = p.row_perm ? p.row_perm[n] : n;
          p.Y[(int64_t)m * p.N + col] = (_Float16)acc[sigma][r];
        }
      }
    }
    return;
  }
#pragma unroll
  for (int r = 0; r < MR; ++r) {
    const int m = 4 * g + r;
    if (m < M) {
      float* dst = p.partial + ((int64_t)chunk * M + m) * p.N + n0;
      reinterpret_cast<float4*>(dst)[0] = make_float4(acc[0][r], acc[1][r], acc[2][r], acc[3][r]);
      reinterpret_cast<float4*>(dst)[1] = make_float4(acc[4][r], acc[5][r], acc[6][r], acc[7][r]);
    }
  }
  __threadfence();  // release this wavefront's partial before announcing it
  int old = 0;
  if (lane == 0) old = atomicAdd(p.counters + tr, 1);
  old = __builtin_amdgcn_readfirstlane(old);
  if (old != p.nchunk - 1) return;
  __threadfence();  // acquire the other wavefronts' partials
  const int64_t n = (int64_t)tr * kTile + 2 * lane;
  int64_t c0 = n, c1 = n + 1;
  if (p.row_perm) {
    c0 = p.row_perm[n];
    c1 = p.row_perm[n + 1];
  }
  for (int m = 0; m < M; ++m) {
    float s0 = 0.f, s1 = 0.f;
    const float* src = p.partial + (int64_t)m * p.N + n;
    for (int c = 0; c < p.nchunk; ++c) {
      const float2 v = *reinterpret_cast<const float2*>(src + (int64_t)c * M * p.N);
      s0 += v.x;
      s1 += v.y;
    }
    p.Y[(int64_t)m * p.N + c0] = (_Float16)s0;
    p.Y[(int64_t)m * p.N + c1] = (_Float16)s1;
  }
  if (lane == 0) p.counters[tr] = 0;  // ready for the next call
}

DecodePlan make_decode_plan(int32_t N, int32_t K, int32_t M) {
  DecodePlan d;
  const int32_t ntr = N / kTile, ntc = K / kTile;
  // Few, long chunks keep the partial-sum traffic (128*M fp32 per wavefront, written and read
  // once) small next to the tile bytes; many chunks keep all 256 CUs busy.  Start from a chunk
  // length that grows with M and shorten it until about 2048 wavefronts exist.
  int32_t tpc = M <= 1 ? 4 : M <= 4 ? 4 : 8;
  while (tpc > 1 && (int64_t)ntr * ((ntc + tpc - 1) / tpc) < 2048) tpc /= 2;
  while (tpc * M > 128) tpc /= 2;  // LDS: tpc * M * 256 bytes <= 32 KiB
  if (tpc < 1) tpc = 1;
  d.tiles_per_chunk = tpc;
  d.nchunk = (ntc + tpc - 1) / tpc;
  d.row_groups = (ntr + 3) / 4;
  d.counter_bytes = round_up_256((int64_t)ntr * 4);
  d.partial_bytes = d.nchunk > 1 ? round_up_256((int64_t)d.nchunk * M * N * 4) : 0;
  d.lds_bytes = tpc * M * 256;
  return d;
}

int launch_decode(const GemmArgs& a, void* stream) {
  const sfmp_layout_t* L = a.L;
  const DecodePlan d = make_decode_plan(L->N, L->K, a.M);
  DecodeParams p;
  p.X = (const _Float16*)a.X;
  p.col_perm = a.col_perm;
  p.s2 = a.s2;
  p.s3 = a.s3;
  p.s4 = a.s4;
  p.tile_desc = a.index + 3;
  p.scales = (const _Float16*)a.scales;
  p.zeros = (const _Float16*)a.zeros;
  p.row_perm = a.row_perm;
  p.Y = (_Float16*)a.Y;
  p.counters = (int32_t*)a.workspace;
  p.partial = (float*)((char*)a.workspace + d.counter_bytes);
  p.M = a.M;
  p.N = L->N;
  p.K = L->K;
  p.ntr = L->N / kTile;
  p.ntc = L->K / kTile;
  p.tiles_per_chunk = d.tiles_per_chunk;
  p.nchunk = d.nchunk;
  const dim3 grid((unsigned)(d.row_groups * d.nchunk));
  if (a.M == 1)
    hipLaunchKernelGGL(decode_kernel<1>, grid, dim3(256), (size_t)d.lds_bytes, (hipStream_t)stream, p);
  else
    hipLaunchKernelGGL(decode_kernel<4>, grid, dim3(256), (size_t)d.lds_bytes, (hipStream_t)stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error("sfmp_gemm decode launch", hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return SFMP_OK;
}

}  // namespace sfmp
