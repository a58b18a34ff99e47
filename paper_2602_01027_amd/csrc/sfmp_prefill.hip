// Prefill path (M > 16): dequantise-to-LDS + fp16 MFMA GEMM for gfx950.
//
// Step 1 (only when a column permutation is given): Xp[m, j] = X[m, col_perm[j]] is written
// once to the workspace by a row-through-LDS gather (coalesced read of a whole row,
// coalesced 16-byte writes).  A random column gather inside the GEMM would turn every
// 2-byte element into its own cache-line request for every one of the N/128 workgroups that
// need it; doing it once costs 4*M*K bytes of streaming traffic instead.
//
// Step 2: workgroup = 128 (M) x 128 (N, one tile row) output block, 4 wavefronts in a 2x2
// arrangement of 64x64 sub-blocks, K walked one 128x128 weight tile (= one quantisation
// group) at a time.  Per step the packed tile (4-8 KiB) is loaded slab by slab (4*b bytes per lane),
// unpacked with the shared routines, dequantised exactly to fp16 (w = fp16(s*q + z), one
// rounding, Appendix B Eq. 11) and stored to LDS; the activation block is copied to LDS; both
// are then read as 16x16x32 MFMA operands (fp32 accumulate).  Rows of both LDS blocks are
// 256 bytes with their 16-byte units XOR-swizzled by (row%16)^(row/16) so that operand reads
// (16 consecutive rows) and dequant writes (rows 8 apart) are bank-conflict free.
// Global loads of step t+1 are issued before the MFMAs of step t (register prefetch).
// Epilogue: fp32 -> fp16 (RNE) and the row scatter Y[m, row_perm[n]].
#include "sfmp_device.h"
#include "sfmp_internal.h"

namespace sfmp {

// -------------------------------------------------------------------------------------------
// column gather
// -------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_cols_kernel(const _Float16* __restrict__ X,
                                                          const int32_t* __restrict__ col_perm,
                                                          _Float16* __restrict__ Xp, int K) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  _Float16* row = reinterpret_cast<_Float16*>(lds_raw);
  const int64_t m = blockIdx.x;
  const uint4* src = reinterpret_cast<const uint4*>(X + m * K);
  for (int i = threadIdx.x; i < K / 8; i += 256) reinterpret_cast<uint4*>(row)[i] = src[i];
  __syncthreads();
  uint4* dst = reinterpret_cast<uint4*>(Xp + m * K);
  for (int i = threadIdx.x; i < K / 8; i += 256) {
    const int4 c0 = reinterpret_cast<const int4*>(col_perm)[2 * i];
    const int4 c1 = reinterpret_cast<const int4*>(col_perm)[2 * i + 1];
    union {
      _Float16 h[8];
      uint4 u;
    } v;
    v.h[0] = row[c0.x];
    v.h[1] = row[c0.y];
    v.h[2] = row[c0.z];
    v.h[3] = row[c0.w];
    v.h[4] = row[c1.x];
    v.h[5] = row[c1.y];
    v.h[6] = row[c1.z];
    v.h[7] = row[c1.w];
    dst[i] = v.u;
  }
}

// -------------------------------------------------------------------------------------------
// dequant + MFMA GEMM
// -------------------------------------------------------------------------------------------
struct PrefillParams {
  const _Float16* Xp;  // [M, K], columns already in reordered order
  const uint8_t* s2;
  const uint8_t* s3;
  const uint8_t* s4;
  const int32_t* tile_desc;
  const _Float16* scales;
  const _Float16* zeros;
  const int32_t* row_perm;
  _Float16* Y;
  int32_t M, N, K, ntr, ntc, n_mtiles;
};

constexpr int kBM = 128;

__device__ __forceinline__ int swz(int row, int unit) { return unit ^ ((row & 15) ^ ((row >> 4) & 7)); }

// Exact fp16 dequantisation of one slab and store to the LDS weight block.
template <int B>
__device__ __forceinline__ void dequant_slab_to_lds(const uint32_t* w, _Float16 s, _Float16 z, _Float16* Ws, int row,
                                                    int kb) {
  uint32_t op[4][4];
  unpack_slab<B>(w, op);
  const half2_ s2 = {s, s}, z2 = {z, z};
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa) {
    const int p = step_pos<B>(kappa);
    const _Float16 inv = (_Float16)(1.0f / (float)(1 << p));
    const _Float16 off = (_Float16)(-1024.0f / (float)(1 << p));
    const half2_ inv2 = {inv, inv}, off2 = {off, off};
    union {
      half2_ h[4];
      uint4 u;
    } out;
#pragma unroll
    for (int reg = 0; reg < 4; ++reg) {
      union {
        uint32_t u;
        half2_ h;
      } t;
      t.u = op[kappa][reg] | 0x64006400u;                           // 1024 + q*2^p in both halves
      const half2_ q = __builtin_elementwise_fma(t.h, inv2, off2);  // exact: q in [0, 15]
      out.h[reg] = __builtin_elementwise_fma(q, s2, z2);            // one rounding
    }
    const int unit = 4 * kappa + kb;
    *reinterpret_cast<uint4*>(Ws + row * 128 + swz(row, unit) * 8) = out.u;
  }
}

__global__ __launch_bounds__(256) void prefill_kernel(const PrefillParams p) {
  __shared__ __align__(16) _Float16 Xs[kBM * 128];
  __shared__ __align__(16) _Float16 Ws[128 * 128];

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = tid / kWave;
  // blocks are dealt round-robin to the 8 XCDs: keep all tile rows of one M block on one XCD so
  // that its activation rows and its output rows stay in that XCD's L2.
  const int xcd = blockIdx.x % 8;
  const int within = blockIdx.x / 8;
  const int mt = xcd + 8 * (within / p.ntr);
  const int tr = within % p.ntr;
  if (mt >= p.n_mtiles) return;
  const int m0 = mt * kBM;

  const int wm = wave / 2, wn = wave % 2;
  floatx4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  // register staging for the next step
  uint4 xreg[8];
  uint32_t wreg[8];
  uint32_t szreg[2];  // (s, s') and (z, z') of slabs 2*wave, 2*wave+1
  int32_t desc;

  const int xrow = tid / 16, xunit = tid % 16;  // + 16*pass rows
  const int i16 = lane % 16, kb = lane / 16;
  const int nloc = 8 * i16 + 2 * wave;  // weight row (in tile) of slab 2*wave for this lane

  auto issue = [&](int tc) {
#pragma unroll
    for (int ps = 0; ps < 8; ++ps) {
      const int m = m0 + xrow + 16 * ps;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (m < p.M) v = *reinterpret_cast<const uint4*>(p.Xp + (int64_t)m * p.K + tc * 128 + xunit * 8);
      xreg[ps] = v;
    }
    desc = __builtin_amdgcn_readfirstlane(p.tile_desc[(int64_t)tr * p.ntc + tc]);
    const int64_t slot = desc >> 2;
    switch (desc & 3) {  // slabs 2*wave and 2*wave+1 of this lane
      case 0:
        load_slab_words<2>(p.s2 + slot * 4096, 2 * wave, lane, wreg);
        load_slab_words<2>(p.s2 + slot * 4096, 2 * wave + 1, lane, wreg + 2);
        break;
      case 1:
        load_slab_words<3>(p.s3 + slot * 6144, 2 * wave, lane, wreg);
        load_slab_words<3>(p.s3 + slot * 6144, 2 * wave + 1, lane, wreg + 3);
        break;
      default:
        load_slab_words<4>(p.s4 + slot * 8192, 2 * wave, lane, wreg);
        load_slab_words<4>(p.s4 + slot * 8192, 2 * wave + 1, lane, wreg + 4);
        break;
    }
    const int64_t off = (int64_t)tc * p.N + (int64_t)tr * 128 + nloc;
    szreg[0] = *reinterpret_cast<const uint32_t*>(p.scales + off);
    szreg[1] = *reinterpret_cast<const uint32_t*>(p.zeros + off);
  };

  issue(0);
  for (int tc = 0; tc < p.ntc; ++tc) {
    __syncthreads();  // previous step's MFMA reads of LDS are done
#pragma unroll
    for (int ps = 0; ps < 8; ++ps) {
      const int row = xrow + 16 * ps;
      *reinterpret_cast<uint4*>(Xs + row * 128 + swz(row, xunit) * 8) = xreg[ps];
    }
    {
      union {
        uint32_t u;
        half2_ h;
      } s, z;
      s.u = szreg[0];
      z.u = szreg[1];
      switch (desc & 3) {
        case 0:
          dequant_slab_to_lds<2>(wreg, s.h[0], z.h[0], Ws, nloc, kb);
          dequant_slab_to_lds<2>(wreg + 2, s.h[1], z.h[1], Ws, nloc + 1, kb);
          break;
        case 1:
          dequant_slab_to_lds<3>(wreg, s.h[0], z.h[0], Ws, nloc, kb);
          dequant_slab_to_lds<3>(wreg + 3, s.h[1], z.h[1], Ws, nloc + 1, kb);
          break;
        default:
          dequant_slab_to_lds<4>(wreg, s.h[0], z.h[0], Ws, nloc, kb);
          dequant_slab_to_lds<4>(wreg + 4, s.h[1], z.h[1], Ws, nloc + 1, kb);
          break;
      }
    }
    __syncthreads();
    if (tc + 1 < p.ntc) issue(tc + 1);
#pragma unroll
    for (int kappa = 0; kappa < 4; ++kappa) {
      half8 a[4], b[4];
      const int unit = 4 * kappa + kb;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 64 * wm + 16 * i + i16;
        a[i] = *reinterpret_cast<const half8*>(Xs + row * 128 + swz(row, unit) * 8);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = 64 * wn + 16 * j + i16;
        b[j] = *reinterpret_cast<const half8*>(Ws + row * 128 + swz(row, unit) * 8);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue: acc[i][j][r] = C[m0 + 64wm + 16i + 4*kb + r][128tr + 64wn + 16j + i16]
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t n = (int64_t)tr * 128 + 64 * wn + 16 * j + i16;
    const int64_t col = p.row_perm ? p.row_perm[n] : n;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + 64 * wm + 16 * i + 4 * kb + r;
        if (m < p.M) p.Y[(int64_t)m * p.N + col] = (_Float16)acc[i][j][r];
      }
  }
}

PrefillPlan make_prefill_plan(int32_t N, int32_t K, int32_t M) {
  PrefillPlan d;
  (void)N;
  d.xperm_bytes = round_up_256((int64_t)M * K * 2);
  return d;
}

int launch_prefill(const GemmArgs& a, void* stream) {
  const sfmp_layout_t* L = a.L;
  const _Float16* Xp = (const _Float16*)a.X;
  if (a.col_perm) {
    _Float16* dst = (_Float16*)a.workspace;
    hipLaunchKernelGGL(gather_cols_kernel, dim3((unsigned)a.M), dim3(256), (size_t)L->K * 2, (hipStream_t)stream,
                       (const _Float16*)a.X, a.col_perm, dst, (int)L->K);
    Xp = dst;
  }
  PrefillParams p;
  p.Xp = Xp;
  p.s2 = a.s2;
  p.s3 = a.s3;
  p.s4 = a.s4;
  p.tile_desc = a.index + 3;
  p.scales = (const _Float16*)a.scales;
  p.zeros = (const _Float16*)a.zeros;
  p.row_perm = a.row_perm;
  p.Y = (_Float16*)a.Y;
  p.M = a.M;
  p.N = L->N;
  p.K = L->K;
  p.ntr = L->N / kTile;
  p.ntc = L->K / kTile;
  p.n_mtiles = (a.M + kBM - 1) / kBM;
  const unsigned grid = 8u * (unsigned)((p.n_mtiles + 7) / 8) * (unsigned)p.ntr;
  hipLaunchKernelGGL(prefill_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error("sfmp_gemm prefill launch", hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return SFMP_OK;
}

}  // namespace sfmp
