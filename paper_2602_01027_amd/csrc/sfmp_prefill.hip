// Prefill path (M > 16): dequantise-to-LDS + fp16 MFMA GEMM for gfx950.
//
// Three kernels on one stream:
//  1. gather_cols_kernel (only with a column permutation): Xp[m, j] = X[m, col_perm[j]], one row
//     through LDS per workgroup (coalesced read, coalesced 16-byte writes).  A random column gather
//     inside the GEMM would turn every 2-byte element into its own cache-line request for each of
//     the N/128 workgroups that need it; doing it once costs 4*M*K bytes of streaming traffic.
//  2. prefill_kernel: workgroup = 128 (M) x 128 (N, one tile row) output block, 4 wavefronts in a
//     2x2 arrangement of 64x64 sub-blocks, two workgroups per CU.  K is walked one 128x128 weight
//     tile (= one quantisation group) per step: packed slabs -> shared unpack routines -> exact q
//     (0x6400 magic + one exact FMA) -> fp16(s*q + z) with one FMA (Appendix B Eq. 11) -> LDS; the
//     activation block is copied to LDS; both are read as 16x16x32 MFMA operands (fp32 accumulate).
//     LDS rows are 256 bytes with 16-byte units XOR-swizzled by (row%16)^(row/16), so operand reads
//     (16 consecutive rows) and dequant writes (rows 8 apart) are bank-conflict free.  Weight loads
//     run TWO steps ahead of their use (two register sets, loop unrolled by two), activation
//     loads one step; the tile descriptors are read once into LDS.  With the descriptor load and one
//     step of look-ahead inside the loop every step waited a full memory latency (about 3000 cycles
//     against about 1000 cycles of MFMA work).
//  3. scatter_cols_kernel (only with a row permutation): the GEMM writes the product in reordered
//     row order with coalesced stores into the workspace, then Y[m, row_perm[i]] = Yt[m, i] is done
//     one row through LDS.  Scattering 2-byte results straight from the GEMM epilogue leaves
//     half-written cache lines all over Y and doubled the kernel time.
#include "sfmp_device.h"
#include "sfmp_internal.h"

namespace sfmp {

// -------------------------------------------------------------------------------------------
// column gather / column scatter, one row of fp16 through LDS per workgroup
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

// Y[m, row_perm[i]] = Yt[m, i]
__global__ __launch_bounds__(256) void scatter_cols_kernel(const _Float16* __restrict__ Yt,
                                                           const int32_t* __restrict__ row_perm,
                                                           _Float16* __restrict__ Y, int N) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  _Float16* row = reinterpret_cast<_Float16*>(lds_raw);
  const int64_t m = blockIdx.x;
  const uint4* src = reinterpret_cast<const uint4*>(Yt + m * N);
  for (int i = threadIdx.x; i < N / 8; i += 256) {
    const int4 c0 = reinterpret_cast<const int4*>(row_perm)[2 * i];
    const int4 c1 = reinterpret_cast<const int4*>(row_perm)[2 * i + 1];
    union {
      _Float16 h[8];
      uint4 u;
    } v;
    v.u = src[i];
    row[c0.x] = v.h[0];
    row[c0.y] = v.h[1];
    row[c0.z] = v.h[2];
    row[c0.w] = v.h[3];
    row[c1.x] = v.h[4];
    row[c1.y] = v.h[5];
    row[c1.z] = v.h[6];
    row[c1.w] = v.h[7];
  }
  __syncthreads();
  uint4* dst = reinterpret_cast<uint4*>(Y + m * N);
  for (int i = threadIdx.x; i < N / 8; i += 256) dst[i] = reinterpret_cast<const uint4*>(row)[i];
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
  _Float16* Yt;  // [M, N], rows of Wt in reordered order
  int32_t M, N, K, ntr, ntc, n_mtiles;
};

constexpr int kBM = 128;
constexpr int kPrefillMaxTiles = 224 * 2;  // K <= 57344

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
  __shared__ int32_t descs[kPrefillMaxTiles];

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  // blocks are dealt round-robin to the 8 XCDs: keep all tile rows of one M block on one XCD so
  // that its activation rows stay in that XCD's L2.
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

  const int xrow = tid / 16, xunit = tid % 16;  // + 16*pass rows
  const int i16 = lane % 16, kb = lane / 16;
  const int nloc = 8 * i16 + 2 * wave;  // weight row (in tile) of slab 2*wave for this lane

  // descriptors of this tile row, fetched once (a load of the descriptor inside the K loop would put
  // a dependent memory round trip in front of every step's weight loads)
  for (int i = tid; i < p.ntc; i += 256) descs[i] = p.tile_desc[(int64_t)tr * p.ntc + i];
  __syncthreads();

  // (clang vector types, not HIP uint4: arrays or structs of the HIP type stayed in scratch memory)
  struct XRegs {
    u32x4 v0, v1, v2, v3, v4, v5, v6, v7;
  };
#define SFMP_FOR8(M) M(0) M(1) M(2) M(3) M(4) M(5) M(6) M(7)
  auto issue_x = [&](int tc, XRegs& xr) __attribute__((always_inline)) {
    // rows past M re-read the last row (never stored): no branch, so the load count is fixed
#define SFMP_LDX(i)                                                                                             \
  xr.v##i = *reinterpret_cast<const u32x4*>(p.Xp + (int64_t)min(m0 + xrow + 16 * i, p.M - 1) * p.K + tc * 128 + \
                                            xunit * 8);
    SFMP_FOR8(SFMP_LDX)
#undef SFMP_LDX
  };
  // Same instruction sequence for every width (the compiler can then count outstanding loads exactly and
  // let younger loads stay in flight): four dword loads per slab; the words a narrower width does not
  // have re-read its last word.
  auto issue_w = [&](int tc, uint32_t (&rw)[8], uint32_t (&rsz)[2], int32_t& rdesc) __attribute__((always_inline)) {
    rdesc = __builtin_amdgcn_readfirstlane(descs[tc]);
    const int bw = (rdesc & 3) + 2;
    const uint8_t* stream = bw == 2 ? p.s2 : bw == 3 ? p.s3 : p.s4;
    const uint8_t* tile = stream + (int64_t)(rdesc >> 2) * (2048 * bw);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const uint32_t* src = reinterpret_cast<const uint32_t*>(tile + (2 * wave + q) * (256 * bw) + lane * (4 * bw));
#pragma unroll
      for (int i = 0; i < 4; ++i) rw[4 * q + i] = __builtin_nontemporal_load(src + (i < bw ? i : bw - 1));
    }
    const int64_t off = (int64_t)tc * p.N + (int64_t)tr * 128 + nloc;
    rsz[0] = *reinterpret_cast<const uint32_t*>(p.scales + off);
    rsz[1] = *reinterpret_cast<const uint32_t*>(p.zeros + off);
  };

  // One K step.  r holds the weights of tile tc and xr its activations.  Afterwards xr is refilled with
  // step tc+1 (mostly L2 hits: the M block is shared by all tile rows on this XCD) and r with step
  // tc+2 (first touch of a weight tile goes to HBM: it needs the longer look-ahead).  Loads past the
  // end re-read the last tile: unconditional, so that the counts stay exact.
  auto step = [&](int tc, XRegs& xr, uint32_t (&rw)[8], uint32_t (&rsz)[2], int32_t& rdesc) __attribute__((always_inline)) {
    __syncthreads();  // previous step's MFMA reads of LDS are done
#define SFMP_STX(i)                                                                 \
  {                                                                                 \
    const int row = xrow + 16 * i;                                                  \
    *reinterpret_cast<u32x4*>(Xs + row * 128 + swz(row, xunit) * 8) = xr.v##i;      \
  }
    SFMP_FOR8(SFMP_STX)
#undef SFMP_STX
    {
      union {
        uint32_t u;
        half2_ h;
      } s, z;
      s.u = rsz[0];
      z.u = rsz[1];
      switch (rdesc & 3) {
        case 0:
          dequant_slab_to_lds<2>(&rw[0], s.h[0], z.h[0], Ws, nloc, kb);
          dequant_slab_to_lds<2>(&rw[4], s.h[1], z.h[1], Ws, nloc + 1, kb);
          break;
        case 1:
          dequant_slab_to_lds<3>(&rw[0], s.h[0], z.h[0], Ws, nloc, kb);
          dequant_slab_to_lds<3>(&rw[4], s.h[1], z.h[1], Ws, nloc + 1, kb);
          break;
        default:
          dequant_slab_to_lds<4>(&rw[0], s.h[0], z.h[0], Ws, nloc, kb);
          dequant_slab_to_lds<4>(&rw[4], s.h[1], z.h[1], Ws, nloc + 1, kb);
          break;
      }
    }
    __syncthreads();
    issue_x(min(tc + 1, p.ntc - 1), xr);
    issue_w(min(tc + 2, p.ntc - 1), rw, rsz, rdesc);
#pragma unroll 1
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
  };

  uint32_t w0[8], w1[8], sz0[2], sz1[2];
  int32_t d0, d1;
  issue_w(0, w0, sz0, d0);
  issue_w(min(1, p.ntc - 1), w1, sz1, d1);
  XRegs xr;  // 8 rows x 16 bytes of the activation block of the next step
  issue_x(0, xr);
  int tc = 0;
  for (; tc + 1 < p.ntc; tc += 2) {
    step(tc, xr, w0, sz0, d0);
    step(tc + 1, xr, w1, sz1, d1);
  }
  if (tc < p.ntc) step(tc, xr, w0, sz0, d0);

  // epilogue: acc[i][j][r] = C[m0 + 64wm + 16i + 4*kb + r][128tr + 64wn + 16j + i16]; 16 lanes write 32
  // contiguous bytes of one row
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t n = (int64_t)tr * 128 + 64 * wn + 16 * j + i16;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + 64 * wm + 16 * i + 4 * kb + r;
        if (m < p.M) p.Yt[(int64_t)m * p.N + n] = (_Float16)acc[i][j][r];
      }
  }
}

PrefillPlan make_prefill_plan(int32_t N, int32_t K, int32_t M) {
  PrefillPlan d;
  d.xperm_bytes = round_up_256((int64_t)M * K * 2);
  d.ytmp_bytes = round_up_256((int64_t)M * N * 2);
  return d;
}

static int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error(what, hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return SFMP_OK;
}

int launch_prefill(const GemmArgs& a, void* stream) {
  const sfmp_layout_t* L = a.L;
  const PrefillPlan plan = make_prefill_plan(L->N, L->K, a.M);
  // the gather / scatter passes hold one fp16 row in LDS
  if ((a.col_perm && (int64_t)L->K * 2 > 160 * 1024) || (a.row_perm && (int64_t)L->N * 2 > 160 * 1024) ||
      L->K / kTile > kPrefillMaxTiles)
    return SFMP_ERR_SHAPE;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_cols_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void*>(&scatter_cols_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e1 != hipSuccess || e2 != hipSuccess) {
      note_hip_error("hipFuncSetAttribute(gather/scatter)", hipGetErrorString(e1 != hipSuccess ? e1 : e2));
      return SFMP_ERR_HIP;
    }
    attr_set = true;
  }
  const _Float16* Xp = (const _Float16*)a.X;
  if (a.col_perm) {
    _Float16* dst = (_Float16*)a.workspace;
    hipLaunchKernelGGL(gather_cols_kernel, dim3((unsigned)a.M), dim3(256), (size_t)L->K * 2, (hipStream_t)stream,
                       (const _Float16*)a.X, a.col_perm, dst, (int)L->K);
    if (int e = check_launch("sfmp_gemm column gather launch")) return e;
    Xp = dst;
  }
  _Float16* Yt = a.row_perm ? (_Float16*)((char*)a.workspace + plan.xperm_bytes) : (_Float16*)a.Y;
  PrefillParams p;
  p.Xp = Xp;
  p.s2 = a.s2;
  p.s3 = a.s3;
  p.s4 = a.s4;
  p.tile_desc = a.index + 3;
  p.scales = (const _Float16*)a.scales;
  p.zeros = (const _Float16*)a.zeros;
  p.Yt = Yt;
  p.M = a.M;
  p.N = L->N;
  p.K = L->K;
  p.ntr = L->N / kTile;
  p.ntc = L->K / kTile;
  p.n_mtiles = (a.M + kBM - 1) / kBM;
  const unsigned grid = 8u * (unsigned)((p.n_mtiles + 7) / 8) * (unsigned)p.ntr;
  hipLaunchKernelGGL(prefill_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, p);
  if (int e = check_launch("sfmp_gemm prefill launch")) return e;
  if (a.row_perm) {
    hipLaunchKernelGGL(scatter_cols_kernel, dim3((unsigned)a.M), dim3(256), (size_t)L->N * 2, (hipStream_t)stream,
                       (const _Float16*)Yt, a.row_perm, (_Float16*)a.Y, (int)L->N);
    if (int e = check_launch("sfmp_gemm row scatter launch")) return e;
  }
  return SFMP_OK;
}

}  // namespace sfmp
