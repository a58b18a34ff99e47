// Prefill path (M > 16): fp16 MFMA GEMM with the weights dequantised in registers, for gfx950.
//
// Three kernels on one stream:
//  1. gather_cols_kernel: Xp[m, j] = X[m, col_perm[j]] (identity without a permutation), one row through
//     LDS per workgroup (coalesced read, coalesced 16-byte writes), written as contiguous 128x128 blocks so
//     that a GEMM step reads 32 contiguous KiB instead of 128 row pieces K*2 bytes apart (10 % faster
//     GEMM).  A random column gather inside the GEMM would turn every 2-byte element into its own
//     cache-line request for each of the N/128 workgroups that need it; doing it once costs 4*M*K bytes
//     of streaming traffic.
//  2. prefill_kernel: workgroup = 128 (M) x 128 (N, one tile row) output block, 4 wavefronts, each
//     128 rows x 32 columns (two slabs), two workgroups per CU.  K is walked one 128x128 weight tile
//     (= one quantisation group) per step, the tiles of the tile row sorted by width (the order of a
//     sum is free, and the CSR part of the block-index table lists exactly these runs): three loops,
//     each with a straight-line body for its width.  A packed slab is already laid out as an MFMA B
//     operand (lane = weight row-in-16 x k-block of 8), so the weights never touch LDS: each
//     wavefront loads the slabs of its own output columns and dequantises them in registers (mask-or
//     into the 0x6400 magic, exact q, then fp16(s*q + z) with one FMA, Appendix B Eq. 11) straight
//     into the B operands of v_mfma_f32_16x16x32_f16; every operand feeds eight MFMAs.  The activation
//     block goes from global memory directly into LDS (LDS-DMA, double-buffered, 256-byte rows,
//     16-byte units XOR-swizzled by row%16: conflict-free operand reads whose addresses differ by
//     immediates).  A step is software-pipelined over its four k-steps and into the next step; one
//     barrier per step.  The product leaves through LDS in whole 256-byte row segments.
//  3. scatter_cols_kernel (only with a row permutation): the GEMM writes the product in reordered
//     row order into the workspace, then Y[m, row_perm[i]] = Yt[m, i] is done one row through LDS.
//     Scattering 2-byte results straight from the GEMM epilogue leaves half-written cache lines all
//     over Y and doubled the kernel time.
#include <cstdlib>
#include <type_traits>

#include "sfmp_device.h"
#include "sfmp_internal.h"

namespace sfmp {

// -------------------------------------------------------------------------------------------
// column gather / column scatter, one row of fp16 through LDS per workgroup
// -------------------------------------------------------------------------------------------
// R rows per workgroup: the permutation entries of a unit of 8 columns are loaded once and serve all R rows (they
// are twice the bytes of the data they steer), and R rows of loads are in flight per workgroup.
template <int R>
__global__ __launch_bounds__(1024) void gather_cols_kernel(const _Float16* __restrict__ X,
                                                           const int32_t* __restrict__ col_perm,
                                                           _Float16* __restrict__ Xp, int M, int K) {
  // Output layout: blocks of 128 rows x 128 columns, each block contiguous (32 KiB), block (mt, tc) at
  // (mt * K/128 + tc) * 16384 elements: the GEMM then reads one contiguous block per step instead of 128
  // row pieces K*2 bytes apart.
  extern __shared__ __align__(16) unsigned char lds_raw[];
  _Float16* rows = reinterpret_cast<_Float16*>(lds_raw);  // [R][K]
  const int64_t m0 = (int64_t)blockIdx.x * R;
  const int units = K / 8;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    if (m0 + r < M) {
      const uint4* src = reinterpret_cast<const uint4*>(X + (m0 + r) * K);
      for (int i = threadIdx.x; i < units; i += 1024) reinterpret_cast<uint4*>(rows + (size_t)r * K)[i] = src[i];
    }
  }
  __syncthreads();
  const int64_t ntc = K / kTile;
  for (int i = threadIdx.x; i < units; i += 1024) {
    int4 c0 = int4{8 * i, 8 * i + 1, 8 * i + 2, 8 * i + 3}, c1 = int4{8 * i + 4, 8 * i + 5, 8 * i + 6, 8 * i + 7};
    if (col_perm) {  // (no permutation: the pass only changes the layout)
      c0 = reinterpret_cast<const int4*>(col_perm)[2 * i];
      c1 = reinterpret_cast<const int4*>(col_perm)[2 * i + 1];
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t m = m0 + r;
      if (m < M) {
        const _Float16* row = rows + (size_t)r * K;
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
        _Float16* dst = Xp + (m / kTile) * ntc * (kTile * kTile) + (m % kTile) * kTile;
        *reinterpret_cast<uint4*>(dst + (int64_t)(i / 16) * (kTile * kTile) + (i % 16) * 8) = v.u;
      }
    }
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

// Y[m, row_perm[i]] (or Y[m, i]) = fp16( sum over the K ranges, in range order, of partial[ks][m][i] ): the second
// half of a split-K product, one row through LDS per workgroup.
__global__ __launch_bounds__(1024) void reduce_split_kernel(const float* __restrict__ partial, int ksplit, int M,
                                                            const int32_t* __restrict__ row_perm,
                                                            _Float16* __restrict__ Y, int N) {
  // (1024 threads and all loads of a thread's column group issued before the sum: with few rows there are few
  // workgroups, and a chain of dependent round trips per thread made this pass longer than the GEMM)
  extern __shared__ __align__(16) unsigned char lds_raw[];
  _Float16* row = reinterpret_cast<_Float16*>(lds_raw);
  const int64_t m = blockIdx.x;
  for (int i = threadIdx.x; i < N / 4; i += 1024) {
    floatx4 v[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      v[ks] = ks < ksplit ? *reinterpret_cast<const floatx4*>(partial + ((int64_t)ks * M + m) * N + 4 * i)
                          : floatx4{0.f, 0.f, 0.f, 0.f};
    floatx4 s = v[0];
#pragma unroll
    for (int ks = 1; ks < 8; ++ks) s += v[ks];  // range order; the ranges past ksplit add zeros
    if (row_perm) {
      const int4 c = reinterpret_cast<const int4*>(row_perm)[i];
      row[c.x] = (_Float16)s[0];
      row[c.y] = (_Float16)s[1];
      row[c.z] = (_Float16)s[2];
      row[c.w] = (_Float16)s[3];
    } else {
      row[4 * i] = (_Float16)s[0];
      row[4 * i + 1] = (_Float16)s[1];
      row[4 * i + 2] = (_Float16)s[2];
      row[4 * i + 3] = (_Float16)s[3];
    }
  }
  __syncthreads();
  uint4* dst = reinterpret_cast<uint4*>(Y + m * N);
  for (int i = threadIdx.x; i < N / 8; i += 1024) dst[i] = reinterpret_cast<const uint4*>(row)[i];
}

// -------------------------------------------------------------------------------------------
// dequant + MFMA GEMM
// -------------------------------------------------------------------------------------------
struct PrefillParams {
  const _Float16* Xp;  // staged activations, columns in reordered order, as contiguous 128x128 blocks (mt, tc)
  const uint8_t* s2;
  const uint8_t* s3;
  const uint8_t* s4;
  const int32_t* index;  // the whole block-index table
  const _Float16* scales;
  const _Float16* zeros;
  _Float16* Yt;  // [M, N], rows of Wt in reordered order
  int32_t M, N, K, ntr, ntc, n_mtiles;
  int32_t gshift;  // log2(group / 128): tile column tc uses parameter row tc >> gshift
  int32_t bf16;    // scales and zeros are bfloat16 (else fp16)
  int32_t ksplit;  // K ranges (1 = the whole K in one workgroup)
  float* partial;  // ksplit > 1: fp32 partial products [ksplit][M][N], rows of Wt in reordered order
};

constexpr int kPrefillMaxTiles = 224 * 2;  // K <= 57344

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// 16 bytes per lane from global memory straight into LDS at lds_base + 16*lane.  Written as inline
// assembly so that the compiler's wait-count bookkeeping does not see it: the kernel orders these
// loads itself (they complete in issue order with the ordinary loads around them).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // m0 is named as clobbered on purpose
__device__ __forceinline__ void load_to_lds_16(const void* base, uint32_t byte_offset, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0" ::"s"(base), "v"(byte_offset), "s"(lds_base)
               : "memory", "m0");
}
#pragma clang diagnostic pop

// 256-byte LDS rows of the activation block: 16-byte unit u of row r is stored at position u ^ (r % 16).  The 16
// rows that one quarter of a wavefront reads for an MFMA operand then hit 16 different positions (all 64
// banks once), and the position does not depend on the 16-row block, so operand addresses of a lane differ
// by multiples of 4096 bytes: immediate offsets.
__device__ __forceinline__ int swz(int row, int unit) { return unit ^ (row & 15); }

// One MFMA B operand in registers: the 16 weight rows {8i + sigma} x the 32 columns of k-step KAPPA of a
// slab, dequantised exactly: q from the 0x6400 magic (1024 + q*2^p) by one exact FMA, then
// fp16(s*q + z) by one FMA (Appendix B Eq. 11, a single rounding).  `magic` is 0x64006400 held in a
// vector register so that mask-and-or is one instruction (two literals do not fit into one).
template <int B, int KAPPA>
__device__ __forceinline__ half8 dequant_operand(const uint32_t* w, half2_ s2, half2_ z2, uint32_t magic) {
  uint32_t op[4][4];
  unpack_slab<B>(w, op);  // the other k-steps are dead code here and shared between the four calls
  constexpr int p = step_pos<B>(KAPPA);
  const _Float16 inv = (_Float16)(1.0f / (float)(1 << p));
  const _Float16 off = (_Float16)(-1024.0f / (float)(1 << p));
  const half2_ inv2 = {inv, inv}, off2 = {off, off};
  union {
    half2_ h[4];
    half8 v;
  } out;
#pragma unroll
  for (int reg = 0; reg < 4; ++reg) {
    union {
      uint32_t u;
      half2_ h;
    } t;
    t.u = op[KAPPA][reg] | magic;
    const half2_ q = __builtin_elementwise_fma(t.h, inv2, off2);  // exact: q in [0, 15]
    out.h[reg] = __builtin_elementwise_fma(q, s2, z2);            // one rounding
  }
  return out.v;
}

// Workgroup = BM x 128 output block, WM x WN wavefronts, wavefront tile (BM/WM) x (128/WN): MI = BM/WM/16
// row blocks x NS = 8/WN slabs.  A dequantised B operand feeds MI MFMAs, so the dequantisation cost per
// MFMA falls with MI; the activation operand reads from LDS grow with WN.
template <int BM, int WM, int WN>
struct PrefillShape {
  static constexpr int kThreads = 64 * WM * WN;
  static constexpr int kMI = BM / WM / 16;
  static constexpr int kNS = 8 / WN;
  static constexpr int kRowsPerPass = kThreads / 16;
  static constexpr int kPasses = BM / kRowsPerPass;
};

// G64: group length 64 - a tile column has two (scale, zero) pairs per row, one for its k-steps 0-1 and one for 2-3.
template <int BM, int WM, int WN, int IL = 2, bool G64 = false>
__global__ __launch_bounds__(64 * WM * WN, (BM <= 128 ? 2 : 1) * ((WM * WN + 3) / 4)) void prefill_kernel(const PrefillParams p) {
  using S = PrefillShape<BM, WM, WN>;
  constexpr int MI = S::kMI, NS = S::kNS;
  constexpr uint32_t kBufBytes = BM * 256;
  __shared__ __align__(16) unsigned char Xs[2 * kBufBytes];  // activation block, double-buffered
  __shared__ int32_t seq[kPrefillMaxTiles];                  // (slot << 9) | tc of this tile row, width-sorted

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  // Work items (tile row, M block) are numbered with the M blocks innermost, and block b (which runs on XCD
  // b % 8) takes item b.  With a multiple of 8 M blocks an XCD always sees the same M blocks (their activation
  // rows stay in its L2), and in any case the blocks that run at the same time need the same weight tiles, so
  // a tile comes from HBM once per XCD, not once per M block.  (Every XCD works for any number of M blocks.)
  // With K split into ranges (few workgroups otherwise: short prompts), the ranges of an item are innermost.
  const int ks = (int)blockIdx.x % p.ksplit;
  const int mt = ((int)blockIdx.x / p.ksplit) % p.n_mtiles;
  const int tr = ((int)blockIdx.x / p.ksplit) / p.n_mtiles;
  const int m0 = mt * BM;
  // this workgroup's share of the width-sorted tile sequence: positions [e_first, e_end)
  const int e_first = (int)((int64_t)ks * p.ntc / p.ksplit), e_end = (int)((int64_t)(ks + 1) * p.ntc / p.ksplit);
  const int e_last = e_end - 1;

  // The K reduction runs over the tiles of this tile row sorted by width (first all 2-bit tiles, then
  // the 3-bit, then the 4-bit ones; the order of a sum is free): three loops, each with a straight-line
  // body for its width.  The CSR part of the block-index table lists exactly these runs: the i-th
  // width-b tile of row tr is tile number row_ptr_b[tr] + i of stream S_b, in tile column
  // col_idx_b[row_ptr_b[tr] + i].
  const int32_t* row_ptr = p.index + 3 + p.ntr * p.ntc;
  const int32_t* col_idx = row_ptr + 3 * (p.ntr + 1);
  const int32_t first2 = row_ptr[tr], first3 = row_ptr[(p.ntr + 1) + tr], first4 = row_ptr[2 * (p.ntr + 1) + tr];
  const int end2 = row_ptr[tr + 1] - first2;
  const int end3 = end2 + row_ptr[(p.ntr + 1) + tr + 1] - first3;
  const int32_t total2 = p.index[0], total3 = p.index[1];
  for (int e = tid; e < p.ntc; e += S::kThreads) {
    // Position in its stream, and position of that stream's column list.  Each tile row walks its runs
    // from a slightly different starting point: the workgroups of one XCD all read the same activation rows,
    // and 256-byte pieces at the same tile column of rows K*2 bytes apart sit in the same L2 channel, so
    // workgroups marching exactly in step would all queue at one channel.  The starting points lie within 8
    // tiles of each other, no further: the workgroups that share an M block then sweep the tile columns
    // together, in ascending order inside a run, and an activation block that one of them has brought into
    // the XCD's L2 is still there for the others.  (With starting points spread over the whole run, as they
    // were at first, every workgroup streamed its M block by itself as soon as that no longer fitted in L2:
    // 6.9 GB fetched per call on 28672 -> 8192 at M = 2048 instead of 1.9 GB, 1003 us instead of 901.)
    const int32_t lo = e < end2 ? 0 : e < end3 ? end2 : end3;
    const int32_t n = (e < end2 ? end2 : e < end3 ? end3 : p.ntc) - lo;
    const int32_t i = (e - lo + (tr * 5) % 8) % n;
    const int32_t slot = (e < end2 ? first2 : e < end3 ? first3 : first4) + i;
    const int32_t cols = e < end2 ? 0 : e < end3 ? total2 : total2 + total3;
    seq[e] = (slot << 9) | col_idx[cols + slot];
  }
  __syncthreads();

  const int wm = wave / WN, wn = wave % WN;  // this wavefront: rows 16*MI*wm.., slabs NS*wn .. NS*wn+NS-1
  floatx4 acc[MI][NS];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NS; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int xrow = tid / 16, xunit = tid % 16;  // + kRowsPerPass*pass rows
  const int i16 = lane % 16, kb = lane / 16;
  uint32_t magic;
  asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(magic));

  // The activation block goes from global memory straight into LDS (no staging registers).  A 16-byte
  // LDS-DMA load of a wavefront fills 1024 contiguous bytes = four 256-byte rows, lane l -> row l/16,
  // 16-byte position l%16; the swizzle is applied on the global side: position u of row r receives
  // unit u ^ (r%16).
  uint32_t xoff[S::kPasses];  // byte offsets from Xp + m0*K + tc*128
#pragma unroll
  for (int i = 0; i < S::kPasses; ++i) {
    const int row = xrow + S::kRowsPerPass * i;
    xoff[i] = 2u * (uint32_t)(row * kTile + swz(row, xunit) * 8);
  }
  // block (mt, tc) of the staged activations starts at (mt * ntc + tc) * 16384 elements; rows past M of the last
  // row block are never written and feed only output rows that are never stored
  const _Float16* xbase = p.Xp + (int64_t)(m0 / kTile) * p.ntc * (kTile * kTile) + (m0 % kTile) * kTile;
  constexpr int xstep = kTile * kTile;  // elements between consecutive tile columns
  const uint32_t xs_base = (uint32_t)(uintptr_t)(lptr_t)Xs;
  // block of tile position e into the buffer that block `like` uses (like = e mod 2, except for the idle
  // loads past the end)
  auto issue_x = [&](int e, int like) __attribute__((always_inline)) {
    const int tc = __builtin_amdgcn_readfirstlane(seq[e]) & 511;
    const uint32_t dst = xs_base + (like & 1) * kBufBytes + wave * 1024;
    const _Float16* src = xbase + (int64_t)tc * xstep;
#pragma unroll
    for (int i = 0; i < S::kPasses; ++i) load_to_lds_16(src, xoff[i], dst + i * (S::kRowsPerPass * 256));
  };
  // operand read addresses: row 16*(MI*wm + i) + i16, unit 4*kappa + kb -> byte offset aoff[kappa] + 4096*i
  uint32_t aoff[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) aoff[k] = (uint32_t)((16 * MI * wm + i16) * 256 + swz(i16, 4 * k + kb) * 16);

  // Packed weights of one tile for this wavefront: one load of 4*b bytes per slab and lane, whatever the
  // width (equal load counts on the three paths keep the compiler's wait counts exact), plus NS
  // consecutive fp16 scales and zeros (rows 8*i16 + NS*wn + 0..NS-1 of the tile).
  constexpr int NG = G64 ? 2 : 1;  // parameter pairs per row and tile column
  struct SZ {
    uint32_t s[NG][NS / 2], z[NG][NS / 2];
  };
  auto issue_sz = [&](int tc, SZ& rsz) __attribute__((always_inline)) {
    const int64_t off = (int64_t)(G64 ? 2 * tc : tc >> p.gshift) * p.N + (int64_t)tr * 128 + 8 * i16 + NS * wn;
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int q = 0; q < NS / 2; ++q) {
        rsz.s[g][q] = reinterpret_cast<const uint32_t*>(p.scales + off + (int64_t)g * p.N)[q];
        rsz.z[g][q] = reinterpret_cast<const uint32_t*>(p.zeros + off + (int64_t)g * p.N)[q];
      }
  };
  // width known at compile time (the next tile belongs to the same run): no branch around the loads, so
  // they land in place and nothing waits for them before the next step
  auto issue_w_static = [&](auto btag, int e, u32x4 (&rw)[NS], SZ& rsz) __attribute__((always_inline)) {
    constexpr int B = decltype(btag)::value;
    const int32_t d = __builtin_amdgcn_readfirstlane(seq[e]);
    const uint8_t* stream = B == 2 ? p.s2 : B == 3 ? p.s3 : p.s4;
    const uint8_t* src = stream + (int64_t)(d >> 9) * (2048 * B) + (NS * wn) * (256 * B) + lane * (4 * B);
#pragma unroll
    for (int q = 0; q < NS; ++q) {
      if constexpr (B == 4) {
        rw[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + q * 1024));
      } else if constexpr (B == 3) {
        const uint32_t* s3 = reinterpret_cast<const uint32_t*>(src + q * 768);  // 4-byte aligned: three dwords, merged
        rw[q][0] = __builtin_nontemporal_load(s3);
        rw[q][1] = __builtin_nontemporal_load(s3 + 1);
        rw[q][2] = __builtin_nontemporal_load(s3 + 2);
      } else {
        const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src + q * 512));
        rw[q][0] = v[0];
        rw[q][1] = v[1];
      }
    }
    issue_sz(d & 511, rsz);
  };
  // width decided at run time (near the end of a run, where the tile two steps ahead has another width):
  // the same load sequence for every width, the words a narrower width does not have re-read its last
  // word.  No branch around the loads, so they land in place.
  auto issue_w_generic = [&](int e, u32x4 (&rw)[NS], SZ& rsz) __attribute__((always_inline)) {
    const int32_t d = __builtin_amdgcn_readfirstlane(seq[e]);
    const int bw = e < end2 ? 2 : e < end3 ? 3 : 4;
    const uint8_t* stream = bw == 2 ? p.s2 : bw == 3 ? p.s3 : p.s4;
    const uint8_t* src = stream + (int64_t)(d >> 9) * (2048 * bw) + (NS * wn) * (256 * bw) + lane * (4 * bw);
#pragma unroll
    for (int q = 0; q < NS; ++q) {
      const uint32_t* s = reinterpret_cast<const uint32_t*>(src + q * (256 * bw));
      const uint32_t v0 = __builtin_nontemporal_load(s), v1 = __builtin_nontemporal_load(s + 1),
                     v2 = __builtin_nontemporal_load(s + min(2, bw - 1)), v3 = __builtin_nontemporal_load(s + bw - 1);
      rw[q] = u32x4{v0, v1, v2, v3};
    }
    issue_sz(d & 511, rsz);
  };

  u32x4 fw[NS];  // landing registers of the next tile's packed words
#pragma unroll
  for (int q = 0; q < NS; ++q) fw[q] = u32x4{0u, 0u, 0u, 0u};
  SZ fsz;

  // ---- the software pipeline -------------------------------------------------------------------------
  // State between steps: w / s2 / z2 = packed words, scales, zeros of tile e; a0 / b0 = the MFMA operands
  // of its k-step 0; in flight: activation block e+1 (into the other LDS buffer) and the weights of tile
  // e+1 (into fw).  A step runs four groups; in each the MFMAs of one k-step are interleaved with the LDS
  // reads and the dequantisation of the next one (an MFMA occupies the matrix pipe for 16 cycles but the
  // issue port for 4).  Between the third and the fourth group sits the only synchronisation point: all
  // operand reads of block e have returned, block e+1 and tile e+1 have landed, a barrier, and the loads of
  // e+2 start; the fourth group then already prepares k-step 0 of tile e+1.
  u32x4 w[NS];
  half2_ s2[NG][NS], z2[NG][NS];
  half8 a0[MI], a1[MI], b0[NS], b1[NS];

  auto read_a = [&](int e, auto ktag, half8(&a)[MI]) __attribute__((always_inline)) {
    const unsigned char* base = Xs + (e & 1) * kBufBytes + aoff[decltype(ktag)::value];
#pragma unroll
    for (int i = 0; i < MI; ++i) a[i] = *reinterpret_cast<const half8*>(base + i * 4096);
  };
  auto make_b = [&](auto btag, auto ktag, half8(&b)[NS]) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      const uint32_t words[4] = {w[j][0], w[j][1], w[j][2], w[j][3]};
      constexpr int g = G64 ? decltype(ktag)::value / 2 : 0;  // k-steps 0-1 / 2-3 = columns 0-63 / 64-127
      b[j] = dequant_operand<decltype(btag)::value, decltype(ktag)::value>(words, s2[g][j], z2[g][j], magic);
    }
  };
  auto make_b_any = [&](int e, auto ktag, half8(&b)[NS]) __attribute__((always_inline)) {
    if (e < end2)
      make_b(std::integral_constant<int, 2>{}, ktag, b);
    else if (e < end3)
      make_b(std::integral_constant<int, 3>{}, ktag, b);
    else
      make_b(std::integral_constant<int, 4>{}, ktag, b);
  };
  auto mfmas = [&](const half8(&a)[MI], const half8(&b)[NS]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NS; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], b[j], acc[i][j], 0, 0, 0);
  };
  auto interleave = [&]() __attribute__((always_inline)) {
    if constexpr (IL > 0) {
#pragma unroll
      for (int g = 0; g < MI * NS; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
        __builtin_amdgcn_sched_group_barrier(0x002, IL, 0);  // VALU
      }
    }
  };
  // Synchronisation point.  Loads complete in issue order and X(e+1) was issued before W(e+1): the wait
  // the compiler puts in front of the moves out of the landing registers also covers the LDS-DMA loads of
  // block e+1.  No operand read may still be in the LDS queue when the barrier opens this step's buffer
  // for overwriting.
  auto sync_and_issue = [&](int e, auto in_run, auto btag) __attribute__((always_inline)) {
    SZ rsz;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      w[i] = fw[i];
      asm volatile("" : "+v"(w[i]));
    }
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int i = 0; i < NS / 2; ++i) {
        rsz.s[g][i] = fsz.s[g][i];
        rsz.z[g][i] = fsz.z[g][i];
        asm volatile("" : "+v"(rsz.s[g][i]), "+v"(rsz.z[g][i]));
      }
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int j = 0; j < NS; ++j) {
        union {
          uint32_t u;
          _Float16 h[2];
        } sv, zv;
        sv.u = rsz.s[g][j / 2];
        zv.u = rsz.z[g][j / 2];
        _Float16 sh = sv.h[j % 2], zh = zv.h[j % 2];
        if (p.bf16) {  // bfloat16 = top half of a float; the dequantisation runs in fp16
          sh = (_Float16)__uint_as_float((j % 2 ? sv.u >> 16 : sv.u & 0xFFFFu) << 16);
          zh = (_Float16)__uint_as_float((j % 2 ? zv.u >> 16 : zv.u & 0xFFFFu) << 16);
        }
        s2[g][j] = half2_{sh, sh};
        z2[g][j] = half2_{zh, zh};
      }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // past the end the last tile is loaded again, into the idle buffer and the landing registers: same
    // load count on every path
    const int nn = min(e + 2, e_last);
    issue_x(nn, e);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(in_run)::value)
      issue_w_static(btag, nn, fw, fsz);
    else
      issue_w_generic(nn, fw, fsz);
    __builtin_amdgcn_sched_barrier(0);
  };
  const std::integral_constant<int, 0> k0;
  const std::integral_constant<int, 1> k1;
  const std::integral_constant<int, 2> k2;
  const std::integral_constant<int, 3> k3;

  // in_run: tiles e+1 and e+2 have the same width B as tile e
  auto step = [&](auto btag, auto in_run, int e) __attribute__((always_inline)) {
    // Two workgroups share a CU.  A wavefront inside the three groups that only compute is served before one that is
    // at the synchronisation point or in the group right after it (whose loads have just been issued): the matrix
    // pipe waits less on the other workgroup's bookkeeping (2-4 % measured, same box).
    __builtin_amdgcn_s_setprio(1);
    mfmas(a0, b0);
    read_a(e, k1, a1);
    make_b(btag, k1, b1);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    mfmas(a1, b1);
    read_a(e, k2, a0);
    make_b(btag, k2, b0);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    mfmas(a0, b0);
    read_a(e, k3, a1);
    make_b(btag, k3, b1);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(0);
    sync_and_issue(e, in_run, btag);
    mfmas(a1, b1);
    read_a(e + 1, k0, a0);
    if constexpr (decltype(in_run)::value) {
      make_b(btag, k0, b0);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
    } else {
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      make_b_any(min(e + 1, e_last), k0, b0);
    }
  };

  // prologue: the first tile lands, then its k-step 0 is prepared while the second is on its way
  issue_x(e_first, e_first);
  __builtin_amdgcn_sched_barrier(0);
  issue_w_generic(e_first, fw, fsz);
  __builtin_amdgcn_sched_barrier(0);
  sync_and_issue(e_first - 1, std::integral_constant<bool, false>{}, k0);
  read_a(e_first, k0, a0);
  make_b_any(e_first, k0, b0);
  __builtin_amdgcn_sched_barrier(0);

  const std::integral_constant<bool, true> in_run;
  const std::integral_constant<bool, false> run_ends;
  const std::integral_constant<int, 2> b2;
  const std::integral_constant<int, 3> b3;
  const std::integral_constant<int, 4> b4;
  // the runs of this workgroup's share: [e_first, r2) 2-bit, [r2, r3) 3-bit, [r3, e_end) 4-bit
  const int r2 = min(max(end2, e_first), e_end), r3 = min(max(end3, e_first), e_end);
  int e = e_first;
  for (; e + 2 < r2; ++e) step(b2, in_run, e);
  for (; e < r2; ++e) step(b2, run_ends, e);
  for (; e + 2 < r3; ++e) step(b3, in_run, e);
  for (; e < r3; ++e) step(b3, run_ends, e);
  for (; e + 2 < e_end; ++e) step(b4, in_run, e);
  for (; e < e_end; ++e) step(b4, run_ends, e);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the idle loads of the last two steps

  // epilogue: the block goes through LDS (the activation buffers are free now) so that it leaves in whole
  // 256-byte row segments: acc[i][j][r] = C[16*MI*wm + 16i + 4kb + r][8*i16 + NS*wn + j], the NS values j of
  // a lane being consecutive columns.
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();  // every wavefront's idle loads have landed and its operand reads returned
  asm volatile("" ::: "memory");
  if (p.ksplit > 1) {
    // partial product in fp32: rows of 512 bytes through LDS (BM x 512 bytes = the two activation buffers)
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = 16 * MI * wm + 16 * i + 4 * kb + r;
        float* dst = reinterpret_cast<float*>(Xs + row * 512 + (8 * i16 + NS * wn) * 4);
#pragma unroll
        for (int j = 0; j < NS; ++j) dst[j] = acc[i][j][r];
      }
    __syncthreads();
    float* pbase = p.partial + ((int64_t)ks * p.M + m0) * p.N + (int64_t)tr * 128;
    const int prow = tid / 32, punit = tid % 32;
#pragma unroll
    for (int i = 0; i < BM / (S::kThreads / 32); ++i) {
      const int row = prow + (S::kThreads / 32) * i;
      const u32x4 v = *reinterpret_cast<const u32x4*>(Xs + row * 512 + punit * 16);
      if (m0 + row < p.M) *reinterpret_cast<u32x4*>(pbase + (int64_t)row * p.N + punit * 4) = v;
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = 16 * MI * wm + 16 * i + 4 * kb + r;
      union {
        _Float16 h[NS];
        uint32_t u[NS / 2];
      } o;
#pragma unroll
      for (int j = 0; j < NS; ++j) o.h[j] = (_Float16)acc[i][j][r];
      uint32_t* dst = reinterpret_cast<uint32_t*>(Xs + row * 256 + (8 * i16 + NS * wn) * 2);
#pragma unroll
      for (int q = 0; q < NS / 2; ++q) dst[q] = o.u[q];
    }
  __syncthreads();
  _Float16* ybase = p.Yt + (int64_t)m0 * p.N + (int64_t)tr * 128;
#pragma unroll
  for (int i = 0; i < S::kPasses; ++i) {
    const int row = xrow + S::kRowsPerPass * i;
    const u32x4 v = *reinterpret_cast<const u32x4*>(Xs + row * 256 + xunit * 16);
    if (m0 + row < p.M) *reinterpret_cast<u32x4*>(ybase + (int64_t)row * p.N + xunit * 8) = v;
  }
}

template <int BM, int WM, int WN, bool G64>
static void launch_prefill_shape(PrefillParams p, int M, hipStream_t stream) {
  p.n_mtiles = (M + BM - 1) / BM;
  const unsigned grid = (unsigned)p.n_mtiles * (unsigned)p.ntr * (unsigned)p.ksplit;
  hipLaunchKernelGGL((prefill_kernel<BM, WM, WN, 2, G64>), dim3(grid), dim3(64 * WM * WN), 0, stream, p);
}

PrefillPlan make_prefill_plan(int32_t N, int32_t K, int32_t M) {
  PrefillPlan d;
  const int64_t ntr = N / kTile, ntc = K / kTile;
  // 64-row blocks when 128-row blocks would leave half of the CUs without a workgroup (short prompts on narrow
  // matrices): twice the workgroups, each half as long; measured 8 to 13 % faster there, slower elsewhere
  d.bm = (int64_t)((M + 127) / 128) * ntr <= 128 ? 64 : 128;
  // Still at most one workgroup per CU: a workgroup walks its K/128 tiles one after the other (about 0.95 us
  // each) while most of the machine idles, so K is cut into ranges of at least 8 tiles, one workgroup each
  // (up to two workgroups per CU), fp32 partial products, and a reduction pass in a fixed order.
  const int64_t blocks = (int64_t)((M + d.bm - 1) / d.bm) * ntr;
  int64_t ks = 1;
  if (blocks <= 256) {
    ks = 512 / blocks;
    if (ks > ntc / 8) ks = ntc / 8;
    if (ks > 8) ks = 8;
    if (ks < 3 && ntc < 64) ks = 1;  // two ranges of a short K measured between -5 and +6 %; of a long K +20 %
  }
  d.ksplit = (int32_t)ks;
  d.xperm_bytes = round_up_256((int64_t)((M + kTile - 1) / kTile) * kTile * K * 2);  // whole 128-row blocks
  d.ytmp_bytes = round_up_256(ks > 1 ? ks * (int64_t)M * N * 4 : (int64_t)M * N * 2);
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
  // the staging / scatter passes hold one fp16 row in LDS (K <= 57344 fits)
  if (((a.row_perm || plan.ksplit > 1) && (int64_t)L->N * 2 > 160 * 1024) ||
      L->K / kTile > kPrefillMaxTiles)
    return SFMP_ERR_SHAPE;
  if (plan.ksplit > 1) {
    if (int e = allow_full_lds(reinterpret_cast<const void*>(&reduce_split_kernel), "hipFuncSetAttribute(reduce)")) return e;
  } else if (a.row_perm) {
    if (int e = allow_full_lds(reinterpret_cast<const void*>(&scatter_cols_kernel), "hipFuncSetAttribute(scatter)")) return e;
  }
  // activations -> workspace: column permutation applied (if any), 128x128 blocks each contiguous.  Rows per
  // workgroup: as many as fit in 128 KiB of LDS (8 at most), fewer while that would leave compute units without a
  // workgroup.
  _Float16* Xp = (_Float16*)a.workspace;
  {
    int R = L->K <= 8192 ? 8 : L->K <= 16384 ? 4 : L->K <= 32768 ? 2 : 1;
    while (R > 1 && (a.M + R - 1) / R < 256) R /= 2;
    const void* fn = R == 8   ? reinterpret_cast<const void*>(&gather_cols_kernel<8>)
                     : R == 4 ? reinterpret_cast<const void*>(&gather_cols_kernel<4>)
                     : R == 2 ? reinterpret_cast<const void*>(&gather_cols_kernel<2>)
                              : reinterpret_cast<const void*>(&gather_cols_kernel<1>);
    if (int e = allow_full_lds(fn, "hipFuncSetAttribute(gather)")) return e;
    const _Float16* Xa = (const _Float16*)a.X;
    const int32_t* cp = a.col_perm;
    int Ma = a.M, Ka = L->K;
    void* kargs[] = {&Xa, &cp, &Xp, &Ma, &Ka};
    hipError_t e = hipLaunchKernel(fn, dim3((unsigned)((a.M + R - 1) / R)), dim3(1024), kargs, (size_t)R * L->K * 2,
                                   (hipStream_t)stream);
    if (e != hipSuccess) {
      note_hip_error("sfmp_gemm activation staging launch", hipGetErrorString(e));
      return SFMP_ERR_HIP;
    }
    if (int e2 = check_launch("sfmp_gemm activation staging launch")) return e2;
  }
  _Float16* Yt = a.row_perm ? (_Float16*)((char*)a.workspace + plan.xperm_bytes) : (_Float16*)a.Y;
  PrefillParams p;
  p.Xp = Xp;
  p.s2 = a.s2;
  p.s3 = a.s3;
  p.s4 = a.s4;
  p.index = a.index;
  p.scales = (const _Float16*)a.scales;
  p.zeros = (const _Float16*)a.zeros;
  p.Yt = Yt;
  p.M = a.M;
  p.N = L->N;
  p.K = L->K;
  p.ntr = L->N / kTile;
  p.ntc = L->K / kTile;
  p.gshift = L->group == 512 ? 2 : L->group == 256 ? 1 : 0;
  p.bf16 = L->scale_format == SFMP_SCALE_BF16;
  p.n_mtiles = 0;
  p.ksplit = plan.ksplit;
  p.partial = plan.ksplit > 1 ? (float*)((char*)a.workspace + plan.xperm_bytes) : nullptr;
  const bool g64 = L->group == 64;
  if (plan.bm == 64) {
    if (g64)
      launch_prefill_shape<64, 1, 4, true>(p, a.M, (hipStream_t)stream);
    else
      launch_prefill_shape<64, 1, 4, false>(p, a.M, (hipStream_t)stream);
  } else {
    if (g64)
      launch_prefill_shape<128, 1, 4, true>(p, a.M, (hipStream_t)stream);
    else
      launch_prefill_shape<128, 1, 4, false>(p, a.M, (hipStream_t)stream);
  }
  if (int e = check_launch("sfmp_gemm prefill launch")) return e;
  if (plan.ksplit > 1) {
    hipLaunchKernelGGL(reduce_split_kernel, dim3((unsigned)a.M), dim3(1024), (size_t)L->N * 2, (hipStream_t)stream,
                       (const float*)p.partial, (int)plan.ksplit, (int)a.M, a.row_perm, (_Float16*)a.Y, (int)L->N);
    if (int e = check_launch("sfmp_gemm split-K reduction launch")) return e;
  } else if (a.row_perm) {
    hipLaunchKernelGGL(scatter_cols_kernel, dim3((unsigned)a.M), dim3(256), (size_t)L->N * 2, (hipStream_t)stream,
                       (const _Float16*)Yt, a.row_perm, (_Float16*)a.Y, (int)L->N);
    if (int e = check_launch("sfmp_gemm row scatter launch")) return e;
  }
  return SFMP_OK;
}

}  // namespace sfmp
