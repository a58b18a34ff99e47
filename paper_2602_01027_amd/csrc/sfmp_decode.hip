// Decode path (M <= 16): bandwidth-bound mixed-precision GEMV (M = 1) and skinny GEMM
// (2 <= M <= 16) for gfx950.
//
// Common arithmetic.  Codes are masked out of the packed words as fp16 denormals q*2^(p-24)
// and contracted against the fp16 activations by MFMA 16x16x32 (activations = A operand, 16
// rows of which at most M are non-zero; 16 weight rows = B operand).  The matrix pipe is the
// MAC engine of a memory-bound kernel: at HBM speed only 2-4 VALU lane-ops per weight are
// available and they are spent on the unpack (about 0.6 per weight); the MFMA cost is
// independent of M.  One accumulator per field position p; per 128-column group the result is
// scaled in fp32:  y += s * sum_p 2^(24-p) C_p + z * sum(x)      (Appendix B Eq. 11, re-associated).
//
// GEMV (M = 1): a workgroup owns whole 16-row slabs of tile rows over the WHOLE K range, so a
// result never leaves the workgroup: no global partial sums, no atomics, no fences.  The
// activation vector is copied to LDS and permuted there (the column permutation is fused into
// this load); wavefront w walks the tiles w, w+NW, ... of its slabs, each slab arriving in a
// two-slot ring by direct global->LDS copies; per-wavefront sums are combined through LDS and the
// outputs are scattered through row_perm.  Workgroups are numbered so that the 8 slabs of a
// tile row run on the same XCD (they share scale/zero cache lines and the index table).
//
// Skinny GEMM (2..16), and any M = 1 problem whose activation vector does not fit in LDS beside the
// rings: the same scheme with the activations of each tile column travelling through the ring slots,
// or resident in LDS when there are few of them (see rskinny_kernel).
#include <algorithm>
#include <cstddef>
#include <cstdlib>

#include "sfmp_device.h"
#include "sfmp_internal.h"

namespace sfmp {


// Sum over the slab's 128 columns of q * x for the 16 rows of the slab (lane%16) and the 16 activation rows
// (4*(lane/16) + r), in units of 2^-24 (class 0 counts 1, class i counts 2^-pos(i)): the caller multiplies by 2^24
// once per slab instead of once per item.
template <int B>
__device__ __forceinline__ floatx4 slab_dot_units(const uint32_t* w, const half8 (&a)[4]) {
  uint32_t op[4][4];
  unpack_slab<B>(w, op);
  floatx4 c[num_classes<B>()];
#pragma unroll
  for (int i = 0; i < num_classes<B>(); ++i) c[i] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa)
    c[step_class<B>(kappa)] =
        __builtin_amdgcn_mfma_f32_16x16x32_f16(a[kappa], as_half8(op[kappa]), c[step_class<B>(kappa)], 0, 0, 0);
  floatx4 t = c[0];
#pragma unroll
  for (int i = 1; i < num_classes<B>(); ++i) t += c[i] * pow2f(-class_pos<B>(i));
  return t;
}

// The same sum for activation row 0 only, in units of 2^-24: class 0 counts 1, class i counts 2^-pos(i); the
// caller multiplies by 2^24 once per slab instead of once per item.
template <int B>
__device__ __forceinline__ float slab_dot_row0_units(const uint32_t* w, const half8 (&a)[4]) {
  uint32_t op[4][4];
  unpack_slab<B>(w, op);
  floatx4 c[num_classes<B>()];
#pragma unroll
  for (int i = 0; i < num_classes<B>(); ++i) c[i] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa)
    c[step_class<B>(kappa)] =
        __builtin_amdgcn_mfma_f32_16x16x32_f16(a[kappa], as_half8(op[kappa]), c[step_class<B>(kappa)], 0, 0, 0);
  float t = c[0][0];
#pragma unroll
  for (int i = 1; i < num_classes<B>(); ++i) t += c[i][0] * pow2f(-class_pos<B>(i));
  return t;
}

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // m0 is named as clobbered on purpose
// The same for a group length of 64: the sums over columns 0-63 (k-steps 0, 1) and over columns 64-127 (k-steps 2, 3)
// of the slab apart, both in units of 2^-24: one accumulator per k-step, each weighted by 2^-(its field position).
template <int B>
__device__ __forceinline__ void slab_dot_row0_halves(const uint32_t* w, const half8 (&a)[4], float& t_lo, float& t_hi) {
  uint32_t op[4][4];
  unpack_slab<B>(w, op);
  floatx4 c[4];
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa)
    c[kappa] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[kappa], as_half8(op[kappa]), floatx4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
  t_lo = c[0][0] * pow2f(-step_pos<B>(0)) + c[1][0] * pow2f(-step_pos<B>(1));
  t_hi = c[2][0] * pow2f(-step_pos<B>(2)) + c[3][0] * pow2f(-step_pos<B>(3));
}
template <int B>
__device__ __forceinline__ void slab_dot_halves(const uint32_t* w, const half8 (&a)[4], floatx4& t_lo, floatx4& t_hi) {
  uint32_t op[4][4];
  unpack_slab<B>(w, op);
  floatx4 c[4];
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa)
    c[kappa] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[kappa], as_half8(op[kappa]), floatx4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
  t_lo = c[0] * pow2f(-step_pos<B>(0)) + c[1] * pow2f(-step_pos<B>(1));
  t_hi = c[2] * pow2f(-step_pos<B>(2)) + c[3] * pow2f(-step_pos<B>(3));
}

// Direct global->LDS copies written out by hand: scalar base address + 32-bit lane offset (no 64-bit vector
// address arithmetic per copy), lanes chosen by a mask in scalar registers.  Lane l writes 16 bytes at LDS byte
// lds_off + 16 l.  EXEC is restored inside the statement.  The compiler does not count these copies: the
// caller waits for them with s_waitcnt vmcnt, and no compiler-placed wait stands in front of later LDS stores.
__device__ __forceinline__ void lds_copy_b128(uint64_t sbase, uint32_t voff, uint32_t lds_off, uint64_t lanes) {
  uint64_t saved;
  asm volatile(
      "s_mov_b64 %0, exec\n\t"
      "s_mov_b64 exec, %4\n\t"
      "s_mov_b32 m0, %3\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %2, %1\n\t"
      "s_mov_b64 exec, %0"
      : "=&s"(saved)
      : "s"(sbase), "v"(voff), "s"(lds_off), "s"(lanes)
      : "memory", "m0");
}

// The two copies of a GEMV item in one statement: 32 parameter dwords (lanes 0-31, a full 64-bit address per lane) to
// LDS byte lds_off, then 16 bytes per lane of the slab (scalar base + lane offset; lanes 0-31 always, of lanes 32-63
// those whose bit is set in hi_lanes) to lds_off + slab_off.  Only the upper half of EXEC changes, and it is put back;
// the writes to EXEC sit between each write of M0 and the copy that uses it (the wait state M0 needs).
// (par_hi_lanes: 0, or all ones for a group length of 64, where lanes 32-63 bring the parameters of the tile column's
// second group)
__device__ __forceinline__ void lds_copy_item(uint64_t par_vaddr, uint64_t slab_sbase, uint32_t slab_voff,
                                              uint32_t lds_off, uint32_t lds_off_slab, uint32_t hi_lanes,
                                              uint32_t par_hi_lanes = 0) {
  uint32_t saved;
  asm volatile(
      "s_mov_b32 m0, %3\n\t"
      "s_mov_b32 %0, exec_hi\n\t"
      "s_mov_b32 exec_hi, %7\n\t"
      "global_load_lds_dword %1, off\n\t"
      "s_mov_b32 m0, %4\n\t"
      "s_mov_b32 exec_hi, %5\n\t"
      "global_load_lds_dwordx4 %6, %2\n\t"
      "s_mov_b32 exec_hi, %0"
      : "=&s"(saved)
      : "v"(par_vaddr), "s"(slab_sbase), "s"(lds_off), "s"(lds_off_slab), "s"(hi_lanes), "v"(slab_voff),
        "s"(par_hi_lanes)
      : "memory", "m0");
}
#pragma clang diagnostic pop

// ============================================================================================
// GEMV, M = 1
// ============================================================================================
struct GemvParams {
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
  int32_t N, K, ntr, ntc;
  // slabs of workgroup b of the problem's G workgroups: nj_q + (b < nj_r), with 8 ntr = nj_q G + nj_r (divided on the host)
  int32_t nj_q, nj_r;
  int32_t max_slabs;  // slabs per workgroup (upper bound), sizes the reduction buffer
  int32_t gshift;     // log2(group / 128): tile column tc uses parameter row tc >> gshift
  int32_t bf16;       // scales and zeros are bfloat16 (else fp16)
  int32_t g64;        // group length 64 (read by the host only: it selects the kernel instantiation)
};

constexpr int kGemvWaves = 16;       // wavefronts per workgroup; one workgroup per CU
constexpr int kGemvMaxGrid = 256;    // persistent grid: at most one workgroup per CU (two per CU, which the GEMV
                                     // kernels' 60 registers and LDS footprint allow on most shapes, measured 2-5 % slower)
// Ring slots per wavefront.  Two: one item being consumed, one on its way.  The 4096 wavefronts of a launch are
// what keeps the memory system busy; deeper rings (up to 8 were tried, all that LDS allows) were measured slower by
// up to 14 %: every wavefront then requests its whole share at once, the data comes back wavefront by wavefront,
// and the arithmetic of the wavefronts served last starts when the transfer is nearly over.
constexpr int kGemvMaxSlots = 2;
constexpr int kGemvMinSlots = 2;
constexpr int kGemvMaxSlabs = 16;    // slabs per workgroup kept in register accumulators
constexpr int kGemvMaxItems = 64;    // items per wavefront: one lane of the item registers each
constexpr int kSlotBytes = 1024 + 128;  // slab bytes (<= 1 KiB) + 16 scale dwords + 16 zero dwords
constexpr int kGemvSlotParamBytes = 128;  // GEMV slots: [16 scale dwords | 16 zero dwords | slab]
// group length 64: [16 scale + 16 zero dwords of columns 0-63 | the same of columns 64-127 | slab]
constexpr int kGemvSlotParamBytes64 = 256;
constexpr int kSlotBytes64 = 1024 + 256;

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// The scale and the zero of an item as floats.  Each sits in the low or the high half (shift = 0 or 16, the same
// for the whole wavefront) of its dword, as IEEE fp16 or as bfloat16 (= the top half of a float).  `bf16` is
// wave-uniform; the marker keeps the two formats on separate paths instead of computing both and selecting.
__device__ __forceinline__ void params_to_float(uint32_t scale_dword, uint32_t zero_dword, uint32_t shift, bool bf16,
                                                float& sf, float& zf) {
  const uint32_t sb = scale_dword >> shift, zb = zero_dword >> shift;
  if (bf16) {
    asm volatile("; bfloat16 parameters");
    sf = __uint_as_float(sb << 16);
    zf = __uint_as_float(zb << 16);
  } else {
    union {
      uint16_t u;
      _Float16 h;
    } a, b;
    a.u = (uint16_t)sb;
    b.u = (uint16_t)zb;
    sf = (float)a.h;
    zf = (float)b.h;
  }
}

// sum of the 8 halves of a 16-byte unit, then over the 16 lanes (= 128 columns = one tile column)
__device__ __forceinline__ float unit_group_sum(const half8& v) {
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) s += (float)v[e];
  // rotations inside each row of 16 lanes (data-parallel primitives of the vector ALU, no trip through LDS)
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), 0x128, 0xF, 0xF, false));  // row_ror:8
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), 0x124, 0xF, 0xF, false));  // row_ror:4
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), 0x122, 0xF, 0xF, false));  // row_ror:2
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), 0x121, 0xF, 0xF, false));  // row_ror:1
  return s;
}


// the same over 8 lanes (= 64 columns = half a tile column): mirror inside each half row, then inside each quad
__device__ __forceinline__ float unit_half_group_sum(const half8& v) {
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) s += (float)v[e];
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), 0x141, 0xF, 0xF, false));  // row_half_mirror
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  return s;
}

// LDS stores the compiler does not see as LDS accesses.  After a direct global->LDS copy has been issued the
// compiler puts a wait for ALL outstanding copies in front of every ordinary LDS store (it cannot tell the
// destinations apart); these stores are used while ring copies are in flight, to regions no copy writes.
// The caller waits with s_waitcnt lgkmcnt(0) before anyone reads what was stored.
__device__ __forceinline__ void lds_store_b128_untracked(void* dst, const half8& v) {
  const uint32_t off = (uint32_t)(uintptr_t)(lptr_t)dst;
  asm volatile("ds_write_b128 %0, %1" ::"v"(off), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_store_b32_untracked(void* dst, float v) {
  const uint32_t off = (uint32_t)(uintptr_t)(lptr_t)dst;
  asm volatile("ds_write_b32 %0, %1" ::"v"(off), "v"(v) : "memory");
}
// workgroup barrier that waits for this wavefront's LDS traffic only, not for its outstanding global->LDS copies
__device__ __forceinline__ void barrier_lds_only() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

constexpr int kGemvUnitIters = 4;  // 16-byte activation units per thread: K <= 8 * 4 * 1024 = 32768

// bytes of the region shared by the raw activation copy (start of the kernel) and the reduction buffer (end)
__host__ __device__ inline int64_t gemv_shared_region_bytes(int32_t K, int32_t max_slabs, int nw) {
  const int64_t raw = (int64_t)K * 2, red = (int64_t)max_slabs * nw * 64;
  return ((raw > red ? raw : red) + 15) & ~(int64_t)15;
}

// NW wavefronts per workgroup, S ring slots per wavefront.
//
// A wavefront's work is a list of at most 64 "items" (one 16-row slab of one tile each).  Everything
// an item needs (offset of its slab in its stream, offset of its parameters, tile column, flags) is computed
// once, by lane e for item e, and later broadcast with v_readlane; the addresses of the copies are scalar.
// The ring is refilled item by item, so S-1 items per wavefront are always in flight.
//
// Order of the start: a launch of this size lasts about 10 us, of which each dependent trip to memory is most of
// a microsecond, so everything that depends on the arguments alone (tile descriptors, raw activations, column
// permutation, the output positions of the end) is requested at once; the ring is filled as soon as the
// descriptors are there, and the activations are permuted inside LDS while the first slabs are on their way.
// G64: group length 64 - two (scale, zero) pairs per row and tile column, the activation sums per half tile column.
template <int NW, int S, bool PRELOADED, bool ANYFMT, bool G64 = false>
__device__ __forceinline__ void gemv_body(const GemvParams& p_in, const int bid, const int G, unsigned char* lds_raw) {
  constexpr int NT = NW * 64;
  constexpr int kPar = G64 ? kGemvSlotParamBytes64 : kGemvSlotParamBytes;  // parameter bytes in front of the slab
  constexpr int kSlot = 1024 + kPar;
  // PRELOADED (the plain kernel): the integers and the four pointers of the first requests are in scalar registers
  // when the kernel starts; the other pointers are fetched behind those requests, see below.
  // Otherwise (a problem of a batch, whose arguments lie in the argument block): all arguments are fetched now, by
  // scalar loads issued together: fetched where they are first used they arrive in two to four dependent trips to
  // memory (the block spans two cache lines), of which a launch this short has no microsecond to spare.  The integers
  // pass through the statement as outputs, so nothing computed from them can be placed in front of it.
  GemvParams p = p_in;
  if constexpr (!PRELOADED)
    asm volatile(""
                 : "+s"(p.N), "+s"(p.K), "+s"(p.ntr), "+s"(p.ntc), "+s"(p.nj_q), "+s"(p.nj_r), "+s"(p.max_slabs), "+s"(p.gshift),
                   "+s"(p.bf16)
                 : "s"(p.X), "s"(p.col_perm), "s"(p.s2), "s"(p.s3), "s"(p.s4), "s"(p.tile_desc), "s"(p.scales),
                   "s"(p.zeros), "s"(p.row_perm), "s"(p.Y));
  // LDS: Xs [K] fp16 | Sx [2 ntc] f32 (one sum per tile column, or two per tile column at group length 64) |
  //      shared region: raw activations, later red [max_slabs][NW][16] f32 | rings [NW][S][slot bytes]
  _Float16* Xs = reinterpret_cast<_Float16*>(lds_raw);
  float* Sx = reinterpret_cast<float*>(lds_raw + (size_t)p.K * 2);
  unsigned char* shared_region = lds_raw + (((size_t)p.K * 2 + (size_t)p.ntc * 8 + 15) & ~(size_t)15);
  _Float16* Xraw = reinterpret_cast<_Float16*>(shared_region);
  float* red = reinterpret_cast<float*>(shared_region);
  unsigned char* rings = shared_region + gemv_shared_region_bytes(p.K, p.max_slabs, NW);

  // (index arithmetic below is unsigned and free of integer division: these instructions stand between the start of
  // a wavefront and its first load, four wavefronts deep on every SIMD)
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid % kWave;
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / kWave));
  const uint32_t ubid = (uint32_t)bid, uG = (uint32_t)G, untr = (uint32_t)p.ntr, untc = (uint32_t)p.ntc;
  // Virtual slab index v = bid + G*j (G is a multiple of 8, block b runs on XCD b%8): XCD x gets
  // the contiguous slab range [x*ntr, (x+1)*ntr), so the 8 slabs of a tile row run on one XCD.
  const int nj = p.nj_q + (bid < p.nj_r ? 1 : 0);                        // slabs of this workgroup
  const int my_cnt = untc > wave ? (int)((untc - wave + NW - 1) / NW) : 0;  // tiles per slab of this wavefront
  const int E = nj * my_cnt;                                             // items of this wavefront (<= 64)

  // ---- requests that depend on the arguments alone, all issued before the first wait
  // (1) tile descriptor of item `lane`: item e = j*my_cnt + i is tile column wave + NW*i of slab j
  // (j = lane / my_cnt through a float reciprocal: exact, since lane + 0.5 is at least 0.5 / 64 away from a multiple
  // of my_cnt <= 64 and the reciprocal is good to 2^-22)
  const uint32_t it_j = (uint32_t)(((float)lane + 0.5f) * __builtin_amdgcn_rcpf((float)(my_cnt > 0 ? my_cnt : 1)));
  const uint32_t it_i = lane - it_j * (uint32_t)my_cnt;
  const uint32_t it_v = ubid + uG * it_j;
  const uint32_t it_slab = (it_v % 8) * untr + it_v / 8;
  const uint32_t it_tr = it_slab / 8, it_sigma = it_slab % 8;
  const uint32_t it_tc = wave + NW * it_i;
  // (every load below is unconditional, from a clamped and always valid address: a load under a condition makes
  // the compiler wait for it at the end of the condition, and the requests would go out one after the other)
  const int32_t d = p.tile_desc[(int)lane < E ? it_tr * untc + it_tc : 0u];
  // (2) where the sum that thread tid adds up at the end goes: output row 8*r16 + sigma of slab tid/16
  uint32_t out_row = 0;
  if (tid < (uint32_t)nj * 16) {
    const uint32_t v = ubid + uG * (tid / 16);
    const uint32_t slab = (v % 8) * untr + v / 8;
    out_row = (slab / 8) * kTile + 8 * (tid % 16) + (slab % 8);
  }
  int32_t out_col = *(p.row_perm ? p.row_perm + out_row : p.tile_desc);
  // (3) activations: raw copy straight into LDS (into their final place when there is no permutation);
  //     column permutation into registers (entries of the last unit for threads beyond the end)
  const int units = p.K / 8;
  int4 c0[kGemvUnitIters], c1[kGemvUnitIters];
  {
    _Float16* xdst = p.col_perm ? Xraw : Xs;
    const int4* cp = reinterpret_cast<const int4*>(p.col_perm ? (const void*)p.col_perm : (const void*)p.X);
#pragma unroll
    for (int u = 0; u < kGemvUnitIters; ++u) {
      if (u * NT < units) {  // uniform
        const int i = tid + u * NT;
        if (i < units)
          __builtin_amdgcn_global_load_lds((gptr_t)(p.X + 8 * (size_t)i),
                                           (lptr_t)(xdst + 8 * (size_t)(wave * 64 + u * NT)), 16, 0, 0);
        const int ic = p.col_perm ? min(i, units - 1) : 0;
        c0[u] = cp[2 * ic];
        c1[u] = cp[2 * ic + 1];
      }
    }
  }
  if constexpr (PRELOADED)  // the remaining arguments travel together with the requests above
    asm volatile("" : "+s"(p.N) : "s"(p.s2), "s"(p.s3), "s"(p.s4), "s"(p.scales), "s"(p.zeros), "s"(p.Y));
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // one trip to memory for all of the above
  // (the loaded registers are "used" here so that the compiler places its own wait for them here as well: placed
  // after the ring has been filled it would have to be a wait for every ring copy)
#pragma unroll
  for (int u = 0; u < kGemvUnitIters; ++u)
    if (u * NT < units)
      asm volatile("" : "+v"(c0[u].x), "+v"(c0[u].y), "+v"(c0[u].z), "+v"(c0[u].w), "+v"(c1[u].x), "+v"(c1[u].y),
                   "+v"(c1[u].z), "+v"(c1[u].w));
  asm volatile("" : "+v"(out_col));

  // ---- per-item registers of lane e: address of the slab, upper half of the lane mask of its copy, 32-bit offset of
  // the parameter dwords inside the scale / zero arrays (each stream and array is below 4 GiB), and the item's flags
  uint32_t it_wlo = 0, it_whi = 0, it_xhi = 0, it_soff = 0, it_misc = 0;
  {
    const uint32_t bm2 = (uint32_t)d & 3u;  // bit-width - 2 (the use of d makes the compiler wait for the loads above, here)
    const uint32_t slab_bytes = 256u * (bm2 + 2u);
    if (lane < E) {
      // address of the slab (the choice of the stream is made here, once, by the lane that describes the item) and
      // the upper half of the lane mask of its copy: 32, 48 or 64 lanes of 16 bytes
      const uint64_t waddr = (uint64_t)(bm2 == 0 ? p.s2 : bm2 == 1 ? p.s3 : p.s4) +
                             (((uint32_t)d >> 2) * (8u * slab_bytes) + (uint32_t)it_sigma * slab_bytes);
      it_wlo = (uint32_t)waddr, it_whi = (uint32_t)(waddr >> 32);
      it_xhi = bm2 == 0 ? 0u : bm2 == 1 ? 0xFFFFu : 0xFFFFFFFFu;
      // the aligned dword holding the fp16 scale of row 128*tr + sigma (rows 8*l + sigma are 16 bytes apart);
      // direct-to-LDS copies need dword-aligned addresses, the wanted fp16 is the low half for even sigma and
      // the high half for odd sigma
      it_soff = 2u * (uint32_t)((G64 ? 2u * it_tc : it_tc >> p.gshift) * p.N + it_tr * kTile + (it_sigma & ~1));
      it_misc = (uint32_t)it_tc | ((it_i == my_cnt - 1) ? 0x10000u : 0u) | ((uint32_t)it_j << 17) | (bm2 << 24) |
                ((uint32_t)(it_sigma & 1) << 26);
    }
  }
  // per-lane offsets of the copies of an item (bytes from the item's scalar base address)
  const uint32_t data_voff = lane * 16;
  // parameters: lanes 0-15 read the scale dwords, lanes 16-31 the zero dwords, in one copy (the two arrays may lie
  // anywhere, hence a 64-bit lane part: array base + 16 bytes per row pair, to which the item's offset is added);
  // at group length 64 lanes 32-63 read the same of the next parameter row (columns 64-127 of the tile column)
  const uint64_t par_vbase = ((lane & 16) == 0 ? (uint64_t)p.scales : (uint64_t)p.zeros) + (uint64_t)((lane & 15) * 16) +
                             (G64 && lane >= 32 ? (uint64_t)p.N * 2 : (uint64_t)0);

  // Issue item e into ring slot s: two direct global->LDS copies, the 16 scale dwords + 16 zero dwords (lanes
  // 0-15 / 16-31) and the slab (16 B per lane, 32/48/64 lanes, scalar address).
  const uint32_t ring_off = (uint32_t)(uintptr_t)(lptr_t)(rings + (size_t)wave * S * kSlot);
  auto issue_item = [&](int e, uint32_t slot) __attribute__((always_inline)) {
    const uint32_t wlo = (uint32_t)__builtin_amdgcn_readlane((int)it_wlo, e);
    const uint32_t whi = (uint32_t)__builtin_amdgcn_readlane((int)it_whi, e);
    const uint32_t xhi = (uint32_t)__builtin_amdgcn_readlane((int)it_xhi, e);
    const uint32_t soff = (uint32_t)__builtin_amdgcn_readlane((int)it_soff, e);
    lds_copy_item(par_vbase + soff, ((uint64_t)whi << 32) | wlo, data_voff, slot, slot + kPar, xhi, G64 ? ~0u : 0u);
  };
  constexpr int kCopiesPerItem = 2;

  // ---- prologue: fill the ring.  The first kEarly items of every wavefront go out now and start the stream;
  // the rest of the ring follows after the activations are in place: filling a whole ring takes about a
  // microsecond (the copies of 16 wavefronts queue up in one address unit), and the permutation would wait for it
  constexpr int kEarly = 2;
  const int npro = min(S, E);
  for (int e = 0; e < min(kEarly, npro); ++e) issue_item(e, ring_off + (uint32_t)e * kSlot);

  // ---- while those copies are on their way: permute the activations inside LDS and add up each tile column
  barrier_lds_only();  // every wavefront's part of the raw copy has landed (each waited for its own above)
#pragma unroll
  for (int u = 0; u < kGemvUnitIters; ++u) {
    const int i = tid + u * NT;
    if (i < units) {
      half8 v;
      if (p.col_perm) {
        v[0] = Xraw[c0[u].x];
        v[1] = Xraw[c0[u].y];
        v[2] = Xraw[c0[u].z];
        v[3] = Xraw[c0[u].w];
        v[4] = Xraw[c1[u].x];
        v[5] = Xraw[c1[u].y];
        v[6] = Xraw[c1[u].z];
        v[7] = Xraw[c1[u].w];
        lds_store_b128_untracked(Xs + 8 * i, v);
      } else {
        v = *reinterpret_cast<const half8*>(Xs + 8 * i);
      }
      if constexpr (G64) {
        const float s = unit_half_group_sum(v);
        if ((lane & 7) == 0) lds_store_b32_untracked(Sx + i / 8, s);
      } else {
        const float s = unit_group_sum(v);
        if ((lane & 15) == 0) lds_store_b32_untracked(Sx + i / 16, s);
      }
    }
  }
  barrier_lds_only();  // Xs and Sx are complete
  for (int e = kEarly; e < npro; ++e) issue_item(e, ring_off + (uint32_t)e * kSlot);

  half8 a[4];
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa) a[kappa] = half8{0, 0, 0, 0, 0, 0, 0, 0};
  // One fp32 sum per slab of this workgroup and wavefront (16 output features: lanes 0-15), written into the
  // reduction buffer as the slab finishes: red [slab][wavefront][16].  (The buffer shares its LDS with the raw copy of
  // the activations, which nobody reads after the barrier above.  Held in a 16-element register vector instead, the
  // sums cost 16 registers and an indexed register move per slab: 1.5 % of a layer, 4 % of the small launches.)
  float* red_mine = red + wave * 16 + lane;
  // running sums of the current slab: scale * (code sum, in units of 2^-24) and zero * (activation sum)
  float acc_q = 0.f, acc_z = 0.f;

  // Vector instructions per item are kept few (going from 48 to 38 of them gave 3-5 % per launch; from here on they
  // matter little: with the unpack, a third of them, left out the large launches are 1.5-4 % faster): everything that
  // can be is kept off the vector ALU:
  // addresses are scalar plus a loop-invariant lane offset, the tile-column sums sit in one register (lane i:
  // this wavefront's i-th tile column) and reach a scalar register by v_readlane, the two parameters are
  // brought together by one byte permute and widened inside the fused multiply-adds.
  float sx_lane = 0.f, sx_hi_lane = 0.f;  // (group length 64: the sums of columns 0-63 and 64-127)
  if (lane < my_cnt) {
    if constexpr (G64) {
      sx_lane = Sx[2 * (wave + NW * lane)];
      sx_hi_lane = Sx[2 * (wave + NW * lane) + 1];
    } else {
      sx_lane = Sx[wave + NW * lane];
    }
  }
  uint32_t lane_w2 = kPar + lane * 8, lane_w3 = kPar + lane * 12, lane_w4 = kPar + lane * 16, lane_p = (lane & 15) * 4;
  asm volatile("" : "+v"(lane_w2), "+v"(lane_w3), "+v"(lane_w4), "+v"(lane_p), "+v"(sx_lane), "+v"(sx_hi_lane));
  const unsigned char* lds0 = lds_raw - (uint32_t)(uintptr_t)(lptr_t)lds_raw;  // LDS byte 0

  auto consume = [&](int e, uint32_t slot) __attribute__((always_inline)) {
    const uint32_t misc = (uint32_t)__builtin_amdgcn_readlane((int)it_misc, e);
    const int tc = misc & 0xFFFF;
    if ((lane & 15) == 0) {  // only activation row 0 exists: lanes 0,16,32,48 feed it
#pragma unroll
      for (int kappa = 0; kappa < 4; ++kappa)
        a[kappa] = *reinterpret_cast<const half8*>(Xs + tc * kTile + 32 * kappa + 8 * (lane / 16));
    }
    const float sx = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sx_lane), tc / NW));
    const uint32_t scw = *reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_p));
    const uint32_t zrw = *reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_p) + 64);
    // low half: scale, high half: zero (bit 26 of misc: odd sigma -> the high halves of the two dwords)
    const uint32_t sel = (misc & (1u << 26)) ? 0x07060302u : 0x05040100u;
    uint32_t w[4];
    const uint32_t* src;
    if constexpr (G64) {
      const float sx_hi =
          __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sx_hi_lane), tc / NW));
      const uint32_t scw_hi = *reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_p) + 128);
      const uint32_t zrw_hi = *reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_p) + 192);
      float t_lo, t_hi;
      if (misc & (2u << 24)) {
        src = reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_w4));
        w[0] = src[0], w[1] = src[1], w[2] = src[2], w[3] = src[3];
        slab_dot_row0_halves<4>(w, a, t_lo, t_hi);
      } else if (misc & (1u << 24)) {
        src = reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_w3));
        w[0] = src[0], w[1] = src[1], w[2] = src[2];
        slab_dot_row0_halves<3>(w, a, t_lo, t_hi);
      } else {
        src = reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_w2));
        w[0] = src[0], w[1] = src[1];
        slab_dot_row0_halves<2>(w, a, t_lo, t_hi);
      }
      const uint32_t sz_lo = __builtin_amdgcn_perm(zrw, scw, sel), sz_hi = __builtin_amdgcn_perm(zrw_hi, scw_hi, sel);
      float s_lo, z_lo, s_hi, z_hi;
      params_to_float(sz_lo, sz_lo >> 16, 0, ANYFMT && p.bf16, s_lo, z_lo);
      params_to_float(sz_hi, sz_hi >> 16, 0, ANYFMT && p.bf16, s_hi, z_hi);
      acc_q += s_lo * t_lo + s_hi * t_hi;
      acc_z += z_lo * sx + z_hi * sx_hi;
      if (misc & 0x10000u) {  // this wavefront's share of slab j is complete
        asm volatile("" ::: "memory");
        if (lane < 16) red_mine[((misc >> 17) & 15) * (NW * 16)] = acc_q * 16777216.f + acc_z;
        acc_q = 0.f, acc_z = 0.f;
      }
      return;
    }
    float t;
    if (misc & (2u << 24)) {
      src = reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_w4));
      w[0] = src[0], w[1] = src[1], w[2] = src[2], w[3] = src[3];
      t = slab_dot_row0_units<4>(w, a);
    } else if (misc & (1u << 24)) {
      src = reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_w3));
      w[0] = src[0], w[1] = src[1], w[2] = src[2];
      t = slab_dot_row0_units<3>(w, a);
    } else {
      src = reinterpret_cast<const uint32_t*>(lds0 + (slot + lane_w2));
      w[0] = src[0], w[1] = src[1];
      t = slab_dot_row0_units<2>(w, a);
    }
    const uint32_t sz = __builtin_amdgcn_perm(zrw, scw, sel);
    // (ANYFMT: the storage type of the parameters is looked up per item; the kernels for fp16 alone have no such
    // branch in the loop, which also spares the register copies where its two sides meet)
    if (ANYFMT && p.bf16) {
      asm volatile("; bfloat16 parameters");
      acc_q += __uint_as_float(sz << 16) * t;
      acc_z += __uint_as_float(sz & 0xFFFF0000u) * sx;
    } else {
      // fp32 multiply-adds that read their first factor as fp16 from the low / high half of sz
      asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "+v"(acc_q) : "v"(sz), "v"(t));
      asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(acc_z) : "v"(sz), "s"(sx));
    }
    if (misc & 0x10000u) {  // this wavefront's share of slab j is complete
      asm volatile("" ::: "memory");  // keeps this a branch: as a select it copied all 16 sums after every item
      if (lane < 16) red_mine[((misc >> 17) & 15) * (NW * 16)] = acc_q * 16777216.f + acc_z;
      acc_q = 0.f, acc_z = 0.f;
    }
  };

  // ---- steady state: item e has landed once at most the S-1 younger items (2 copies each) are
  // outstanding; consume it and refill its slot with item e + S
  // (the LDS address of the current slot is carried along: with two slots the next one is a subtraction away)
  uint32_t slot = ring_off;
  auto next_slot = [&]() __attribute__((always_inline)) {
    if constexpr (S == 2) {
      slot = (2u * ring_off + kSlot) - slot;
    } else {
      slot += kSlot;
      if (slot == ring_off + S * kSlot) slot = ring_off;
    }
  };
  int e = 0;
  for (; e + S < E; ++e) {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerItem * (S - 1)) : "memory");
    // a wavefront whose item has landed is served before one that is issuing copies or about to wait (2-3 %)
    __builtin_amdgcn_s_setprio(1);
    consume(e, slot);
    __builtin_amdgcn_s_setprio(0);
    issue_item(e + S, slot);
    next_slot();
  }
  // ---- tail: nothing left to issue; item e has landed once at most the E-1-e younger items are outstanding
  // (most launches of a decoder layer have no more than S items per wavefront and are all tail: waiting for
  // everything first would put the whole arithmetic behind the whole transfer)
  for (; e < E; ++e) {
    switch (E - 1 - e) {
      case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
      case 1: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerItem * 1) : "memory"); break;
      case 2: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerItem * 2) : "memory"); break;
      case 3: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerItem * 3) : "memory"); break;
      case 4: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerItem * 4) : "memory"); break;
      case 5: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerItem * 5) : "memory"); break;
      case 6: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerItem * 6) : "memory"); break;
      default: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerItem * 7) : "memory"); break;
    }
    __builtin_amdgcn_s_setprio(1);
    consume(e, slot);
    __builtin_amdgcn_s_setprio(0);
    next_slot();
  }
  static_assert(S <= 8 && kCopiesPerItem * 7 < 64, "the tail's waits cover up to 7 younger items");

  if (my_cnt == 0 && lane < 16)  // a wavefront without a tile column has written no sums: zeros
    for (int q = 0; q < nj; ++q) red_mine[q * (NW * 16)] = 0.f;
  __syncthreads();
  if (tid < nj * 16) {  // nj <= 16: one sum per thread at most
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += red[((tid / 16) * NW + w) * 16 + tid % 16];
    p.Y[p.row_perm ? (int64_t)out_col : out_row] = (_Float16)sum;
  }
}

// The arguments are scalars rather than one struct: built with -mllvm -amdgpu-kernarg-preload-count=16, the first
// 14 dwords of scalar arguments (the four pointers of the first requests and the integers that address them) are
// placed in scalar registers by the command processor before the first wavefront starts, so the kernel's first global
// requests wait for no argument load; the rest of the arguments travel while those requests are in flight.
template <int NW, int S, bool ANYFMT, bool G64 = false>
__global__ __launch_bounds__(NW * 64) void gemv_kernel(
    const int32_t* tile_desc, const _Float16* X, const int32_t* col_perm, const int32_t* row_perm, int32_t nj_q,
    int32_t nj_r, int32_t ntr, int32_t ntc, int32_t K, int32_t grid, int32_t N, int32_t max_slabs, int32_t gshift,
    int32_t bf16, const uint8_t* s2, const uint8_t* s3, const uint8_t* s4, const _Float16* scales, const _Float16* zeros,
    _Float16* Y) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  GemvParams p;
  p.X = X, p.col_perm = col_perm, p.s2 = s2, p.s3 = s3, p.s4 = s4, p.tile_desc = tile_desc, p.scales = scales;
  p.zeros = zeros, p.row_perm = row_perm, p.Y = Y, p.N = N, p.K = K, p.ntr = ntr, p.ntc = ntc, p.nj_q = nj_q, p.nj_r = nj_r;
  p.max_slabs = max_slabs, p.gshift = gshift, p.bf16 = bf16;
  gemv_body<NW, S, true, ANYFMT, G64>(p, (int)blockIdx.x, grid, lds_raw);  // (gridDim.x would be one more load at entry)
}

// Several independent M = 1 problems in one launch (for example q, k and v, or gate and up of a
// decoder layer): the persistent grid is split between the problems in proportion to their bytes;
// workgroups [first[i], first[i+1]) run problem i exactly as a launch of that size would.
constexpr int kGemvMaxBatch = 8;
struct GemvBatchProblems {
  GemvParams p[kGemvMaxBatch];
};
// host-side description of a batch: first[i] = first workgroup of problem i; entries from `count` on hold the total
struct GemvBatch {
  int32_t first[kGemvMaxBatch + 1];
  int32_t count;
  GemvBatchProblems probs;
};

// index of the problem that workgroup `bid` belongs to: the number of problems whose first workgroup is <= bid, minus one
__device__ __forceinline__ int batch_problem_of(const int32_t (&first)[kGemvMaxBatch + 1], int bid) {
  int i = 0;
#pragma unroll
  for (int k = 1; k < kGemvMaxBatch; ++k) i += bid >= first[k] ? 1 : 0;
  return i;
}

// (first[1..8] arrive as scalar arguments, hence in preloaded scalar registers: a workgroup finds its problem, and
// its range of workgroups, without a load and without a loop of dependent ones, then fetches that problem's arguments
// in one go)
template <int NW, int S, bool ANYFMT, bool G64 = false>
__global__ __launch_bounds__(NW * 64) void gemv_batched_kernel(int32_t f1, int32_t f2, int32_t f3, int32_t f4,
                                                               int32_t f5, int32_t f6, int32_t f7, int32_t f8,
                                                               const GemvBatchProblems b) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int bid = (int)blockIdx.x;
  const int32_t f[kGemvMaxBatch + 1] = {0, f1, f2, f3, f4, f5, f6, f7, f8};
  int i = 0, lo = 0, hi = f8;
#pragma unroll
  for (int k = kGemvMaxBatch - 1; k >= 1; --k) {
    const bool at_or_after = bid >= f[k];
    i += at_or_after ? 1 : 0;
    lo = at_or_after && f[k] > lo ? f[k] : lo;
    hi = at_or_after ? hi : f[k];
  }
  const GemvParams p = b.p[i];
  gemv_body<NW, S, false, ANYFMT, G64>(p, bid - lo, hi - lo, lds_raw);
}

// ============================================================================================
// skinny GEMM through the rings, 2 <= M <= 16
// ============================================================================================
// The GEMV scheme carried over to a few activation rows: a workgroup owns whole 16-row slabs over the
// whole K range (no partial sums leave it), its wavefronts walk the tile columns, and everything an
// item needs arrives in a ring slot by direct global->LDS copies.  With M rows the activation vector no
// longer fits in LDS beside the rings, so the activations of an item's tile column (MB rows x 128
// columns, MB = 4, 8 or 16 >= M) travel through the ring slot as well; a small pass before the GEMM
// writes them into the workspace per tile column, column permutation applied, rows >= M zero, 16-byte
// units of row m stored at position u ^ m (conflict-free MFMA operand reads).  These copies hit in L2.
// The group sums of the activations come from one more MFMA against a vector of ones.
struct RSkinnyParams {
  const unsigned char* xblk;  // staged activations [ntc][MB][256 bytes], swizzled (not used by the resident variant)
  const _Float16* X;          // resident variant: the caller's activations [M, K] ...
  const int32_t* col_perm;    // ... and column permutation (or NULL); staged into LDS by every workgroup
  const uint8_t* s2;
  const uint8_t* s3;
  const uint8_t* s4;
  const int32_t* tile_desc;
  const _Float16* scales;
  const _Float16* zeros;
  const int32_t* row_perm;
  _Float16* Y;
  int32_t M, N, K, ntr, ntc, max_slabs;
  int32_t nj_q, nj_r;  // as in GemvParams: slabs of workgroup b = nj_q + (b < nj_r)
  int32_t gshift, bf16;  // as in GemvParams
  int32_t g64;           // group length 64 (read by the host only: it selects the kernel instantiation)
};

// one workgroup per tile column; thread (m, u) gathers the 8 columns of unit u' = u ^ m of row m
template <int MB>
__device__ __forceinline__ void stage_rows_tile(const _Float16* __restrict__ X, const int32_t* __restrict__ col_perm,
                                                unsigned char* xblk, int M, int K, int tc) {
  const int m = threadIdx.x / 16, pos = threadIdx.x % 16;
  const int unit = pos ^ m;
  half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
  if (m < M) {
    const int k0 = tc * kTile + unit * 8;
    if (col_perm) {
      const int4 c0 = reinterpret_cast<const int4*>(col_perm + k0)[0];
      const int4 c1 = reinterpret_cast<const int4*>(col_perm + k0)[1];
      const _Float16* row = X + (int64_t)m * K;
      v[0] = row[c0.x];
      v[1] = row[c0.y];
      v[2] = row[c0.z];
      v[3] = row[c0.w];
      v[4] = row[c1.x];
      v[5] = row[c1.y];
      v[6] = row[c1.z];
      v[7] = row[c1.w];
    } else {
      v = *reinterpret_cast<const half8*>(X + (int64_t)m * K + k0);
    }
  }
  *reinterpret_cast<half8*>(xblk + ((int64_t)tc * MB + m) * 256 + pos * 16) = v;
}

template <int MB>
__global__ __launch_bounds__(MB * 16) void stage_rows_kernel(const _Float16* __restrict__ X,
                                                            const int32_t* __restrict__ col_perm, unsigned char* xblk,
                                                            int M, int K) {
  stage_rows_tile<MB>(X, col_perm, xblk, M, K, (int)blockIdx.x);
}

// The same in operand order, for the kernels that keep their activations in registers: always 16 rows (rows >= M
// zero), 4 KiB per tile column laid out as [k-step][lane][16 bytes], lane = 16 * (unit % 4) + row: a wavefront loads the
// matrix-instruction operand of a k-step with one 16-byte load per lane, 1 KiB contiguous.
__device__ __forceinline__ void stage_rows_tile_operand_order(const _Float16* __restrict__ X,
                                                              const int32_t* __restrict__ col_perm, unsigned char* xblk,
                                                              int M, int K, int tc) {
  const int m = threadIdx.x / 16, unit = threadIdx.x % 16;
  half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
  if (m < M) {
    const int k0 = tc * kTile + unit * 8;
    if (col_perm) {
      const int4 c0 = reinterpret_cast<const int4*>(col_perm + k0)[0];
      const int4 c1 = reinterpret_cast<const int4*>(col_perm + k0)[1];
      const _Float16* row = X + (int64_t)m * K;
      v[0] = row[c0.x];
      v[1] = row[c0.y];
      v[2] = row[c0.z];
      v[3] = row[c0.w];
      v[4] = row[c1.x];
      v[5] = row[c1.y];
      v[6] = row[c1.z];
      v[7] = row[c1.w];
    } else {
      v = *reinterpret_cast<const half8*>(X + (int64_t)m * K + k0);
    }
  }
  *reinterpret_cast<half8*>(xblk + (((int64_t)tc * 4 + unit / 4) * 64 + 16 * (unit % 4) + m) * 16) = v;
}
__global__ __launch_bounds__(256) void stage_rows_operand_order_kernel(const _Float16* __restrict__ X,
                                                                       const int32_t* __restrict__ col_perm,
                                                                       unsigned char* xblk, int M, int K) {
  stage_rows_tile_operand_order(X, col_perm, xblk, M, K, (int)blockIdx.x);
}

template <int MB>
constexpr int rskinny_slot_bytes() { return kSlotBytes + MB * 256; }
// resident variant: bytes of the raw copy of the activations in LDS
__host__ __device__ inline size_t rskinny_raw_bytes(int32_t M, int32_t K) { return ((size_t)M * K * 2 + 15) & ~(size_t)15; }

// RES (resident): when MB x K fp16 fit in LDS beside the rings, every workgroup stages the activations itself,
// exactly as the GEMV kernel does (raw copy into the idle rings, permute inside LDS) into the same per-tile-column
// swizzled layout; there is then no staging kernel and an item brings only its slab and parameters.
// ACC: slabs per workgroup whose finished sums are held in registers (4, 8 or 16; 4 x ACC registers).  With 16
// the kernel needs about 130 vector registers and runs 8 wavefronts per CU; with 4 or 8 it stays below 128 and runs
// 16, which is what covers the latencies of its loop.  The forms with MB = 4 and with RA hold no sums in registers
// (they write them to LDS as a slab finishes); there ACC only tells the variants for 16 and for 8 wavefronts apart.
// G64: group length 64 (two parameter pairs per row and tile column; never together with RES).
// RA (activations in registers; 0, 2 or 4): when a wavefront has at most RA tile columns (K <= 128 RA NW) it loads
// their matrix-instruction operands once, from a staged copy in operand order (stage_rows_operand_order_kernel), and
// keeps them in registers (16 per tile column) for all its slabs: an item then brings only its slab and parameters
// (small slots, two of them per wavefront at any M), and nothing is read from LDS for the activations.  16 rows
// always (MB = 16).
template <int NW, int S, int MB, bool RES, int ACC, bool G64 = false, int RA = 0>
__device__ __forceinline__ void rskinny_body(const RSkinnyParams& p, const int bid, const int G, unsigned char* lds_raw) {
  static_assert(!(RES && G64), "the resident form keeps one activation sum per tile column");
  static_assert(!(RES && RA) && (!RA || MB == 16) && (RA == 0 || RA == 2 || RA == 4), "activations in registers: 16 rows, no copy in LDS");
  constexpr int NT = NW * 64;
  constexpr int kBase = G64 ? kSlotBytes64 : kSlotBytes;  // slab + parameters; the staged activations follow
  constexpr int kSlot = (RES || RA) ? kBase : kBase + MB * 256;
  constexpr int kCopies = (RES || RA) ? 2 : 2 + MB / 4;  // direct copies per item: slab, scales+zeros, MB/4 x 1 KiB of activations
  constexpr int kRedGroups = NW / 4;  // the final sum over the wavefronts is taken in groups of four
  // DS: the sums of a finished slab go straight into the wavefront's own block of LDS and none are held in
  // registers: with the activations in registers (all 64 lanes hold sums) and with up to four activation rows
  // (lanes 0-15 hold them all: output rows 4 (lane / 16) + r)
  constexpr bool DS = RA || MB == 4;
  constexpr int kFinLanes = RA ? 64 : 16;
  // LDS: red [NW/4][max_slabs][4][64] f32 | (Xs [ntc][MB][256 B] | SxL | raw activations [M][K] fp16) |
  //      rings [NW][S][kSlot];  with RA: fin [NW][max_slabs][64][4] f32 | rings
  float* red = reinterpret_cast<float*>(lds_raw);
  unsigned char* Xs = lds_raw + (DS ? (size_t)p.max_slabs * NW * kFinLanes * 16 : (size_t)p.max_slabs * 1024 * kRedGroups);
  // (resident) SxL [ntc][4 lane groups][4] f32: the sums of the activations of rows 4g..4g+3 over a tile column
  float* SxL = reinterpret_cast<float*>(Xs + (RES ? (size_t)p.ntc * (MB * 256) : (size_t)0));
  unsigned char* raw_region = reinterpret_cast<unsigned char*>(SxL) + (RES ? (size_t)p.ntc * 64 : (size_t)0);
  unsigned char* rings = raw_region + (RES ? rskinny_raw_bytes(p.M, p.K) : (size_t)0);

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int i16 = lane % 16, kb = lane / 16;
  // same slab numbering as the GEMV kernel: the 8 slabs of a tile row run on one XCD
  const int nj = p.nj_q + (bid < p.nj_r ? 1 : 0);
  const int my_cnt = p.ntc > wave ? (p.ntc - wave + NW - 1) / NW : 0;
  const int E = nj * my_cnt;  // items of this wavefront, handled in batches of 64 (one lane describes one item)

  // per-item registers of lane e: address of the slab, upper half of the lane mask of its copy, 32-bit offset of the
  // parameter dwords inside the scale / zero arrays, and the item's flags (as in the GEMV kernel)
  uint32_t it_wlo = 0, it_whi = 0, it_xhi = 0, it_soff = 0, it_misc = 0;
  auto describe = [&](int e0, int Eb) {
    if (lane < Eb) {
      // (unsigned arithmetic, and ge / my_cnt through a float reciprocal: exact for ge < 2^10 and my_cnt <= 64, since
      // ge + 0.5 is at least 0.5 / 64 away from a multiple of my_cnt; as in the GEMV kernel)
      const uint32_t ge = (uint32_t)(e0 + lane);
      const uint32_t j = (uint32_t)(((float)ge + 0.5f) * __builtin_amdgcn_rcpf((float)my_cnt));
      const uint32_t i = ge - j * (uint32_t)my_cnt;
      const uint32_t v = (uint32_t)bid + (uint32_t)G * j;
      const uint32_t slab = (v % 8) * (uint32_t)p.ntr + v / 8;
      const uint32_t tr = slab / 8, sigma = slab % 8;
      const uint32_t tc = (uint32_t)wave + NW * i;
      const uint32_t d = (uint32_t)p.tile_desc[tr * (uint32_t)p.ntc + tc];
      const uint32_t bm2 = d & 3u;
      const uint32_t slab_bytes = 256u * (bm2 + 2u);
      // (address of the slab and upper half of the lane mask of its copy, as in the GEMV kernel; the three bases
      // pass through an empty statement: chosen straight from the argument struct, the choice became an indexed load
      // from a copy of the struct in scratch memory)
      uint64_t b2 = (uint64_t)p.s2, b3 = (uint64_t)p.s3, b4 = (uint64_t)p.s4;
      asm volatile("" : "+s"(b2), "+s"(b3), "+s"(b4));
      const uint64_t waddr = (bm2 == 0 ? b2 : bm2 == 1 ? b3 : b4) +
                             ((d >> 2) * (8u * slab_bytes) + (uint32_t)sigma * slab_bytes);
      it_wlo = (uint32_t)waddr, it_whi = (uint32_t)(waddr >> 32);
      it_xhi = bm2 == 0 ? 0u : bm2 == 1 ? 0xFFFFu : 0xFFFFFFFFu;
      it_soff = 2u * (uint32_t)((G64 ? 2u * tc : tc >> p.gshift) * p.N + tr * kTile + (sigma & ~1));
      it_misc = (uint32_t)tc | ((i == (uint32_t)(my_cnt - 1)) ? 0x10000u : 0u) | ((uint32_t)j << 17) | (bm2 << 24) |
                ((uint32_t)(sigma & 1) << 26);
    }
  };
  const uint32_t data_voff = lane * 16;
  // (group length 64: lanes 32-63 read the next parameter row, as in the GEMV kernel)
  const uint64_t par_vbase = ((lane & 16) == 0 ? (uint64_t)p.scales : (uint64_t)p.zeros) + (uint64_t)((lane & 15) * 16) +
                             (G64 && lane >= 32 ? (uint64_t)p.N * 2 : (uint64_t)0);

  // Issue item e into ring slot s: the slab (scalar address, 32/48/64 lanes), the 16 scale + 16 zero dwords, and
  // without resident activations MB/4 KiB of staged activations of the item's tile column (scalar address)
  const uint32_t ring_off = (uint32_t)(uintptr_t)(lptr_t)(rings + (size_t)wave * S * kSlot);
  const unsigned char* ring = rings + (size_t)wave * S * kSlot;
  const uint64_t xb = (uint64_t)p.xblk;
  auto issue_item = [&](int e, int s) __attribute__((always_inline)) {
    const uint32_t wlo = (uint32_t)__builtin_amdgcn_readlane((int)it_wlo, e);
    const uint32_t whi = (uint32_t)__builtin_amdgcn_readlane((int)it_whi, e);
    const uint32_t xhi = (uint32_t)__builtin_amdgcn_readlane((int)it_xhi, e);
    const uint32_t soff = (uint32_t)__builtin_amdgcn_readlane((int)it_soff, e);
    const uint32_t slot = ring_off + (uint32_t)s * kSlot;
    lds_copy_item(par_vbase + soff, ((uint64_t)whi << 32) | wlo, data_voff, slot + 1024, slot, xhi, G64 ? ~0u : 0u);
    if constexpr (!RES && !RA) {
      const uint32_t misc = (uint32_t)__builtin_amdgcn_readlane((int)it_misc, e);
      const uint64_t xsrc = xb + (uint64_t)(misc & 0xFFFF) * (MB * 256);
#pragma unroll
      for (int c = 0; c < MB / 4; ++c) lds_copy_b128(xsrc + c * 1024, data_voff, slot + kBase + c * 1024, ~0ull);
    }
  };

  int issued_early = 0;  // items of the first batch that are already on their way when the loop below starts
  if constexpr (RES) {
    // Start of the resident form, ordered as in the GEMV kernel: everything that depends on the arguments alone is
    // requested at once (raw copies of the M rows into their own LDS region, 1 KiB per wavefront and copy; the
    // column permutation into registers; the tile descriptors of the first batch of items), the first items of
    // every ring go out as soon as the descriptors are there, and the activations are permuted inside LDS while
    // those are on their way.  One thread serves one (tile column, unit of 8 columns) for every row: the
    // permutation entries are the same for all rows.
    _Float16* Xraw = reinterpret_cast<_Float16*>(raw_region);
    const uint32_t raw_off = (uint32_t)(uintptr_t)(lptr_t)raw_region;
    const int raw_bytes = p.M * p.K * 2;  // a multiple of 256
    for (int c = wave * 1024; c < raw_bytes; c += NW * 1024) {
      const int nl = min(64, (raw_bytes - c) / 16);
      lds_copy_b128((uint64_t)p.X + (uint64_t)c, data_voff, raw_off + (uint32_t)c, nl == 64 ? ~0ull : (1ull << nl) - 1);
    }
    const int units = p.ntc * 16;
    int4 c0[kGemvUnitIters], c1[kGemvUnitIters];
#pragma unroll
    for (int ui = 0; ui < kGemvUnitIters; ++ui) {
      if (ui * NT < units) {  // uniform
        const int u = min(tid + ui * NT, units - 1);
        const int k0 = u * 8;  // = 128 * (tile column) + 8 * (unit)
        if (p.col_perm) {
          c0[ui] = reinterpret_cast<const int4*>(p.col_perm + k0)[0];
          c1[ui] = reinterpret_cast<const int4*>(p.col_perm + k0)[1];
        } else {
          c0[ui] = int4{k0, k0 + 1, k0 + 2, k0 + 3};
          c1[ui] = int4{k0 + 4, k0 + 5, k0 + 6, k0 + 7};
        }
      }
    }
    const int Eb0 = min(64, E);
    describe(0, Eb0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // one trip to memory for all of the above
#pragma unroll
    for (int ui = 0; ui < kGemvUnitIters; ++ui)
      if (ui * NT < units)
        asm volatile("" : "+v"(c0[ui].x), "+v"(c0[ui].y), "+v"(c0[ui].z), "+v"(c0[ui].w), "+v"(c1[ui].x),
                     "+v"(c1[ui].y), "+v"(c1[ui].z), "+v"(c1[ui].w));
    asm volatile("" : "+v"(it_wlo), "+v"(it_whi), "+v"(it_xhi), "+v"(it_soff), "+v"(it_misc));
    issued_early = min(2, min(S, Eb0));
    for (int e = 0; e < issued_early; ++e) issue_item(e, e);
    barrier_lds_only();  // every wavefront's part of the raw copy has landed (each waited for its own above)
#pragma unroll
    for (int ui = 0; ui < kGemvUnitIters; ++ui) {
      const int u = tid + ui * NT;
      if (u < units) {
        const int tc = u / 16, unit = u % 16;
        static_assert(MB == 4, "the resident variant keeps one group of four activation rows");
        floatx4 sums;
#pragma unroll
        for (int m = 0; m < MB; ++m) {
          half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
          if (m < p.M) {
            const _Float16* row = Xraw + (size_t)m * p.K;
            v[0] = row[c0[ui].x];
            v[1] = row[c0[ui].y];
            v[2] = row[c0[ui].z];
            v[3] = row[c0[ui].w];
            v[4] = row[c1[ui].x];
            v[5] = row[c1[ui].y];
            v[6] = row[c1[ui].z];
            v[7] = row[c1[ui].w];
          }
          *reinterpret_cast<half8*>(Xs + ((size_t)tc * MB + m) * 256 + ((unit ^ m) * 16)) = v;
          sums[m] = unit_group_sum(v);  // over the 16 units of the tile column (16 consecutive lanes)
        }
        // rows 0-3 belong to lane group 0 of the product; the groups of rows 4-15 (not present) read zeros
        if (unit < 4)
          *reinterpret_cast<floatx4*>(SxL + tc * 16 + unit * 4) = unit == 0 ? sums : floatx4{0.f, 0.f, 0.f, 0.f};
      }
    }
    barrier_lds_only();  // Xs and SxL are complete
  }

  half8 ones;
#pragma unroll
  for (int v = 0; v < 8; ++v) ones[v] = (_Float16)1.0f;
  half8 a[4];
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa) a[kappa] = half8{0, 0, 0, 0, 0, 0, 0, 0};
  // (RA) the operands of this wavefront's tile columns, requested now (the address of the last tile column for a
  // wavefront that has fewer: the loads are unconditional); first used when the first item is consumed
  half8 aset[RA > 0 ? RA : 1][4];
  if constexpr (RA > 0) {
#pragma unroll
    for (int t = 0; t < RA; ++t) {
      const int tc = min(wave + NW * t, p.ntc - 1);
#pragma unroll
      for (int kappa = 0; kappa < 4; ++kappa)
        aset[t][kappa] = *reinterpret_cast<const half8*>(p.xblk + (((size_t)tc * 4 + kappa) * 64 + lane) * 16);
    }
  }
  // operand addresses inside a slot: activation row i16, unit 4*kappa + kb at position unit ^ i16
  uint32_t a_off[4];
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa)
    a_off[kappa] = (RES ? 0 : kBase) + i16 * 256 + (((4 * kappa + kb) ^ i16) * 16);

  // finished sums: accs[r][q] = output element r of this lane for slab q (register-indexed writes, no switch)
  static_assert(ACC == 4 || ACC == 8 || ACC == 16, "the finished sums live in 4-, 8- or 16-wide register vectors");
  typedef float accv __attribute__((ext_vector_type(ACC)));
  accv accs0, accs1, accs2, accs3;  // four named vectors: an array of them went to scratch memory
#pragma unroll
  for (int q = 0; q < ACC; ++q) accs0[q] = 0.f, accs1[q] = 0.f, accs2[q] = 0.f, accs3[q] = 0.f;
  // Keeping the sums of a finished slab (q is uniform).  A wavefront with one or two tile columns finishes a slab
  // with every or every second item, and a register-indexed write into vectors of up to eight elements costs one
  // conditional move per element (32 per finished slab).  DS: one 16-byte write into fin [NW][max_slabs][kFinLanes][4]
  // f32 instead, and no sums in registers at all.
  float* fin = reinterpret_cast<float*>(lds_raw);
  auto keep_sums = [&](const int q, const floatx4 acc) __attribute__((always_inline)) {
    if constexpr (DS) {
      if (kFinLanes == 64 || lane < kFinLanes)
        *reinterpret_cast<floatx4*>(fin + (((size_t)wave * p.max_slabs + q) * kFinLanes + lane) * 4) = acc;
    } else {
      accs0[q] = acc[0], accs1[q] = acc[1], accs2[q] = acc[2], accs3[q] = acc[3];
    }
  };
  // running sums of the current slab: scale * (code sums, in units of 2^-24) and zero * (activation sums)
  floatx4 acc_q = {0.f, 0.f, 0.f, 0.f}, acc_z = {0.f, 0.f, 0.f, 0.f};

  // one item with its activation operands given (a: four k-steps of 32 columns)
  // (sx_known: the activation sums of the item's tile column when the caller has them already)
  auto consume_with = [&](const uint32_t misc, const unsigned char* slot, const half8 (&a)[4],
                          const floatx4 sx_known) __attribute__((always_inline)) {
    if constexpr (G64) {
      // sums of the activations over columns 0-63 and 64-127, the code sums likewise, one parameter pair for each
      floatx4 sx_lo = {0.f, 0.f, 0.f, 0.f}, sx_hi = {0.f, 0.f, 0.f, 0.f};
      sx_lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[0], ones, sx_lo, 0, 0, 0);
      sx_lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[1], ones, sx_lo, 0, 0, 0);
      sx_hi = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[2], ones, sx_hi, 0, 0, 0);
      sx_hi = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[3], ones, sx_hi, 0, 0, 0);
      floatx4 t_lo, t_hi;
      uint32_t w[4];
      const uint32_t* src;
      switch ((misc >> 24) & 3) {
        case 0:
          src = reinterpret_cast<const uint32_t*>(slot + lane * 8);
          w[0] = src[0], w[1] = src[1];
          slab_dot_halves<2>(w, a, t_lo, t_hi);
          break;
        case 1:
          src = reinterpret_cast<const uint32_t*>(slot + lane * 12);
          w[0] = src[0], w[1] = src[1], w[2] = src[2];
          slab_dot_halves<3>(w, a, t_lo, t_hi);
          break;
        default:
          src = reinterpret_cast<const uint32_t*>(slot + lane * 16);
          w[0] = src[0], w[1] = src[1], w[2] = src[2], w[3] = src[3];
          slab_dot_halves<4>(w, a, t_lo, t_hi);
          break;
      }
      const uint32_t* par = reinterpret_cast<const uint32_t*>(slot + 1024 + (lane & 15) * 4);
      float s_lo, z_lo, s_hi, z_hi;
      params_to_float(par[0], par[16], (misc >> 22) & 16u, p.bf16 != 0, s_lo, z_lo);
      params_to_float(par[32], par[48], (misc >> 22) & 16u, p.bf16 != 0, s_hi, z_hi);
      acc_q += s_lo * t_lo + s_hi * t_hi;
      acc_z += z_lo * sx_lo + z_hi * sx_hi;
      if (misc & 0x10000u) {  // this wavefront's share of slab j is complete
        asm volatile("" ::: "memory");
        const int q = (misc >> 17) & (DS ? 15 : ACC - 1);
        const floatx4 acc = acc_q * 16777216.f + acc_z;
        keep_sums(q, acc);
        acc_q = floatx4{0.f, 0.f, 0.f, 0.f}, acc_z = floatx4{0.f, 0.f, 0.f, 0.f};
      }
      return;
    }
    floatx4 sx;
    if constexpr (RA == 2) {
      sx = sx_known;
    } else if constexpr (RES) {
      sx = *reinterpret_cast<const floatx4*>(SxL + (misc & 0xFFFF) * 16 + kb * 4);
    } else {
      sx = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kappa = 0; kappa < 4; ++kappa) sx = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[kappa], ones, sx, 0, 0, 0);
    }
    floatx4 t;
    {
      uint32_t w[4];
      const uint32_t* src;
      switch ((misc >> 24) & 3) {
        case 0:
          src = reinterpret_cast<const uint32_t*>(slot + lane * 8);
          w[0] = src[0], w[1] = src[1];
          t = slab_dot_units<2>(w, a);
          break;
        case 1:
          src = reinterpret_cast<const uint32_t*>(slot + lane * 12);
          w[0] = src[0], w[1] = src[1], w[2] = src[2];
          t = slab_dot_units<3>(w, a);
          break;
        default:
          src = reinterpret_cast<const uint32_t*>(slot + lane * 16);
          w[0] = src[0], w[1] = src[1], w[2] = src[2], w[3] = src[3];
          t = slab_dot_units<4>(w, a);
          break;
      }
    }
    const uint32_t scw = *reinterpret_cast<const uint32_t*>(slot + 1024 + (lane & 15) * 4);
    const uint32_t zrw = *reinterpret_cast<const uint32_t*>(slot + 1088 + (lane & 15) * 4);
    float sf, zf;
    params_to_float(scw, zrw, (misc >> 22) & 16u, p.bf16 != 0, sf, zf);  // bit 26 of misc: odd sigma -> high half
    acc_q += sf * t;
    acc_z += zf * sx;
    if (misc & 0x10000u) {  // this wavefront's share of slab j is complete
      asm volatile("" ::: "memory");  // keeps this a branch rather than a select over all the sums
      const int q = (misc >> 17) & (DS ? 15 : ACC - 1);
      const floatx4 acc = acc_q * 16777216.f + acc_z;
      keep_sums(q, acc);
      acc_q = floatx4{0.f, 0.f, 0.f, 0.f}, acc_z = floatx4{0.f, 0.f, 0.f, 0.f};
    }
  };
  // (two tile columns in registers, one parameter pair per tile column) the activation sums of the two tile columns,
  // taken once for all slabs: the same four matrix instructions against ones, in the same order, that the other forms
  // issue per item (with four tile columns the registers go to the operands, and the sums are taken per item)
  floatx4 sx0 = {0.f, 0.f, 0.f, 0.f}, sx1 = {0.f, 0.f, 0.f, 0.f};
  if constexpr (RA == 2 && !G64) {
#pragma unroll
    for (int kappa = 0; kappa < 4; ++kappa) sx0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(aset[0][kappa], ones, sx0, 0, 0, 0);
#pragma unroll
    for (int kappa = 0; kappa < 4; ++kappa) sx1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(aset[1][kappa], ones, sx1, 0, 0, 0);
  }
  auto consume = [&](int e, int s) __attribute__((always_inline)) {
    const uint32_t misc = (uint32_t)__builtin_amdgcn_readlane((int)it_misc, e);
    const unsigned char* slot = ring + s * kSlot;
    if constexpr (RA) {
      // which of this wavefront's tile columns (a uniform branch over RA copies of the item's code: selecting the
      // operands into one more set of registers cost 16 more of them)
      const uint32_t t = (misc & 0xFFFF) >> (NW == 16 ? 4 : 3);
      if constexpr (RA == 2) {
        if (t == 0) consume_with(misc, slot, aset[0], sx0);
        else consume_with(misc, slot, aset[1], sx1);
      } else {
        if (t == 0) consume_with(misc, slot, aset[0], sx0);
        else if (t == 1) consume_with(misc, slot, aset[1], sx0);
        else if (t == 2) consume_with(misc, slot, aset[2], sx0);
        else consume_with(misc, slot, aset[3], sx0);
      }
    } else {
      if (MB == 16 || i16 < MB) {
        const unsigned char* abase = RES ? Xs + (size_t)(misc & 0xFFFF) * (MB * 256) : slot;
#pragma unroll
        for (int kappa = 0; kappa < 4; ++kappa) a[kappa] = *reinterpret_cast<const half8*>(abase + a_off[kappa]);
      }
      consume_with(misc, slot, a, floatx4{0.f, 0.f, 0.f, 0.f});
    }
  };

  for (int e0 = 0; e0 < E; e0 += 64) {
    const int Eb = min(64, E - e0);
    if (!RES || e0 > 0) describe(e0, Eb);
    const int npro = min(S, Eb);
    for (int e = (e0 == 0 ? issued_early : 0); e < npro; ++e) issue_item(e, e);
    int s = 0;
    int e = 0;
    for (; e + S < Eb; ++e) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopies * (S - 1)) : "memory");
      __builtin_amdgcn_s_setprio(1);
      consume(e, s);
      __builtin_amdgcn_s_setprio(0);
      issue_item(e + S, s);
      if (++s == S) s = 0;
    }
    // tail: item e has landed once at most the Eb-1-e younger items are outstanding
    for (; e < Eb; ++e) {
      switch (Eb - 1 - e) {
        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
        case 1: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopies * 1) : "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopies * 2) : "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopies * 3) : "memory"); break;
        case 4: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopies * 4) : "memory"); break;
        case 5: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopies * 5) : "memory"); break;
        case 6: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopies * 6) : "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopies * 7) : "memory"); break;
      }
      __builtin_amdgcn_s_setprio(1);
      consume(e, s);
      __builtin_amdgcn_s_setprio(0);
      if (++s == S) s = 0;
    }
  }
  static_assert(S <= 8 && kCopies * 7 < 64, "the tail's waits cover up to 7 younger items");

  // The wavefronts' sums are added in a fixed order, so results repeat bit for bit: inside each group of four
  // (wavefronts 4g..4g+3) one after the other, then the groups in turn.
  if constexpr (DS) {
    // every wavefront's sums are in its block of fin already (a wavefront without a tile column wrote none: zeros)
    if (my_cnt == 0 && lane < kFinLanes)
      for (int q = 0; q < nj; ++q)
        *reinterpret_cast<floatx4*>(fin + (((size_t)wave * p.max_slabs + q) * kFinLanes + lane) * 4) = floatx4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    for (int o = tid; o < nj * kFinLanes * 4; o += NT) {
      const int jj = o / (kFinLanes * 4), rem = o % (kFinLanes * 4);
      const int l = rem / 4, r = rem % 4;
      const int m = 4 * (l / 16) + r;
      if (m < p.M) {
        float sum = 0.f;
#pragma unroll
        for (int g = 0; g < kRedGroups; ++g) {
          float part = 0.f;
#pragma unroll
          for (int w = 0; w < 4; ++w) part += fin[(((size_t)(4 * g + w) * p.max_slabs + jj) * kFinLanes + l) * 4 + r];
          sum = g == 0 ? part : sum + part;
        }
        const int v = bid + G * jj;
        const int slab = (v % 8) * p.ntr + v / 8;
        const int64_t row = (int64_t)(slab / 8) * kTile + 8 * (l % 16) + (slab % 8);
        const int64_t col = p.row_perm ? p.row_perm[row] : row;
        p.Y[(int64_t)m * p.N + col] = (_Float16)sum;
      }
    }
    return;
  }
  {
    float* mine = red + (size_t)(wave / 4) * p.max_slabs * 256;
    for (int w = 0; w < 4; ++w) {
      if (wave % 4 == w) {
#pragma unroll
        for (int q = 0; q < ACC; ++q)
          if (q < nj) {
            const float fin4[4] = {accs0[q], accs1[q], accs2[q], accs3[q]};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              float* dst = mine + (q * 4 + r) * 64 + lane;
              *dst = (w == 0 ? 0.f : *dst) + fin4[r];
            }
          }
      }
      __syncthreads();
    }
  }
  for (int o = tid; o < nj * 256; o += NT) {
    const int jj = o / 256, rem = o % 256;
    const int r = rem / 64, l = rem % 64;
    const int m = 4 * (l / 16) + r;
    if (m < p.M) {
      float sum = red[o];
#pragma unroll
      for (int g = 1; g < kRedGroups; ++g) sum += red[(size_t)g * p.max_slabs * 256 + o];
      const int v = bid + G * jj;
      const int slab = (v % 8) * p.ntr + v / 8;
      const int64_t row = (int64_t)(slab / 8) * kTile + 8 * (l % 16) + (slab % 8);
      const int64_t col = p.row_perm ? p.row_perm[row] : row;
      p.Y[(int64_t)m * p.N + col] = (_Float16)sum;
    }
  }
}

template <int NW, int S, int MB, bool RES, int ACC, bool G64 = false, int RA = 0>
__global__ __launch_bounds__(NW * 64) void rskinny_kernel(const RSkinnyParams p) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  rskinny_body<NW, S, MB, RES, ACC, G64, RA>(p, (int)blockIdx.x, (int)gridDim.x, lds_raw);
}

// Several independent problems with the same M in one launch (q, k and v, or gate and up of a decoder
// layer): the grid is split between the problems as in gemv_batched_kernel.
struct RSkinnyBatch {  // laid out as GemvBatch
  int32_t first[kGemvMaxBatch + 1];
  int32_t count;
  int32_t pad[6];
  RSkinnyParams p[kGemvMaxBatch];
};
static_assert(offsetof(RSkinnyBatch, p) == 64, "the header of a batch is one 64-byte line");

template <int NW, int S, int MB, bool RES, int ACC, bool G64 = false, int RA = 0>
__global__ __launch_bounds__(NW * 64) void rskinny_batched_kernel(const RSkinnyBatch b) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int i = batch_problem_of(b.first, (int)blockIdx.x);
  const RSkinnyParams p = b.p[i];
  rskinny_body<NW, S, MB, RES, ACC, G64, RA>(p, (int)blockIdx.x - b.first[i], b.first[i + 1] - b.first[i], lds_raw);
}

// Staging for a batch: job j (one per distinct activation matrix) owns workgroups [first[j], first[j+1]).
struct StageBatch {
  const _Float16* X[kGemvMaxBatch];
  const int32_t* col_perm[kGemvMaxBatch];
  unsigned char* xblk[kGemvMaxBatch];
  int32_t K[kGemvMaxBatch];
  int32_t first[kGemvMaxBatch + 1];
  int32_t M[kGemvMaxBatch];  // rows of each job's activation matrix (at most MB)
  int32_t count;
};

template <int MB>
__global__ __launch_bounds__(MB * 16) void stage_rows_batched_kernel(const StageBatch b) {
  int j = 0;
  while (j + 1 < b.count && (int)blockIdx.x >= b.first[j + 1]) ++j;
  stage_rows_tile<MB>(b.X[j], b.col_perm[j], b.xblk[j], b.M[j], b.K[j], (int)blockIdx.x - b.first[j]);
}
__global__ __launch_bounds__(256) void stage_rows_operand_order_batched_kernel(const StageBatch b) {
  int j = 0;
  while (j + 1 < b.count && (int)blockIdx.x >= b.first[j + 1]) ++j;
  stage_rows_tile_operand_order(b.X[j], b.col_perm[j], b.xblk[j], b.M[j], b.K[j], (int)blockIdx.x - b.first[j]);
}

// ============================================================================================
// host side
// ============================================================================================
static int after_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error(what, hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return SFMP_OK;
}

// Does an M = 1 problem fit the GEMV kernel when `grid` workgroups (a multiple of 8) work on it?  LDS holds
// the permuted activation vector, the group sums, a region shared by the raw activation copy (start of the kernel)
// and the reduction buffer (end), and the per-wavefront rings.
struct GemvFit {
  bool ok;
  int32_t slots, max_slabs, lds_bytes;
};
// LDS of the GEMV kernel in front of the rings: activations, their tile-column sums, the shared region
static int64_t gemv_fixed_lds_bytes(int32_t K, int32_t max_slabs) {
  return ((int64_t)K * 2 + (int64_t)(K / kTile) * 8 + 15) / 16 * 16 + gemv_shared_region_bytes(K, max_slabs, kGemvWaves);
}
static GemvFit gemv_fit(int32_t N, int32_t K, int32_t grid) {
  GemvFit f;
  const int32_t ntr = N / kTile, ntc = K / kTile, nslab = 8 * ntr;
  f.max_slabs = (nslab + grid - 1) / grid;
  const int64_t fixed = gemv_fixed_lds_bytes(K, f.max_slabs);
  // (the rings are sized for the slots of group length 64, 128 bytes larger, whatever the layout)
  int64_t slots = (160 * 1024 - fixed) / ((int64_t)kGemvWaves * kSlotBytes64);
  if (slots > kGemvMaxSlots) slots = kGemvMaxSlots;
  const int64_t ring_bytes = slots * kGemvWaves * kSlotBytes64;
  const int64_t items = (int64_t)f.max_slabs * ((ntc + kGemvWaves - 1) / kGemvWaves);
  f.ok = grid >= 8 && grid % 8 == 0 && grid <= nslab && slots >= kGemvMinSlots && f.max_slabs <= kGemvMaxSlabs &&
         items <= kGemvMaxItems && K / 8 <= kGemvUnitIters * kGemvWaves * 64;
  f.slots = (int32_t)slots;
  f.lds_bytes = (int32_t)(fixed + ring_bytes);
  return f;
}

// ring-skinny variants: activation rows padded to MB, NW wavefronts, S ring slots, ACC slabs per workgroup in
// registers, activations resident in LDS or travelling through the rings
struct RSkinnyConfig {
  int32_t mb, nw, slots, acc;
  bool resident;
  int32_t ra;  // activations in registers (at most 2 or 4 tile columns per wavefront; 0: not): 16-row operand-order staging, small slots
};
static int32_t rskinny_mb(int32_t M) { return M <= 4 ? 4 : M <= 8 ? 8 : 16; }
// LDS of the ring-skinny kernel: reduction buffers, (resident: activations in operand layout, their tile-column sums,
// their raw copy), rings
static int64_t rskinny_lds_bytes(const RSkinnyConfig& c, int32_t max_slabs, int32_t M, int32_t K) {
  const int64_t red = (int64_t)max_slabs * 1024 * (c.nw / 4);
  // (slots sized for group length 64, 128 bytes larger, whatever the layout)
  if (c.ra) return (int64_t)max_slabs * 1024 * c.nw + (int64_t)c.nw * c.slots * kSlotBytes64;  // fin | rings
  return c.resident ? red + (int64_t)c.mb * K * 2 + (int64_t)(K / kTile) * 64 + (int64_t)rskinny_raw_bytes(M, K) +
                          (int64_t)c.nw * c.slots * kSlotBytes64
                    : red + (int64_t)c.nw * c.slots * (kSlotBytes64 + c.mb * 256);
}
// The resident variant (activations staged into LDS by every workgroup, no staging kernel) exists for blocks of
// 4 rows and M x K activations of at most 32 KiB: measured, the saved launch outweighs 256 workgroups each permuting
// the activations up to that size (8 to 17 % on K = 4096 with M <= 4) and no longer beyond it.
constexpr int64_t kResidentMaxRawBytes = 32 * 1024;
// ring slots per wavefront of the four forms (shallow, as in the GEMV kernel; 3 measured best for the resident form)
constexpr int kSlotsResident = 3, kSlotsMb4 = 2, kSlotsMb8 = 2, kSlotsMb16 = 2;
// 16 rows with 16 wavefronts: a slot carries 4 KiB of activations, and only one per wavefront fits in LDS (the other
// wavefronts of the SIMD cover the wait)
constexpr int kSlotsMb16Wide = 1;
constexpr int kSkinnyWideSlabs = 8;  // slabs per workgroup up to which the ring-skinny kernels run 16 wavefronts
constexpr int kSkinnyMaxRounds = 4;  // workgroups per CU, one after the other, accepted to get there
constexpr int kSlotsRegisterActs = 2;  // activations in registers: the slots hold a slab and its parameters only
// max_slabs: the largest number of slabs of a workgroup over the problems of the launch; K: the largest K
// g64: group length 64, for which the resident form does not exist
static RSkinnyConfig rskinny_config(int32_t M, int32_t K, int32_t max_slabs, bool g64) {
  RSkinnyConfig c;
  c.mb = rskinny_mb(M);
  // 16 wavefronts where the finished sums fit beside the rest in 128 registers and the rings in LDS
  const bool wide = max_slabs <= kSkinnyWideSlabs;
  c.nw = wide ? 16 : 8;
  c.acc = !wide ? 16 : max_slabs <= 4 ? 4 : 8;
  c.resident = false;
  c.ra = 0;
  if (c.mb == 4) c.acc = wide ? 4 : 16;  // up to four rows: the finished sums live in LDS, acc only names the variant
  if (!g64 && c.mb == 4 && (int64_t)M * K * 2 <= kResidentMaxRawBytes && K / 8 <= kGemvUnitIters * c.nw * 64) {
    c.resident = true;
    c.slots = kSlotsResident;
    if (rskinny_lds_bytes(c, max_slabs, M, K) > 160 * 1024) c.resident = false;
  }
  if (!c.resident && K / kTile <= 4 * c.nw) {
    // at most two or four tile columns per wavefront: their operands stay in registers (any M up to 16 as 16 rows)
    // and the finished sums in LDS, one KiB per wavefront and slab (no sums in registers: acc only names the variant);
    // with 8 slabs per workgroup and 16 wavefronts that does not fit beside the rings: the ordinary form then
    RSkinnyConfig r = c;
    r.ra = K / kTile <= 2 * c.nw ? 2 : 4;
    r.mb = 16;
    r.acc = r.nw == 16 ? 4 : 16;
    r.slots = kSlotsRegisterActs;
    if (rskinny_lds_bytes(r, max_slabs, M, K) <= 160 * 1024) return r;
  }
  if (!c.resident) c.slots = c.mb == 4 ? kSlotsMb4 : c.mb == 8 ? kSlotsMb8 : wide ? kSlotsMb16Wide : kSlotsMb16;
  return c;
}

DecodePlan make_decode_plan(int32_t N, int32_t K, int32_t M, int32_t group) {
  DecodePlan d;
  const int32_t ntr = N / kTile, ntc = K / kTile, nslab = 8 * ntr;
  // GEMV: persistent grid of at most 256 workgroups (multiple of 8), 16 wavefronts each.
  if (M == 1) {
    const int32_t grid = nslab < kGemvMaxGrid ? nslab : kGemvMaxGrid;
    const GemvFit f = gemv_fit(N, K, grid);
    if (f.ok) {
      d.gemv = true;
      d.grid = grid;
      d.lds_bytes = f.lds_bytes;
      d.slots = f.slots;
      d.max_slabs = f.max_slabs;
      d.mb = 1;
      d.resident = false;
      d.workspace_bytes = 0;
      return d;
    }
  }
  // Everything else goes through the ring-skinny kernel: one workgroup per CU while a workgroup's share
  // stays within 16 slabs (N <= 65536), more workgroups beyond that.
  int32_t grid = nslab < kGemvMaxGrid ? nslab : kGemvMaxGrid;
  // (two to four workgroups per CU, one after the other, while that brings a workgroup's share down to 8 slabs and
  // the kernel to 16 wavefronts: N up to 131072)
  for (int rounds = 2; rounds <= kSkinnyMaxRounds && (nslab + grid - 1) / grid > kSkinnyWideSlabs; ++rounds)
    if ((nslab + rounds * kGemvMaxGrid - 1) / (rounds * kGemvMaxGrid) <= kSkinnyWideSlabs) grid = rounds * kGemvMaxGrid;
  if ((nslab + grid - 1) / grid > kGemvMaxSlabs) grid = ((nslab + kGemvMaxSlabs - 1) / kGemvMaxSlabs + 7) / 8 * 8;
  d.gemv = false;
  d.grid = grid;
  d.max_slabs = (nslab + grid - 1) / grid;
  const RSkinnyConfig c = rskinny_config(M, K, d.max_slabs, group == 64);
  d.mb = c.mb;
  d.nw = c.nw;
  d.acc = c.acc;
  d.resident = c.resident;
  d.ra = c.ra;
  d.slots = c.slots;
  d.lds_bytes = (int32_t)rskinny_lds_bytes(c, d.max_slabs, M, K);
  d.workspace_bytes = round_up_256((int64_t)ntc * c.mb * 256);
  return d;
}

static GemvParams gemv_params(const GemmArgs& a, int32_t max_slabs, int32_t grid) {
  const sfmp_layout_t* L = a.L;
  GemvParams p;
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
  p.N = L->N;
  p.K = L->K;
  p.ntr = L->N / kTile;
  p.ntc = L->K / kTile;
  p.nj_q = 8 * p.ntr / grid;
  p.nj_r = 8 * p.ntr % grid;
  p.max_slabs = max_slabs;
  p.gshift = L->group == 512 ? 2 : L->group == 256 ? 1 : 0;
  p.bf16 = L->scale_format == SFMP_SCALE_BF16;
  p.g64 = L->group == 64;
  return p;
}

static_assert(kGemvMinSlots == 2 && kGemvMaxSlots == 2, "the GEMV kernels are instantiated for two ring slots");

static int launch_gemv_function(const void* fn, void** kargs, unsigned grid, size_t lds_bytes, void* stream) {
  if (int e = allow_full_lds(fn, "hipFuncSetAttribute(gemv)")) return e;
  hipError_t e = hipLaunchKernel(fn, dim3(grid), dim3(kGemvWaves * 64), kargs, lds_bytes, (hipStream_t)stream);
  if (e != hipSuccess) {
    note_hip_error("sfmp gemv launch", hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return after_launch("sfmp gemv launch");
}

// gemv_kernel over `grid` workgroups (the order of kargs is the kernel's parameter list)
// (two instantiations of each kernel: parameters in fp16 throughout, or a storage type looked up per problem)
static int launch_gemv_plain(GemvParams q, int32_t grid, size_t lds_bytes, void* stream) {
  void* kargs[] = {&q.tile_desc, &q.X, &q.col_perm, &q.row_perm, &q.nj_q, &q.nj_r, &q.ntr, &q.ntc, &q.K, &grid,
                   &q.N, &q.max_slabs, &q.gshift, &q.bf16, &q.s2, &q.s3, &q.s4, &q.scales, &q.zeros, &q.Y};
  const bool any = q.bf16 != 0;
  // (group length 64: one instantiation, which looks the storage type of the parameters up at run time)
  const void* fn = q.g64 ? reinterpret_cast<const void*>(&gemv_kernel<kGemvWaves, 2, true, true>)
                   : any ? reinterpret_cast<const void*>(&gemv_kernel<kGemvWaves, 2, true>)
                         : reinterpret_cast<const void*>(&gemv_kernel<kGemvWaves, 2, false>);
  return launch_gemv_function(fn, kargs, (unsigned)grid, lds_bytes, stream);
}

static int launch_gemv_batch(GemvBatch b, size_t lds_bytes, void* stream) {
  void* kargs[] = {&b.first[1], &b.first[2], &b.first[3], &b.first[4], &b.first[5],
                   &b.first[6], &b.first[7], &b.first[8], &b.probs};
  bool any = false;
  int n64 = 0;
  for (int i = 0; i < b.count; ++i) any = any || b.probs.p[i].bf16 != 0, n64 += b.probs.p[i].g64 != 0;
  if (n64 != 0 && n64 != b.count) return SFMP_ERR_SHAPE;  // one launch runs one group-length class: 64, or the others
  const void* fn = n64    ? reinterpret_cast<const void*>(&gemv_batched_kernel<kGemvWaves, 2, true, true>)
                   : any ? reinterpret_cast<const void*>(&gemv_batched_kernel<kGemvWaves, 2, true>)
                         : reinterpret_cast<const void*>(&gemv_batched_kernel<kGemvWaves, 2, false>);
  return launch_gemv_function(fn, kargs, (unsigned)b.first[kGemvMaxBatch], lds_bytes, stream);
}

// Splits the 256 workgroups of a persistent launch between `count` problems in units of 8 (one per XCD), greedily to
// the problem with the most packed bytes per workgroup, never giving a problem more workgroups than it has slabs.
static int split_grid(const GemmArgs* probs, int count, int32_t* g, int32_t max_grid = kGemvMaxGrid) {
  int64_t bytes[kGemvMaxBatch];
  int32_t total = 0;
  for (int i = 0; i < count; ++i) {
    const sfmp_layout_t* L = probs[i].L;
    bytes[i] = L->bytes_s2 + L->bytes_s3 + L->bytes_s4 + (int64_t)L->N * (L->K / L->group) * 4;
    g[i] = 8;
    total += 8;
  }
  if (total > max_grid) return SFMP_ERR_SHAPE;
  while (total + 8 <= max_grid) {
    int best = -1;
    double best_load = 0.0;
    for (int i = 0; i < count; ++i) {
      if (g[i] + 8 > 8 * (probs[i].L->N / kTile)) continue;
      const double load = (double)bytes[i] / g[i];
      if (load > best_load) {
        best_load = load;
        best = i;
      }
    }
    if (best < 0) break;
    g[best] += 8;
    total += 8;
  }
  return SFMP_OK;
}

static bool decode_offsets_fit(const sfmp_layout_t* L);
int launch_gemv_batched(const GemmArgs* probs, int count, void* stream) {
  if (count < 1 || count > kGemvMaxBatch) return SFMP_ERR_SHAPE;
  for (int i = 0; i < count; ++i)
    if (!decode_offsets_fit(probs[i].L)) return SFMP_ERR_SHAPE;
  // a single problem takes the plain kernel: its arguments are the kernel's own, one line fetched once
  if (count == 1 && probs[0].M == 1 && make_decode_plan(probs[0].L->N, probs[0].L->K, 1, probs[0].L->group).gemv)
    return launch_decode(probs[0], stream);
  int32_t g[kGemvMaxBatch];
  if (int e = split_grid(probs, count, g)) return e;
  GemvBatch b = {};
  b.count = count;
  int32_t slots = kGemvMaxSlots, lds = 0, first = 0;
  for (int i = 0; i < count; ++i) {
    const GemvFit f = gemv_fit(probs[i].L->N, probs[i].L->K, g[i]);
    if (!f.ok) return SFMP_ERR_SHAPE;
    slots = f.slots < slots ? f.slots : slots;
    b.probs.p[i] = gemv_params(probs[i], f.max_slabs, g[i]);
    b.first[i] = first;
    first += g[i];
  }
  b.first[count] = first;
  for (int i = count + 1; i <= kGemvMaxBatch; ++i) b.first[i] = first;
  // with fewer slots than a problem could use alone its LDS footprint only shrinks: size for the largest
  for (int i = 0; i < count; ++i) {
    const sfmp_layout_t* L = probs[i].L;
    const int64_t need = gemv_fixed_lds_bytes(L->K, b.probs.p[i].max_slabs) + (int64_t)slots * kGemvWaves * kSlotBytes64;
    lds = need > lds ? (int32_t)need : lds;
  }
  return launch_gemv_batch(b, (size_t)lds, stream);
}

static RSkinnyParams rskinny_params(const GemmArgs& a, int32_t M, const void* xblk, int32_t max_slabs, int32_t grid) {
  const sfmp_layout_t* L = a.L;
  RSkinnyParams p;
  p.xblk = (const unsigned char*)xblk;
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
  p.M = M;
  p.N = L->N;
  p.K = L->K;
  p.ntr = L->N / kTile;
  p.ntc = L->K / kTile;
  p.nj_q = 8 * p.ntr / grid;
  p.nj_r = 8 * p.ntr % grid;
  p.max_slabs = max_slabs;
  p.gshift = L->group == 512 ? 2 : L->group == 256 ? 1 : 0;
  p.bf16 = L->scale_format == SFMP_SCALE_BF16;
  p.g64 = L->group == 64;
  return p;
}

template <int NW, int S, int MB, bool RES, int ACC, bool G64, int RA>
static int launch_rskinny_variant(const GemmArgs& a, const DecodePlan& d, void* stream) {
  const sfmp_layout_t* L = a.L;
  const void* fn = reinterpret_cast<const void*>(&rskinny_kernel<NW, S, MB, RES, ACC, G64, RA>);
  if (int e = allow_full_lds(fn, "hipFuncSetAttribute(skinny)")) return e;
  if (RA) {
    hipLaunchKernelGGL(stage_rows_operand_order_kernel, dim3((unsigned)(L->K / kTile)), dim3(256), 0, (hipStream_t)stream,
                       (const _Float16*)a.X, a.col_perm, (unsigned char*)a.workspace, (int)a.M, (int)L->K);
    if (int e = after_launch("sfmp_gemm activation staging launch")) return e;
  } else if (!RES) {
    hipLaunchKernelGGL((stage_rows_kernel<MB>), dim3((unsigned)(L->K / kTile)), dim3(MB * 16), 0, (hipStream_t)stream,
                       (const _Float16*)a.X, a.col_perm, (unsigned char*)a.workspace, (int)a.M, (int)L->K);
    if (int e = after_launch("sfmp_gemm activation staging launch")) return e;
  }
  RSkinnyParams p = rskinny_params(a, a.M, a.workspace, d.max_slabs, d.grid);
  void* kargs[] = {&p};
  hipError_t e = hipLaunchKernel(fn, dim3((unsigned)d.grid), dim3(NW * 64), kargs, (size_t)d.lds_bytes, (hipStream_t)stream);
  if (e != hipSuccess) {
    note_hip_error("sfmp_gemm skinny launch", hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return after_launch("sfmp_gemm skinny launch");
}

// The compiled configurations (see rskinny_config): X(NW, S, MB, RES, ACC, RA)
#define SFMP_RSKINNY_CONFIGS(X)                                                                                   \
  X(16, kSlotsResident, 4, true, 4, 0) X(8, kSlotsResident, 4, true, 16, 0)                                        \
  X(16, kSlotsMb4, 4, false, 4, 0) X(8, kSlotsMb4, 4, false, 16, 0)                                                \
  X(16, kSlotsMb8, 8, false, 4, 0) X(16, kSlotsMb8, 8, false, 8, 0) X(8, kSlotsMb8, 8, false, 16, 0)             \
  X(16, kSlotsMb16Wide, 16, false, 4, 0) X(16, kSlotsMb16Wide, 16, false, 8, 0) X(8, kSlotsMb16, 16, false, 16, 0) \
  X(16, kSlotsRegisterActs, 16, false, 4, 2) X(8, kSlotsRegisterActs, 16, false, 16, 2)                                    \
  X(16, kSlotsRegisterActs, 16, false, 4, 4) X(8, kSlotsRegisterActs, 16, false, 16, 4)

static int launch_rskinny(const GemmArgs& a, const DecodePlan& d, void* stream) {
#define SFMP_X(NW_, S_, MB_, RES_, ACC_, RA_)                                                 \
  if (d.nw == NW_ && d.mb == MB_ && d.resident == RES_ && d.acc == ACC_ && d.slots == S_ && d.ra == RA_) { \
    if constexpr (!RES_) {                                                                    \
      if (a.L->group == 64) return launch_rskinny_variant<NW_, S_, MB_, RES_, ACC_, true, RA_>(a, d, stream); \
    }                                                                                         \
    return launch_rskinny_variant<NW_, S_, MB_, RES_, ACC_, false, RA_>(a, d, stream);        \
  }
  SFMP_RSKINNY_CONFIGS(SFMP_X)
#undef SFMP_X
  return SFMP_ERR_SHAPE;
}

// ---- batched launch for 2 <= M <= 16 ---------------------------------------------------------------
// Problems that read the same activation matrix through the same column permutation share one staged copy.
struct BatchStagePlan {
  int32_t job_of[kGemvMaxBatch];    // staging job of each problem
  int32_t rep[kGemvMaxBatch];       // first problem of each job
  int64_t offset[kGemvMaxBatch];    // workspace offset of each job's staged activations
  int32_t njobs;
  int64_t bytes;
};
static BatchStagePlan plan_batch_staging(const GemmArgs* probs, int count, int32_t mb) {
  BatchStagePlan sp;
  sp.njobs = 0;
  sp.bytes = 0;
  for (int i = 0; i < count; ++i) {
    int j = 0;
    for (; j < sp.njobs; ++j) {
      const GemmArgs& r = probs[sp.rep[j]];
      if (r.X == probs[i].X && r.col_perm == probs[i].col_perm && r.L->K == probs[i].L->K && r.M == probs[i].M) break;
    }
    if (j == sp.njobs) {
      sp.rep[j] = i;
      sp.offset[j] = sp.bytes;
      sp.bytes += round_up_256((int64_t)(probs[i].L->K / kTile) * mb * 256);
      ++sp.njobs;
    }
    sp.job_of[i] = j;
  }
  return sp;
}


template <int NW, int S, int MB, bool RES, int ACC, bool G64, int RA>
static int launch_rskinny_batched_variant(const GemmArgs* probs, int count, int32_t M, const int32_t* g,
                                          void* workspace, void* stream) {
  const BatchStagePlan sp = plan_batch_staging(probs, count, MB);
  StageBatch sb;
  sb.count = sp.njobs;
  int32_t sfirst = 0;
  for (int j = 0; j < sp.njobs; ++j) {
    const GemmArgs& r = probs[sp.rep[j]];
    sb.X[j] = (const _Float16*)r.X;
    sb.col_perm[j] = r.col_perm;
    sb.xblk[j] = (unsigned char*)workspace + sp.offset[j];
    sb.K[j] = r.L->K;
    sb.M[j] = r.M;
    sb.first[j] = sfirst;
    sfirst += r.L->K / kTile;
  }
  for (int j = sp.njobs; j <= kGemvMaxBatch; ++j) sb.first[j] = sfirst;
  for (int j = sp.njobs; j < kGemvMaxBatch; ++j) {
    sb.X[j] = nullptr;
    sb.col_perm[j] = nullptr;
    sb.xblk[j] = nullptr;
    sb.K[j] = 0;
    sb.M[j] = 0;
  }
  RSkinnyBatch b = {};
  b.count = count;
  int32_t first = 0;
  int64_t lds = 0;
  for (int i = 0; i < count; ++i) {
    const sfmp_layout_t* L = probs[i].L;
    const int32_t nslab = 8 * (L->N / kTile);
    const int32_t max_slabs = (nslab + g[i] - 1) / g[i];
    if (max_slabs > kGemvMaxSlabs) return SFMP_ERR_SHAPE;
    b.p[i] = rskinny_params(probs[i], probs[i].M, (const unsigned char*)workspace + sp.offset[sp.job_of[i]], max_slabs,
                            g[i]);
    const RSkinnyConfig cfg = {MB, NW, S, ACC, RES, RA};
    if (!RA && MB != 4 && max_slabs > ACC) return SFMP_ERR_SHAPE;  // (those two forms keep no sums in registers)
    const int64_t need = rskinny_lds_bytes(cfg, max_slabs, probs[i].M, L->K);
    lds = need > lds ? need : lds;
    b.first[i] = first;
    first += g[i];
  }
  for (int i = count; i <= kGemvMaxBatch; ++i) b.first[i] = first;
  for (int i = count; i < kGemvMaxBatch; ++i) b.p[i] = b.p[0];
  if (lds > 160 * 1024) return SFMP_ERR_SHAPE;
  const void* fn = reinterpret_cast<const void*>(&rskinny_batched_kernel<NW, S, MB, RES, ACC, G64, RA>);
  if (int e = allow_full_lds(fn, "hipFuncSetAttribute(skinny batched)")) return e;
  if (RA) {
    hipLaunchKernelGGL(stage_rows_operand_order_batched_kernel, dim3((unsigned)sfirst), dim3(256), 0, (hipStream_t)stream, sb);
    if (int e = after_launch("sfmp_gemm_batched activation staging launch")) return e;
  } else if (!RES) {
    hipLaunchKernelGGL((stage_rows_batched_kernel<MB>), dim3((unsigned)sfirst), dim3(MB * 16), 0, (hipStream_t)stream, sb);
    if (int e = after_launch("sfmp_gemm_batched activation staging launch")) return e;
  }
  void* kargs[] = {&b};
  hipError_t e = hipLaunchKernel(fn, dim3((unsigned)first), dim3(NW * 64), kargs, (size_t)lds, (hipStream_t)stream);
  if (e != hipSuccess) {
    note_hip_error("sfmp_gemm_batched launch", hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  return after_launch("sfmp_gemm_batched launch");
}

// One configuration for a whole batched launch: the one that fits the problem with the most slabs per workgroup and
// the largest K (resident or register activations only when every problem of the batch fits them).
static int batch_config(const GemmArgs* probs, int count, int32_t M, int32_t* g, RSkinnyConfig* c, bool* g64) {
  int32_t max_slabs = 0, max_k = 0;
  int n64 = 0;
  // one workgroup per CU, or (rounds) two to four per CU one after the other while that brings a workgroup's share
  // down to 8 slabs: with up to 8 slabs the kernels run 16 wavefronts, with more only 8 (see rskinny_config)
  for (int rounds = 1; rounds <= kSkinnyMaxRounds; ++rounds) {
    if (int e = split_grid(probs, count, g, rounds * kGemvMaxGrid)) return e;
    max_slabs = 0;
    for (int i = 0; i < count; ++i) {
      const int32_t nslab = 8 * (probs[i].L->N / kTile);
      max_slabs = std::max(max_slabs, (nslab + g[i] - 1) / g[i]);
    }
    if (max_slabs <= kSkinnyWideSlabs) break;
  }
  if (max_slabs > kSkinnyWideSlabs) {  // not reachable within four rounds: one round, 8 wavefronts
    if (int e = split_grid(probs, count, g)) return e;
    max_slabs = 0;
    for (int i = 0; i < count; ++i) {
      const int32_t nslab = 8 * (probs[i].L->N / kTile);
      max_slabs = std::max(max_slabs, (nslab + g[i] - 1) / g[i]);
    }
  }
  for (int i = 0; i < count; ++i) {
    max_k = std::max(max_k, probs[i].L->K);
    n64 += probs[i].L->group == 64;
  }
  if (n64 != 0 && n64 != count) return SFMP_ERR_SHAPE;  // one launch runs one group-length class: 64, or the others
  *g64 = n64 != 0;
  *c = rskinny_config(M, max_k, max_slabs, n64 != 0);
  return SFMP_OK;
}

int64_t batched_workspace_bytes(const GemmArgs* probs, int count, int32_t M) {
  if (M < 2) return 0;
  int32_t g[kGemvMaxBatch];
  RSkinnyConfig c;
  bool g64 = false;
  // a batch that the launch will refuse anyway gets the size of the largest staging layout
  const int32_t mb = batch_config(probs, count, M, g, &c, &g64) == SFMP_OK ? c.mb : 16;
  return plan_batch_staging(probs, count, mb).bytes;
}

int launch_decode_batched(const GemmArgs* probs, int count, int32_t M, void* workspace, void* stream) {
  if (count < 1 || count > kGemvMaxBatch || M < 1 || M > kDecodeMaxM) return SFMP_ERR_SHAPE;
  if (M == 1) return launch_gemv_batched(probs, count, stream);
  for (int i = 0; i < count; ++i)
    if (!decode_offsets_fit(probs[i].L)) return SFMP_ERR_SHAPE;
  int32_t g[kGemvMaxBatch];
  RSkinnyConfig c;
  bool n64 = false;
  if (int e = batch_config(probs, count, M, g, &c, &n64)) return e;
#define SFMP_X(NW_, S_, MB_, RES_, ACC_, RA_)                                               \
  if (c.nw == NW_ && c.mb == MB_ && c.resident == RES_ && c.acc == ACC_ && c.slots == S_ && c.ra == RA_) { \
    if constexpr (!RES_) {                                                                  \
      if (n64) return launch_rskinny_batched_variant<NW_, S_, MB_, RES_, ACC_, true, RA_>(probs, count, M, g, workspace, stream); \
    }                                                                                       \
    return launch_rskinny_batched_variant<NW_, S_, MB_, RES_, ACC_, false, RA_>(probs, count, M, g, workspace, stream); \
  }
  SFMP_RSKINNY_CONFIGS(SFMP_X)
#undef SFMP_X
  return SFMP_ERR_SHAPE;
}

// 16 < M <= 128: the product may be cut into chunks of 16 activation rows, one problem of the batched ring kernel
// each (the same weights, its own rows of X and Y).  The chunks run side by side on their shares of the CUs and read
// the same weights at about the same time, so the matrix comes from HBM once and from the caches for the other
// chunks.  Against the MFMA kernel (with a split K on these sizes) the cost grows with the number of chunks and with
// the matrix; measured on the 8B / 70B shapes (same-box A/B, whole calls) the chunked form wins
//   with K <= 8192 (the chunks keep their activations in registers): two chunks on every shape tried (4096 -> 4096
//   12 us against 19 for the MFMA kernel at M = 32, 4096 -> 14336 22 against 27, 8192 -> 28672 66 against 73); three
//   and four chunks up to 1536 tiles (4096 -> 6144: 17 against 21, 20 against 21.5; not 4096 -> 14336: 31 against 29,
//   nor 8192 -> 8192: 33 against 31); five and six up to 1024 tiles (4096 -> 4096: 18.4 against 21.1, 20.1 against 21.8;
//   eight: 33.5 against 22.9); eight on N <= 1024;
//   with a longer K (activations through the ring slots): N <= 1024 up to 8 chunks (14336 -> 1024), N <= 4096 two;
//   with K below 4096 (not measured): never.
bool use_chunked_decode(int32_t N, int32_t K, int32_t M) {
  if (M <= kDecodeMaxM || M > kDecodeMaxM * kGemvMaxBatch) return false;
  const int32_t ntr = N / kTile, ntc = K / kTile, chunks = (M + kDecodeMaxM - 1) / kDecodeMaxM;
  if (ntc < 32) return false;
  if (ntr <= 8) return true;  // (chunks <= 8 here)
  if (ntc <= 64) {
    const int64_t tiles = (int64_t)ntr * ntc;
    return chunks <= 2 || (chunks <= 4 && tiles <= 1536) || (chunks <= 6 && tiles <= 1024);
  }
  return chunks <= 2 && ntr <= 32;
}

static int chunk_problems(const GemmArgs& a, GemmArgs* probs) {
  const sfmp_layout_t* L = a.L;
  const int count = (a.M + kDecodeMaxM - 1) / kDecodeMaxM;
  for (int i = 0; i < count; ++i) {
    probs[i] = a;
    probs[i].X = (const char*)a.X + (int64_t)i * kDecodeMaxM * L->K * 2;
    probs[i].Y = (char*)a.Y + (int64_t)i * kDecodeMaxM * L->N * 2;
    probs[i].M = i + 1 < count ? kDecodeMaxM : a.M - i * kDecodeMaxM;
  }
  return count;
}

int64_t chunked_decode_workspace_bytes(const GemmArgs& a) {
  GemmArgs probs[kGemvMaxBatch];
  const int count = chunk_problems(a, probs);
  return plan_batch_staging(probs, count, rskinny_mb(kDecodeMaxM)).bytes;
}

int launch_decode_chunked(const GemmArgs& a, void* stream) {
  GemmArgs probs[kGemvMaxBatch];
  const int count = chunk_problems(a, probs);
  return launch_decode_batched(probs, count, kDecodeMaxM, a.workspace, stream);
}

// The decode kernels address a slab by a 32-bit offset into its stream and the parameters by a 32-bit offset into
// their arrays: every stream must stay below 4 GiB, which N * K < 2^33 guarantees at any mix of widths.
static bool decode_offsets_fit(const sfmp_layout_t* L) { return (int64_t)L->N * L->K < ((int64_t)1 << 33); }

int launch_decode(const GemmArgs& a, void* stream) {
  const sfmp_layout_t* L = a.L;
  if (!decode_offsets_fit(L)) return SFMP_ERR_SHAPE;
  const DecodePlan d = make_decode_plan(L->N, L->K, a.M, L->group);
  if (d.gemv) {
    const GemvParams p = gemv_params(a, d.max_slabs, d.grid);
    return launch_gemv_plain(p, d.grid, (size_t)d.lds_bytes, stream);
  }
  return launch_rskinny(a, d, stream);
}

}  // namespace sfmp

