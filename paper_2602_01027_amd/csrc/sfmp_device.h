// Device-side unpack routines shared by every kernel of the library (unpack, GEMV, skinny
// GEMM, prefill GEMM).  gfx950 only.
//
// A packed tile is 8 slabs; slab sigma holds tile rows {8i + sigma}.  Inside a slab each of
// the 64 lanes of a wavefront owns B consecutive 32-bit words (B = bit-width) = its 32 codes:
// 4 k-steps of 8 slots.  Masking a slot pair out of a word leaves each code inside the low 10
// bits of a 16-bit half, i.e. inside the mantissa of an fp16 *denormal*: the half reads as
// q * 2^(p - 24), p being the bit position of the field.  The fp16 MFMA units of gfx950 do not
// flush denormal inputs, so an MFMA operand register costs one v_and_b32 per code pair and
// no bias has to be removed.  The format places the fields so that all four registers of one
// k-step share the same p; kernels keep one accumulator per distinct p and fold 2^(24-p) into
// the fp32 scale.  (Precision: the instruction aligns its 32 products by nominal exponents, 2^-14
// for a denormal, and keeps 24 bits below the largest; a product whose activation is 2^(4+p) or
// more below the largest activation of the 32 loses low-order bits, less than 2^(E-38) each with
// E that largest exponent.  See the precision note at sfmp_gemm in sfmp.h.)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sfmp {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2_ __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTile = 128;
constexpr int kWave = 64;

// Number of distinct field positions ("classes") of width B, the class of k-step kappa and the
// bit position of a class.
template <int B>
__host__ __device__ constexpr int num_classes() { return B == 4 ? 2 : B == 2 ? 4 : 3; }
template <int B>
__host__ __device__ constexpr int step_class(int kappa) {
  return B == 4 ? (kappa & 1) : B == 2 ? kappa : (kappa == 3 ? 0 : kappa);
}
template <int B>
__host__ __device__ constexpr int class_pos(int cls) { return B == 4 ? 4 * cls : B == 2 ? 2 * cls : 3 * cls; }
template <int B>
__host__ __device__ constexpr int step_pos(int kappa) { return class_pos<B>(step_class<B>(kappa)); }

__host__ __device__ constexpr float pow2f(int e) {
  float v = 1.0f;
  for (int i = 0; i < e; ++i) v *= 2.0f;
  for (int i = 0; i < -e; ++i) v *= 0.5f;
  return v;
}

// One slab (B words of one lane) -> 4 k-steps x 4 registers.  Register op[kappa][reg] holds, in
// its low / high half, the codes of slots 2*reg / 2*reg+1 of that k-step, each as the 16-bit
// integer q << step_pos<B>(kappa).
template <int B>
__device__ __forceinline__ void unpack_slab(const uint32_t* w, uint32_t (&op)[4][4]);

template <>
__device__ __forceinline__ void unpack_slab<4>(const uint32_t* w, uint32_t (&op)[4][4]) {
#pragma unroll
  for (int reg = 0; reg < 4; ++reg) {
    const uint32_t x = w[reg];
    const uint32_t y = x >> 8;
    op[0][reg] = x & 0x000F000Fu;
    op[1][reg] = x & 0x00F000F0u;
    op[2][reg] = y & 0x000F000Fu;
    op[3][reg] = y & 0x00F000F0u;
  }
}

template <>
__device__ __forceinline__ void unpack_slab<2>(const uint32_t* w, uint32_t (&op)[4][4]) {
#pragma unroll
  for (int wd = 0; wd < 2; ++wd) {
    const uint32_t x = w[wd];
    const uint32_t y = x >> 8;
#pragma unroll
    for (int kappa = 0; kappa < 4; ++kappa) {
      const uint32_t m = 0x00030003u << (2 * kappa);
      op[kappa][wd] = x & m;
      op[kappa][wd + 2] = y & m;
    }
  }
}

template <>
__device__ __forceinline__ void unpack_slab<3>(const uint32_t* w, uint32_t (&op)[4][4]) {
  // fields j = 0..4 of each half at bits 3j; spare bit 15.  (kappa, reg) -> (word, field):
  //   0: (0,0) (1,0) (2,0) (0,3)   1: (0,1) (1,1) (2,1) (0,4)
  //   2: (0,2) (1,2) (2,2) spare   3: (1,3) (2,3) (1,4) (2,4)
  const uint32_t x0 = w[0], x1 = w[1], x2 = w[2];
  const uint32_t y0 = x0 >> 9, y1 = x1 >> 9, y2 = x2 >> 9;
  op[0][0] = x0 & 0x00070007u;
  op[0][1] = x1 & 0x00070007u;
  op[0][2] = x2 & 0x00070007u;
  op[0][3] = y0 & 0x00070007u;
  op[1][0] = x0 & 0x00380038u;
  op[1][1] = x1 & 0x00380038u;
  op[1][2] = x2 & 0x00380038u;
  op[1][3] = y0 & 0x00380038u;
  op[2][0] = x0 & 0x01C001C0u;
  op[2][1] = x1 & 0x01C001C0u;
  op[2][2] = x2 & 0x01C001C0u;
  // spare bits (bit 15 / 31 of each word) sit at bit 6 / 22 of y: code bit t comes from word t
  op[2][3] = ((((y2 & 0x00400040u) << 1) | (y1 & 0x00400040u)) << 1) | (y0 & 0x00400040u);
  op[3][0] = y1 & 0x00070007u;
  op[3][1] = y2 & 0x00070007u;
  op[3][2] = (x1 >> 12) & 0x00070007u;
  op[3][3] = (x2 >> 12) & 0x00070007u;
}

// Loads the B words of lane `lane` of slab `sigma` of a tile (one load of 4*B bytes; the 64
// lanes of a wavefront read 256*B contiguous bytes).
template <int B>
__device__ __forceinline__ void load_slab_words(const uint8_t* tile, int sigma, int lane, uint32_t* w) {
  const uint8_t* src = tile + sigma * (256 * B) + lane * (4 * B);
  if (B == 4) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
    w[0] = v[0];
    w[1] = v[1];
    w[2] = v[2];
    w[3] = v[3];
  } else if (B == 3) {
    // 12-byte lane stride: only 4-byte aligned, so three dword loads (merged into one dwordx3)
    const uint32_t* s = reinterpret_cast<const uint32_t*>(src);
    w[0] = __builtin_nontemporal_load(s);
    w[1] = __builtin_nontemporal_load(s + 1);
    w[2] = __builtin_nontemporal_load(s + 2);
  } else {
    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
    w[0] = v[0];
    w[1] = v[1];
  }
}

__device__ __forceinline__ half8 as_half8(const uint32_t (&r)[4]) {
  union {
    uint32_t u[4];
    half8 h;
  } x;
  x.u[0] = r[0];
  x.u[1] = r[1];
  x.u[2] = r[2];
  x.u[3] = r[3];
  return x.h;
}

}  // namespace sfmp
