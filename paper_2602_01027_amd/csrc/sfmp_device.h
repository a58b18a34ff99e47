// Device-side unpack routines shared by every kernel of the library (unpack, decode GEMV,
// prefill GEMM).  gfx950 only.
//
// A packed tile gives each of the 64 lanes of a wavefront 8 slabs of B 32-bit words
// (B = bit-width); one slab holds the lane's 32 codes of one tile row-in-eight: 4 k-steps
// of 8 slots, a slot pair sharing one 32-bit mask.  Masking a pair out of a word leaves
// each code inside the low 10 bits of a 16-bit half, i.e. inside the mantissa of an fp16
// *denormal*: the half reads as q * 2^(p - 24), p being the bit position of the field.
// The fp16 MFMA units of gfx950 take denormal inputs exactly, so an operand register costs
// one v_and_b32 per pair and no bias has to be removed.  The power of two 2^p is undone on
// the activation side (see kFieldPos / prescale) or by an exact fp16 multiply.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sfmp {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2_ __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 128;
constexpr int kWave = 64;

// Bit position p of the field of pair `pair` (0..3) in k-step `kappa` (0..3), after unpack_slab.
template <int B>
__host__ __device__ constexpr int field_pos(int kappa, int pair) {
  if (B == 4) return (pair & 1) ? 4 : 0;
  if (B == 2) return 2 * pair;
  // B == 3: pairs pi = 4*kappa + pair; pi < 15 -> word pi/5, slot j = pi%5 with positions
  // (0,3,6) taken straight from the word and (0,3) after a shift by 9; the 16th pair is
  // assembled from the three spare bits at position 6.
  int pi = 4 * kappa + pair;
  if (pi == 15) return 6;
  int j = pi % 5;
  return j == 0 ? 0 : j == 1 ? 3 : j == 2 ? 6 : j == 3 ? 0 : 3;
}

// Exponent h such that activations are pre-multiplied by 2^(h - p): keeps the factors
// balanced around 1 (2-bit: 8..1/8, 3-bit: 8..1/8, 4-bit: 4..1/4).
template <int B>
__host__ __device__ constexpr int prescale_exp() { return B == 4 ? 2 : 3; }

// One slab (B words of one lane) -> 4 k-steps x 4 pair registers.  Register op[kappa][pair]
// holds, in its low and high half, the codes of slots 2*pair and 2*pair+1 of that k-step,
// each as the 16-bit integer q << field_pos<B>(kappa, pair).
template <int B>
__device__ __forceinline__ void unpack_slab(const uint32_t* w, uint32_t (&op)[4][4]);

template <>
__device__ __forceinline__ void unpack_slab<4>(const uint32_t* w, uint32_t (&op)[4][4]) {
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa) {
    const uint32_t x = w[kappa];
    const uint32_t y = x >> 8;
    op[kappa][0] = x & 0x000F000Fu;
    op[kappa][1] = x & 0x00F000F0u;
    op[kappa][2] = y & 0x000F000Fu;
    op[kappa][3] = y & 0x00F000F0u;
  }
}

template <>
__device__ __forceinline__ void unpack_slab<2>(const uint32_t* w, uint32_t (&op)[4][4]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const uint32_t x = w[i];
    const uint32_t y = x >> 8;
    op[2 * i][0] = x & 0x00030003u;
    op[2 * i][1] = x & 0x000C000Cu;
    op[2 * i][2] = x & 0x00300030u;
    op[2 * i][3] = x & 0x00C000C0u;
    op[2 * i + 1][0] = y & 0x00030003u;
    op[2 * i + 1][1] = y & 0x000C000Cu;
    op[2 * i + 1][2] = y & 0x00300030u;
    op[2 * i + 1][3] = y & 0x00C000C0u;
  }
}

template <>
__device__ __forceinline__ void unpack_slab<3>(const uint32_t* w, uint32_t (&op)[4][4]) {
  uint32_t f[16];
  uint32_t spare[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const uint32_t x = w[i];
    const uint32_t y = x >> 9;
    f[5 * i + 0] = x & 0x00070007u;
    f[5 * i + 1] = x & 0x00380038u;
    f[5 * i + 2] = x & 0x01C001C0u;
    f[5 * i + 3] = y & 0x00070007u;
    f[5 * i + 4] = y & 0x00380038u;
    spare[i] = y & 0x00400040u;  // bit 15 / 31 of the word, now at bit 6 / 22
  }
  f[15] = (((spare[2] << 1) | spare[1]) << 1) | spare[0];  // code bits 2,1,0 at bits 8,7,6
#pragma unroll
  for (int kappa = 0; kappa < 4; ++kappa)
#pragma unroll
    for (int pair = 0; pair < 4; ++pair) op[kappa][pair] = f[4 * kappa + pair];
}

// Byte offset, inside a tile, of the 16-byte chunk `chunk` (0 .. 2B-1) of lane `lane`.
__device__ __forceinline__ uint32_t chunk_offset(int chunk, int lane) { return chunk * 1024u + lane * 16u; }

// Loads the whole tile share of one lane: 8*B words as 2*B 16-byte loads (each load is
// 1 KiB contiguous across the wavefront).
template <int B>
__device__ __forceinline__ void load_tile_words(const uint8_t* tile, int lane, uint32_t (&w)[8 * B]) {
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

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  union {
    uint32_t u[4];
    half8 h;
  } x;
  x.u[0] = a;
  x.u[1] = b;
  x.u[2] = c;
  x.u[3] = d;
  return x.h;
}

}  // namespace sfmp
