// Declarations shared by the host and device translation units of the library.
#pragma once
#include <stdint.h>

#include "../../include/sfmp.h"

namespace sfmp {

int check_shape(int32_t N, int32_t K);
int check_layout(const sfmp_layout_t* L);
void note_hip_error(const char* what, const char* text);

// How the decode kernel (M <= 16) splits a matrix: a wavefront walks `tiles_per_chunk`
// consecutive tiles of one tile row; `nchunk` chunks cover the K direction.
struct DecodePlan {
  bool gemv;  // M == 1 and K small enough for the whole activation vector to sit in LDS
  int32_t tiles_per_chunk;
  int32_t nchunk;
  int32_t row_groups;  // workgroups along N (4 tile rows each)
  int64_t counter_bytes;
  int64_t partial_bytes;
  int32_t lds_bytes;
  int32_t gemv_slots, gemv_max_slabs;
  // 2 <= M <= 16 through the rings: activation rows padded to mb, staged per tile column in the workspace
  bool rskinny;
  int32_t mb;
  int64_t xblk_bytes;
  int64_t workspace_bytes;  // what sfmp_gemm needs for this plan
};
DecodePlan make_decode_plan(int32_t N, int32_t K, int32_t M);

// Prefill path (M > 16): workspace holds the column-gathered activation.
struct PrefillPlan {
  int64_t xperm_bytes;  // column-gathered activation copy
  int64_t ytmp_bytes;   // product in reordered row order, before the row un-permute pass
};
PrefillPlan make_prefill_plan(int32_t N, int32_t K, int32_t M);

constexpr int32_t kDecodeMaxM = 16;

inline int64_t round_up_256(int64_t v) { return (v + 255) / 256 * 256; }

}  // namespace sfmp

// Kernel launchers (defined in the .hip files).  All are asynchronous on `stream` and return
// SFMP_OK or SFMP_ERR_HIP.
struct GemmArgs {
  const void* X;
  int32_t M;
  const int32_t* col_perm;
  const sfmp_layout_t* L;
  const uint8_t* s2;
  const uint8_t* s3;
  const uint8_t* s4;
  const int32_t* index;
  const void* scales;
  const void* zeros;
  const int8_t* bitmap;
  const int32_t* row_perm;
  void* Y;
  void* workspace;
  int64_t workspace_bytes;
};

namespace sfmp {
int launch_unpack(const sfmp_layout_t* L, const uint8_t* s2, const uint8_t* s3, const uint8_t* s4,
                  const int32_t* index, uint8_t* codes, void* stream);
int launch_fill_zero(void* ptr, int64_t bytes, void* stream);
int launch_decode(const GemmArgs& a, void* stream);
int launch_gemv_batched(const GemmArgs* problems, int count, void* stream);
int launch_prefill(const GemmArgs& a, void* stream);
}  // namespace sfmp
