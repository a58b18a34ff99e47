// Declarations shared by the host and device translation units of the library.
#pragma once
#include <stdint.h>

#include "../../include/sfmp.h"

namespace sfmp {

int check_shape(int32_t N, int32_t K);
int check_layout(const sfmp_layout_t* L);
void note_hip_error(const char* what, const char* text);

// How the decode path (M <= 16) runs a problem.
struct DecodePlan {
  bool gemv;         // M == 1 with the whole activation vector in LDS; otherwise the ring-skinny kernel
  int32_t grid;      // workgroups
  int32_t lds_bytes;
  int32_t slots;     // ring slots per wavefront
  int32_t max_slabs; // 16-row slabs per workgroup (upper bound)
  int32_t mb;        // activation rows padded to this (ring-skinny: 4, 8 or 16)
  int32_t nw;        // ring-skinny: wavefronts per workgroup (8 or 16)
  int32_t acc;       // ring-skinny: slabs per workgroup held in registers (4, 8 or 16)
  bool resident;     // ring-skinny: activations staged into LDS by the kernel itself, no staging launch
  int32_t ra;        // ring-skinny: tile columns per wavefront whose activations are held in registers (0, 2, 4)
  int64_t workspace_bytes;  // staged activations of the ring-skinny kernel
};
DecodePlan make_decode_plan(int32_t N, int32_t K, int32_t M, int32_t group);

// Prefill path (M > 16): workspace holds the column-gathered activation.
struct PrefillPlan {
  int32_t bm;           // rows of a workgroup's block: 128, or 64 on small grids
  int32_t ksplit;       // > 1: K is cut into this many ranges, one workgroup each, fp32 partial products
  int64_t xperm_bytes;  // column-gathered activation copy
  int64_t ytmp_bytes;   // product in reordered row order before the row un-permute pass (ksplit == 1: fp16
                        // [M, N] if a row permutation is given; ksplit > 1: fp32 [ksplit, M, N])
};
PrefillPlan make_prefill_plan(int32_t N, int32_t K, int32_t M);

constexpr int32_t kDecodeMaxM = 16;

// Raises the dynamic-LDS limit of kernel `fn` to the 160 KiB of a gfx950 compute unit.  Done once per (device,
// kernel): the record of what has been done is the only state the library keeps between calls; it is guarded by a
// mutex, so calls from several threads and on several devices are safe.  SFMP_OK or SFMP_ERR_HIP.
int allow_full_lds(const void* fn, const char* what);

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
int launch_decode_batched(const GemmArgs* problems, int count, int32_t M, void* workspace, void* stream);
int64_t batched_workspace_bytes(const GemmArgs* problems, int count, int32_t M);
// 16 < M <= 128 on matrices with few tile rows: chunks of 16 rows through the batched ring kernel
bool use_chunked_decode(int32_t N, int32_t K, int32_t M);
int64_t chunked_decode_workspace_bytes(const GemmArgs& a);
int launch_decode_chunked(const GemmArgs& a, void* stream);
int launch_prefill(const GemmArgs& a, void* stream);
}  // namespace sfmp
