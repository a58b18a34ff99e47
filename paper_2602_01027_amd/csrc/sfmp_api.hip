// extern "C" device entry points: argument checks, workspace sizing, path selection.
#include <hip/hip_runtime.h>

#include <mutex>
#include <utility>
#include <vector>

#include "sfmp_internal.h"

using namespace sfmp;

static bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

namespace sfmp {
int allow_full_lds(const void* fn, const char* what) {
  static std::mutex mu;
  static std::vector<std::pair<int, const void*>> done;  // (device, kernel) pairs whose limit has been raised
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    note_hip_error(what, "hipGetDevice failed");
    return SFMP_ERR_HIP;
  }
  std::lock_guard<std::mutex> lock(mu);
  for (const auto& d : done)
    if (d.first == dev && d.second == fn) return SFMP_OK;
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e != hipSuccess) {
    note_hip_error(what, hipGetErrorString(e));
    return SFMP_ERR_HIP;
  }
  done.emplace_back(dev, fn);
  return SFMP_OK;
}
}  // namespace sfmp

// Scratch memory of sfmp_gemm_static: one array per GPU (every device that loads the library holds its own copy at
// its own address until the process ends).  In host code the array's name is only a handle: its device address on
// the current device comes from hipGetSymbolAddress, once per device, and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char g_static_scratch[SFMP_STATIC_SCRATCH_BYTES];

static int static_scratch_of_current_device(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr_of[kMaxDevices] = {nullptr};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    note_hip_error("sfmp_gemm_static", "hipGetDevice failed or device ordinal above 63");
    return SFMP_ERR_HIP;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess || !p) {
      note_hip_error("hipGetSymbolAddress(static scratch)", hipGetErrorString(e));
      return SFMP_ERR_HIP;
    }
    ptr_of[dev] = p;
  }
  *out = ptr_of[dev];
  return SFMP_OK;
}

extern "C" {

int sfmp_unpack(const sfmp_layout_t* layout, const void* s2_dev, const void* s3_dev, const void* s4_dev,
                const int32_t* index_dev, uint8_t* codes_dev, void* hip_stream) {
  if (int e = check_layout(layout)) return e;
  if (!index_dev || !codes_dev) return SFMP_ERR_NULL;
  if ((layout->count2 && !s2_dev) || (layout->count3 && !s3_dev) || (layout->count4 && !s4_dev)) return SFMP_ERR_NULL;
  if (!aligned(s2_dev, 16) || !aligned(s3_dev, 16) || !aligned(s4_dev, 16) || !aligned(codes_dev, 8) ||
      !aligned(index_dev, 4))
    return SFMP_ERR_ALIGN;
  return launch_unpack(layout, (const uint8_t*)s2_dev, (const uint8_t*)s3_dev, (const uint8_t*)s4_dev, index_dev,
                       codes_dev, hip_stream);
}

int sfmp_gemm_workspace(const sfmp_layout_t* layout, int32_t M, int64_t* bytes) {
  if (!bytes) return SFMP_ERR_NULL;
  if (int e = check_layout(layout)) return e;
  if (M < 1) return SFMP_ERR_SHAPE;
  if (M <= kDecodeMaxM) {
    const DecodePlan d = make_decode_plan(layout->N, layout->K, M, layout->group);
    *bytes = d.workspace_bytes;
  } else if (use_chunked_decode(layout->N, layout->K, M)) {
    GemmArgs a{};
    a.L = layout;
    a.M = M;
    *bytes = chunked_decode_workspace_bytes(a);
  } else {
    const PrefillPlan d = make_prefill_plan(layout->N, layout->K, M);
    *bytes = d.xperm_bytes + d.ytmp_bytes;
  }
  if (*bytes < 256) *bytes = 256;
  return SFMP_OK;
}

int sfmp_workspace_init(void* workspace_dev, int64_t bytes, void* hip_stream) {
  if (!workspace_dev) return SFMP_ERR_NULL;
  if (bytes < 0 || (bytes % 16) != 0 || !aligned(workspace_dev, 256)) return SFMP_ERR_WORKSPACE;
  return launch_fill_zero(workspace_dev, bytes, hip_stream);
}

static int check_gemm_pointers(const void* X_dev, const int32_t* col_perm_dev, const sfmp_layout_t* layout,
                               const void* s2_dev, const void* s3_dev, const void* s4_dev, const int32_t* index_dev,
                               const void* scales_dev, const void* zeros_dev, const int8_t* bitmap_dev,
                               const int32_t* row_perm_dev, const void* Y_dev, int32_t M) {
  if (int e = check_layout(layout)) return e;
  (void)bitmap_dev;  // not read: the block-index table carries every tile's width
  if (!X_dev || !index_dev || !scales_dev || !zeros_dev || !Y_dev) return SFMP_ERR_NULL;
  if ((layout->count2 && !s2_dev) || (layout->count3 && !s3_dev) || (layout->count4 && !s4_dev)) return SFMP_ERR_NULL;
  // 16-byte vector loads / stores on everything but Y at M <= 16 (2-byte stores there)
  if (!aligned(s2_dev, 16) || !aligned(s3_dev, 16) || !aligned(s4_dev, 16) || !aligned(scales_dev, 16) ||
      !aligned(zeros_dev, 16) || !aligned(X_dev, 16) || !aligned(Y_dev, M > kDecodeMaxM ? 16 : 2) ||
      !aligned(col_perm_dev, 16) || !aligned(row_perm_dev, 16) || !aligned(index_dev, 4))
    return SFMP_ERR_ALIGN;
  return SFMP_OK;
}

static int marshal_batch(const sfmp_gemv_problem_t* problems_host, int32_t count, GemmArgs* args) {
  if (!problems_host) return SFMP_ERR_NULL;
  if (count < 1 || count > 8) return SFMP_ERR_SHAPE;
  for (int i = 0; i < count; ++i) {
    const sfmp_gemv_problem_t& q = problems_host[i];
    if (int e = check_gemm_pointers(q.X_dev, q.col_perm_dev, q.layout, q.s2_dev, q.s3_dev, q.s4_dev, q.index_dev,
                                    q.scales_dev, q.zeros_dev, q.bitmap_dev, q.row_perm_dev, q.Y_dev, 1))
      return e;
    GemmArgs& a = args[i];
    a.X = q.X_dev;
    a.M = 1;
    a.col_perm = q.col_perm_dev;
    a.L = q.layout;
    a.s2 = (const uint8_t*)q.s2_dev;
    a.s3 = (const uint8_t*)q.s3_dev;
    a.s4 = (const uint8_t*)q.s4_dev;
    a.index = q.index_dev;
    a.scales = q.scales_dev;
    a.zeros = q.zeros_dev;
    a.bitmap = q.bitmap_dev;
    a.row_perm = q.row_perm_dev;
    a.Y = q.Y_dev;
    a.workspace = nullptr;
    a.workspace_bytes = 0;
  }
  return SFMP_OK;
}

int sfmp_gemv_batched(const sfmp_gemv_problem_t* problems_host, int32_t count, void* hip_stream) {
  GemmArgs args[8];
  if (int e = marshal_batch(problems_host, count, args)) return e;
  return launch_gemv_batched(args, count, hip_stream);
}

int sfmp_gemm_batched_workspace(const sfmp_gemv_problem_t* problems_host, int32_t count, int32_t M, int64_t* bytes) {
  if (!bytes) return SFMP_ERR_NULL;
  if (M < 1 || M > kDecodeMaxM) return SFMP_ERR_SHAPE;
  GemmArgs args[8];
  if (int e = marshal_batch(problems_host, count, args)) return e;
  *bytes = batched_workspace_bytes(args, count, M);
  if (*bytes < 256) *bytes = 256;
  return SFMP_OK;
}

int sfmp_gemm_batched(const sfmp_gemv_problem_t* problems_host, int32_t count, int32_t M, void* workspace_dev,
                      int64_t workspace_bytes, void* hip_stream) {
  if (M < 1 || M > kDecodeMaxM) return SFMP_ERR_SHAPE;
  GemmArgs args[8];
  if (int e = marshal_batch(problems_host, count, args)) return e;
  if (M > 1) {
    const int64_t need = batched_workspace_bytes(args, count, M);
    if (!workspace_dev || !aligned(workspace_dev, 256) || workspace_bytes < need) return SFMP_ERR_WORKSPACE;
  }
  for (int i = 0; i < count; ++i) args[i].M = M;
  return launch_decode_batched(args, count, M, workspace_dev, hip_stream);
}

static int gemm_with_workspace(const void* X_dev, int32_t M, const int32_t* col_perm_dev, const sfmp_layout_t* layout,
                               const void* s2_dev, const void* s3_dev, const void* s4_dev, const int32_t* index_dev,
                               const void* scales_dev, const void* zeros_dev, const int8_t* bitmap_dev,
                               const int32_t* row_perm_dev, void* Y_dev, void* workspace_dev, int64_t workspace_bytes,
                               void* hip_stream) {
  GemmArgs a;
  a.X = X_dev;
  a.M = M;
  a.col_perm = col_perm_dev;
  a.L = layout;
  a.s2 = (const uint8_t*)s2_dev;
  a.s3 = (const uint8_t*)s3_dev;
  a.s4 = (const uint8_t*)s4_dev;
  a.index = index_dev;
  a.scales = scales_dev;
  a.zeros = zeros_dev;
  a.bitmap = bitmap_dev;
  a.row_perm = row_perm_dev;
  a.Y = Y_dev;
  a.workspace = workspace_dev;
  a.workspace_bytes = workspace_bytes;
  if (M <= kDecodeMaxM) return launch_decode(a, hip_stream);
  if (use_chunked_decode(layout->N, layout->K, M)) return launch_decode_chunked(a, hip_stream);
  return launch_prefill(a, hip_stream);
}

int sfmp_gemm(const void* X_dev, int32_t M, const int32_t* col_perm_dev, const sfmp_layout_t* layout,
              const void* s2_dev, const void* s3_dev, const void* s4_dev, const int32_t* index_dev,
              const void* scales_dev, const void* zeros_dev, const int8_t* bitmap_dev, const int32_t* row_perm_dev,
              void* Y_dev, void* workspace_dev, int64_t workspace_bytes, void* hip_stream) {
  if (int e = check_layout(layout)) return e;
  if (M < 1) return SFMP_ERR_SHAPE;
  if (int e = check_gemm_pointers(X_dev, col_perm_dev, layout, s2_dev, s3_dev, s4_dev, index_dev, scales_dev,
                                  zeros_dev, bitmap_dev, row_perm_dev, Y_dev, M))
    return e;
  int64_t need = 0;
  if (int e = sfmp_gemm_workspace(layout, M, &need)) return e;
  if (!workspace_dev || !aligned(workspace_dev, 256) || workspace_bytes < need) return SFMP_ERR_WORKSPACE;
  return gemm_with_workspace(X_dev, M, col_perm_dev, layout, s2_dev, s3_dev, s4_dev, index_dev, scales_dev, zeros_dev,
                             bitmap_dev, row_perm_dev, Y_dev, workspace_dev, workspace_bytes, hip_stream);
}

int sfmp_gemm_static(const void* X_dev, int32_t M, const int32_t* col_perm_dev, const sfmp_layout_t* layout,
                     const void* s2_dev, const void* s3_dev, const void* s4_dev, const int32_t* index_dev,
                     const void* scales_dev, const void* zeros_dev, const int8_t* bitmap_dev,
                     const int32_t* row_perm_dev, void* Y_dev, void* hip_stream) {
  if (int e = check_layout(layout)) return e;
  if (M < 1) return SFMP_ERR_SHAPE;
  if (int e = check_gemm_pointers(X_dev, col_perm_dev, layout, s2_dev, s3_dev, s4_dev, index_dev, scales_dev,
                                  zeros_dev, bitmap_dev, row_perm_dev, Y_dev, M))
    return e;
  int64_t need = 0;
  if (int e = sfmp_gemm_workspace(layout, M, &need)) return e;
  if (need > (int64_t)SFMP_STATIC_SCRATCH_BYTES) return SFMP_ERR_TOO_LARGE;
  void* ws = nullptr;
  if (int e = static_scratch_of_current_device(&ws)) return e;
  return gemm_with_workspace(X_dev, M, col_perm_dev, layout, s2_dev, s3_dev, s4_dev, index_dev, scales_dev, zeros_dev,
                             bitmap_dev, row_perm_dev, Y_dev, ws, (int64_t)SFMP_STATIC_SCRATCH_BYTES, hip_stream);
}

}  // extern "C"
