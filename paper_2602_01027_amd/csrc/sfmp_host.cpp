// Host side of the library: argument validation, layout query, the offline packer and the
// error strings.  Plain C++ (no device code); runs without a GPU.
#include "sfmp_internal.h"

#include <cstdio>
#include <cstring>
#include <vector>

namespace sfmp {

thread_local char g_hip_error_text[256] = {0};

void note_hip_error(const char* what, const char* text) {
  std::snprintf(g_hip_error_text, sizeof(g_hip_error_text), "%s: %s", what, text ? text : "?");
}

int check_shape(int32_t N, int32_t K) {
  if (N <= 0 || K <= 0 || (N % SFMP_TILE) != 0 || (K % SFMP_TILE) != 0) return SFMP_ERR_SHAPE;
  return SFMP_OK;
}

int check_layout(const sfmp_layout_t* L) {
  if (!L) return SFMP_ERR_NULL;
  if (check_shape(L->N, L->K) != SFMP_OK) return SFMP_ERR_SHAPE;
  if (L->tile != SFMP_TILE) return SFMP_ERR_LAYOUT;
  if ((L->group != 64 && L->group != 128 && L->group != 256 && L->group != 512) || (L->K % L->group) != 0)
    return SFMP_ERR_LAYOUT;
  if (L->scale_format != SFMP_SCALE_FP16 && L->scale_format != SFMP_SCALE_BF16) return SFMP_ERR_LAYOUT;
  const int64_t ntr = L->N / SFMP_TILE, ntc = L->K / SFMP_TILE, nt = ntr * ntc;
  if (L->count2 < 0 || L->count3 < 0 || L->count4 < 0) return SFMP_ERR_LAYOUT;
  if ((int64_t)L->count2 + L->count3 + L->count4 != nt) return SFMP_ERR_LAYOUT;
  if (L->bytes_s2 != (int64_t)L->count2 * 4096 || L->bytes_s3 != (int64_t)L->count3 * 6144 ||
      L->bytes_s4 != (int64_t)L->count4 * 8192)
    return SFMP_ERR_LAYOUT;
  if (L->index_words != 3 + nt + 3 * (ntr + 1) + nt || L->bytes_index != 4 * (int64_t)L->index_words)
    return SFMP_ERR_LAYOUT;
  return SFMP_OK;
}

// Word index (32-bit, inside the tile) of word `word` of lane `lane` of slab `slab`.
static inline uint32_t word_index(int b, int lane, int slab, int word) {
  return (uint32_t)(slab * 64 * b + lane * b + word);
}

// (kappa, reg) -> (word, field) of the 3-bit format; field -1 marks the spare-bit code.
static const int8_t kField3[4][4][2] = {
    {{0, 0}, {1, 0}, {2, 0}, {0, 3}},
    {{0, 1}, {1, 1}, {2, 1}, {0, 4}},
    {{0, 2}, {1, 2}, {2, 2}, {0, -1}},
    {{1, 3}, {2, 3}, {1, 4}, {2, 4}},
};

static void pack_one_tile(const uint8_t* codes, int64_t ld, int b, uint8_t* out) {
  uint32_t* words = reinterpret_cast<uint32_t*>(out);  // streams are written on a little-endian host
  std::memset(out, 0, (size_t)2048 * b);
  for (int r = 0; r < SFMP_TILE; ++r) {
    const int slab = r % 8;
    const uint8_t* row = codes + (int64_t)r * ld;
    for (int c = 0; c < SFMP_TILE; ++c) {
      const uint32_t q = row[c];
      const int lane = 16 * ((c % 32) / 8) + r / 8;
      const int kappa = c / 32, v = c % 8, reg = v / 2, half = v % 2;
      if (b == 4) {
        words[word_index(4, lane, slab, reg)] |= q << (16 * half + 4 * kappa);
      } else if (b == 2) {
        words[word_index(2, lane, slab, reg % 2)] |= q << (16 * half + 8 * (reg / 2) + 2 * kappa);
      } else {
        const int8_t* e = kField3[kappa][reg];
        if (e[1] >= 0) {
          words[word_index(3, lane, slab, e[0])] |= q << (16 * half + 3 * e[1]);
        } else {
          for (int t = 0; t < 3; ++t) words[word_index(3, lane, slab, t)] |= ((q >> t) & 1u) << (16 * half + 15);
        }
      }
    }
  }
}

}  // namespace sfmp

using namespace sfmp;

extern "C" {

const char* sfmp_strerror(int code) {
  static thread_local char buf[320];
  switch (code) {
    case SFMP_OK: return "ok";
    case SFMP_ERR_NULL: return "a required pointer is NULL";
    case SFMP_ERR_SHAPE: return "bad shape: N and K must be positive multiples of 128 and M >= 1";
    case SFMP_ERR_BITWIDTH: return "bitmap entry is not 2, 3 or 4";
    case SFMP_ERR_CODE_RANGE: return "code out of range for its tile's bit-width";
    case SFMP_ERR_WORKSPACE: return "workspace missing, not 256-byte aligned, or too small";
    case SFMP_ERR_HIP:
      std::snprintf(buf, sizeof(buf), "HIP error (%s)", g_hip_error_text[0] ? g_hip_error_text : "no detail");
      return buf;
    case SFMP_ERR_PERM: return "not a permutation of 0..n-1";
    case SFMP_ERR_LAYOUT: return "layout struct is inconsistent";
    case SFMP_ERR_ALIGN: return "a device pointer is not aligned as the header requires (16 bytes for most)";
    case SFMP_ERR_TOO_LARGE: return "the problem needs more scratch memory than the static buffer of sfmp_gemm_static holds";
    default: return "unknown sfmp error code";
  }
}

int sfmp_pack_query(const int8_t* bitmap_host, int32_t N, int32_t K, sfmp_layout_t* out) {
  if (!bitmap_host || !out) return SFMP_ERR_NULL;
  if (int e = check_shape(N, K)) return e;
  const int64_t ntr = N / SFMP_TILE, ntc = K / SFMP_TILE, nt = ntr * ntc;
  int64_t cnt[5] = {0, 0, 0, 0, 0};
  for (int64_t i = 0; i < nt; ++i) {
    const int b = bitmap_host[i];
    if (b < 2 || b > 4) return SFMP_ERR_BITWIDTH;
    ++cnt[b];
  }
  std::memset(out, 0, sizeof(*out));
  out->N = N;
  out->K = K;
  out->tile = SFMP_TILE;
  out->group = SFMP_GROUP;
  out->scale_format = SFMP_SCALE_FP16;
  out->count2 = (int32_t)cnt[2];
  out->count3 = (int32_t)cnt[3];
  out->count4 = (int32_t)cnt[4];
  out->index_words = (int32_t)(3 + nt + 3 * (ntr + 1) + nt);
  out->bytes_s2 = cnt[2] * 4096;
  out->bytes_s3 = cnt[3] * 6144;
  out->bytes_s4 = cnt[4] * 8192;
  out->bytes_index = 4 * (int64_t)out->index_words;
  return SFMP_OK;
}

int sfmp_pack(const uint8_t* codes_host, const int8_t* bitmap_host, int32_t N, int32_t K, uint8_t* s2_host,
              uint8_t* s3_host, uint8_t* s4_host, int32_t* index_host, sfmp_layout_t* out) {
  if (!codes_host || !bitmap_host || !index_host || !out) return SFMP_ERR_NULL;
  sfmp_layout_t L;
  if (int e = sfmp_pack_query(bitmap_host, N, K, &L)) return e;
  if ((L.count2 && !s2_host) || (L.count3 && !s3_host) || (L.count4 && !s4_host)) return SFMP_ERR_NULL;
  const int64_t ntr = N / SFMP_TILE, ntc = K / SFMP_TILE, nt = ntr * ntc;

  // range check first, so that nothing is written on failure
  for (int64_t tr = 0; tr < ntr; ++tr)
    for (int64_t r = 0; r < SFMP_TILE; ++r) {
      const uint8_t* row = codes_host + (tr * SFMP_TILE + r) * (int64_t)K;
      for (int64_t tc = 0; tc < ntc; ++tc) {
        const uint8_t limit = (uint8_t)(1u << bitmap_host[tr * ntc + tc]);
        const uint8_t* p = row + tc * SFMP_TILE;
        uint8_t mx = 0;
        for (int c = 0; c < SFMP_TILE; ++c) mx = p[c] > mx ? p[c] : mx;
        if (mx >= limit) return SFMP_ERR_CODE_RANGE;
      }
    }

  uint8_t* streams[5] = {nullptr, nullptr, s2_host, s3_host, s4_host};
  int32_t next_slot[5] = {0, 0, 0, 0, 0};
  int32_t* tile_desc = index_host + 3;
  int32_t* row_ptr[5] = {nullptr, nullptr, index_host + 3 + nt, index_host + 3 + nt + (ntr + 1),
                         index_host + 3 + nt + 2 * (ntr + 1)};
  int32_t* col_idx[5] = {nullptr, nullptr, index_host + 3 + nt + 3 * (ntr + 1),
                         index_host + 3 + nt + 3 * (ntr + 1) + L.count2,
                         index_host + 3 + nt + 3 * (ntr + 1) + L.count2 + L.count3};
  index_host[0] = L.count2;
  index_host[1] = L.count3;
  index_host[2] = L.count4;
  for (int b = 2; b <= 4; ++b) row_ptr[b][0] = 0;
  for (int64_t tr = 0; tr < ntr; ++tr) {
    for (int64_t tc = 0; tc < ntc; ++tc) {
      const int b = bitmap_host[tr * ntc + tc];
      const int32_t slot = next_slot[b]++;
      tile_desc[tr * ntc + tc] = (slot << 2) | (b - 2);
      col_idx[b][slot] = (int32_t)tc;
      pack_one_tile(codes_host + tr * SFMP_TILE * (int64_t)K + tc * SFMP_TILE, K, b,
                    streams[b] + (int64_t)slot * 2048 * b);
    }
    for (int b = 2; b <= 4; ++b) row_ptr[b][tr + 1] = next_slot[b];
  }
  *out = L;
  return SFMP_OK;
}

int sfmp_layout_set_quant(sfmp_layout_t* layout, int32_t group, int32_t scale_format) {
  if (!layout) return SFMP_ERR_NULL;
  sfmp_layout_t t = *layout;
  t.group = group;
  t.scale_format = scale_format;
  if (int e = check_layout(&t)) return e;
  *layout = t;
  return SFMP_OK;
}

int sfmp_check_perm(const int32_t* perm_host, int32_t n) {
  if (!perm_host) return SFMP_ERR_NULL;
  if (n <= 0) return SFMP_ERR_SHAPE;
  std::vector<uint8_t> seen((size_t)n, 0);
  for (int32_t i = 0; i < n; ++i) {
    const int32_t v = perm_host[i];
    if (v < 0 || v >= n || seen[(size_t)v]) return SFMP_ERR_PERM;
    seen[(size_t)v] = 1;
  }
  return SFMP_OK;
}

int sfmp_fold_perms(const int32_t* row_perm_prev_host, const int32_t* col_perm_next_host, int32_t n,
                    int32_t* folded_host) {
  if (!row_perm_prev_host || !folded_host) return SFMP_ERR_NULL;
  if (int e = sfmp_check_perm(row_perm_prev_host, n)) return e;
  if (col_perm_next_host)
    if (int e = sfmp_check_perm(col_perm_next_host, n)) return e;
  std::vector<int32_t> inverse((size_t)n);
  for (int32_t i = 0; i < n; ++i) inverse[(size_t)row_perm_prev_host[i]] = i;
  for (int32_t j = 0; j < n; ++j) folded_host[j] = inverse[(size_t)(col_perm_next_host ? col_perm_next_host[j] : j)];
  return SFMP_OK;
}

// ---- bit-plane format of the lookup-table GEMV ---------------------------------------------------------------
int sfmp_lut_pack_query(const int8_t* bitmap_host, int32_t N, int32_t K, int64_t* plane_bytes, int64_t* table_words) {
  if (!bitmap_host || !plane_bytes || !table_words) return SFMP_ERR_NULL;
  if (int e = sfmp::check_shape(N, K)) return e;
  const int64_t ntiles = (int64_t)(N / 128) * (K / 128);
  int64_t planes = 0;
  for (int64_t t = 0; t < ntiles; ++t) {
    const int b = bitmap_host[t];
    if (b < 2 || b > 4) return SFMP_ERR_BITWIDTH;
    planes += b;
  }
  if (planes >= ((int64_t)1 << 32)) return SFMP_ERR_SHAPE;
  *plane_bytes = planes * 2048;
  *table_words = ntiles + 1;
  return SFMP_OK;
}

int sfmp_lut_pack(const uint8_t* codes_host, const int8_t* bitmap_host, int32_t N, int32_t K, uint8_t* planes_host,
                  uint32_t* tile_off_host) {
  if (!codes_host || !bitmap_host || !planes_host || !tile_off_host) return SFMP_ERR_NULL;
  int64_t plane_bytes = 0, words = 0;
  if (int e = sfmp_lut_pack_query(bitmap_host, N, K, &plane_bytes, &words)) return e;
  const int32_t ntr = N / 128, ntc = K / 128;
  uint32_t off = 0;
  for (int32_t tr = 0; tr < ntr; ++tr)
    for (int32_t tc = 0; tc < ntc; ++tc) {
      const int b = bitmap_host[(int64_t)tr * ntc + tc];
      tile_off_host[(int64_t)tr * ntc + tc] = off;
      for (int i = 0; i < b; ++i) {
        uint8_t* plane = planes_host + ((int64_t)off + i) * 2048;
        for (int r = 0; r < 128; ++r) {
          const uint8_t* row = codes_host + ((int64_t)tr * 128 + r) * K + (int64_t)tc * 128;
          for (int g = 0; g < 16; ++g) {
            unsigned byte = 0;
            for (int t = 0; t < 8; ++t) {
              const unsigned q = row[8 * g + t];
              if (i == 0 && (q >> b) != 0) return SFMP_ERR_CODE_RANGE;
              byte |= ((q >> i) & 1u) << t;
            }
            plane[r * 16 + g] = (uint8_t)byte;
          }
        }
      }
      off += (uint32_t)b;
    }
  tile_off_host[(int64_t)ntr * ntc] = off;
  return SFMP_OK;
}

}  // extern "C"
