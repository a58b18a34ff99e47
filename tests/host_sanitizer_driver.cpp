// Driver for the address / undefined-behaviour sanitizer build of the library's host code (sfmp_host.cpp: packer,
// bit-plane packer, permutation checks and folding, validators).  tests/test_host_sanitizers.py compiles this file
// together with sfmp_host.cpp under -fsanitize=address,undefined, feeds it a case file and compares what it writes
// with the oracle.  Any sanitizer report aborts the run (non-zero exit).
//
// case file:  int32 N, K, n | int8 bitmap[N/128 * K/128] | uint8 codes[N * K] | int32 row_perm[n] | int32 col_perm[n]
// output:     int64 sizes[6] = bytes s2, s3, s4, index words, plane bytes, table words | s2 | s3 | s4 | index |
//             planes | tile_off | folded[n] | int32 error codes of the failing calls tried at the end
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/sfmp.h"

static void must(bool ok, const char* what) {
  if (!ok) {
    std::fprintf(stderr, "host_sanitizer_driver: %s\n", what);
    std::exit(3);
  }
}

template <class T>
static void put(std::FILE* f, const std::vector<T>& v) {
  if (!v.empty()) must(std::fwrite(v.data(), sizeof(T), v.size(), f) == v.size(), "short write");
}

int main(int argc, char** argv) {
  must(argc == 3, "usage: driver <case file> <output file>");
  std::FILE* in = std::fopen(argv[1], "rb");
  must(in != nullptr, "cannot open case file");
  int32_t hdr[3];
  must(std::fread(hdr, 4, 3, in) == 3, "short header");
  const int32_t N = hdr[0], K = hdr[1], n = hdr[2];
  const size_t nt = (size_t)(N / 128) * (size_t)(K / 128);
  // exact-size heap buffers: an access one element past either end is caught
  std::vector<int8_t> bitmap(nt);
  std::vector<uint8_t> codes((size_t)N * K);
  std::vector<int32_t> row_perm((size_t)n), col_perm((size_t)n);
  must(std::fread(bitmap.data(), 1, nt, in) == nt, "short bitmap");
  must(std::fread(codes.data(), 1, codes.size(), in) == codes.size(), "short codes");
  must(std::fread(row_perm.data(), 4, (size_t)n, in) == (size_t)n, "short row_perm");
  must(std::fread(col_perm.data(), 4, (size_t)n, in) == (size_t)n, "short col_perm");
  std::fclose(in);

  sfmp_layout_t L;
  must(sfmp_pack_query(bitmap.data(), N, K, &L) == SFMP_OK, "sfmp_pack_query");
  std::vector<uint8_t> s2((size_t)L.bytes_s2), s3((size_t)L.bytes_s3), s4((size_t)L.bytes_s4);
  std::vector<int32_t> index((size_t)L.index_words);
  sfmp_layout_t out;
  must(sfmp_pack(codes.data(), bitmap.data(), N, K, s2.empty() ? nullptr : s2.data(), s3.empty() ? nullptr : s3.data(),
                 s4.empty() ? nullptr : s4.data(), index.data(), &out) == SFMP_OK, "sfmp_pack");
  int64_t plane_bytes = 0, table_words = 0;
  must(sfmp_lut_pack_query(bitmap.data(), N, K, &plane_bytes, &table_words) == SFMP_OK, "sfmp_lut_pack_query");
  std::vector<uint8_t> planes((size_t)plane_bytes);
  std::vector<uint32_t> tile_off((size_t)table_words);
  must(sfmp_lut_pack(codes.data(), bitmap.data(), N, K, planes.data(), tile_off.data()) == SFMP_OK, "sfmp_lut_pack");
  std::vector<int32_t> folded((size_t)n);
  must(sfmp_check_perm(row_perm.data(), n) == SFMP_OK && sfmp_check_perm(col_perm.data(), n) == SFMP_OK, "perms");
  must(sfmp_fold_perms(row_perm.data(), col_perm.data(), n, folded.data()) == SFMP_OK, "sfmp_fold_perms");
  std::vector<int32_t> folded_id((size_t)n);
  must(sfmp_fold_perms(row_perm.data(), nullptr, n, folded_id.data()) == SFMP_OK, "sfmp_fold_perms(identity)");
  for (int32_t j = 0; j < n; ++j) must(row_perm[(size_t)folded_id[(size_t)j]] == j, "fold with identity = inverse");

  // failing calls: every one must return its code without touching memory it does not own
  std::vector<int32_t> errs;
  {
    std::vector<uint8_t> bad_codes = codes;
    bad_codes.back() = 200;  // out of range for any width
    errs.push_back(sfmp_pack(bad_codes.data(), bitmap.data(), N, K, s2.empty() ? nullptr : s2.data(),
                             s3.empty() ? nullptr : s3.data(), s4.empty() ? nullptr : s4.data(), index.data(), &out));
    errs.push_back(sfmp_lut_pack(bad_codes.data(), bitmap.data(), N, K, planes.data(), tile_off.data()));
    std::vector<int8_t> bad_bitmap = bitmap;
    bad_bitmap[0] = 7;
    errs.push_back(sfmp_pack_query(bad_bitmap.data(), N, K, &L));
    errs.push_back(sfmp_pack_query(bitmap.data(), N + 1, K, &L));
    std::vector<int32_t> bad_perm = row_perm;
    bad_perm[0] = n;  // out of range
    errs.push_back(sfmp_check_perm(bad_perm.data(), n));
    errs.push_back(sfmp_fold_perms(bad_perm.data(), col_perm.data(), n, folded_id.data()));
    bad_perm[0] = -1;
    errs.push_back(sfmp_check_perm(bad_perm.data(), n));
    if (n > 1) {
      bad_perm[0] = row_perm[1];  // duplicate
      errs.push_back(sfmp_check_perm(bad_perm.data(), n));
    } else {
      errs.push_back(SFMP_ERR_PERM);
    }
    sfmp_layout_t L2 = out;
    errs.push_back(sfmp_layout_set_quant(&L2, 96, SFMP_SCALE_FP16));
    errs.push_back(sfmp_layout_set_quant(&L2, K >= 256 && K % 256 == 0 ? 256 : 128, SFMP_SCALE_BF16));
    must(sfmp_strerror(SFMP_ERR_PERM) != nullptr && sfmp_strerror(-1234) != nullptr, "sfmp_strerror");
  }

  std::FILE* of = std::fopen(argv[2], "wb");
  must(of != nullptr, "cannot open output file");
  const int64_t sizes[6] = {out.bytes_s2, out.bytes_s3, out.bytes_s4, out.index_words, plane_bytes, table_words};
  must(std::fwrite(sizes, 8, 6, of) == 6, "short write");
  put(of, s2);
  put(of, s3);
  put(of, s4);
  put(of, index);
  put(of, planes);
  put(of, tile_off);
  put(of, folded);
  put(of, errs);
  std::fclose(of);
  return 0;
}
