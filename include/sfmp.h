/*
 * sfmp.h - C ABI of the MI355X (gfx950) block-wise mixed-precision GEMM / GEMV library.
 *
 * The operation (paper: Fig. 3(c); Section 3.3 block-wise bit allocation; Section 3.4
 * Eq. 8-9 row/column reordering; Section 3.5 unified mixed-precision kernel; Appendix B
 * Eq. 11 dequantisation form):
 *
 *     Y[m, row_perm[i]] = sum_j  X[m, col_perm[j]] * ( s[j/128, i] * q[i, j] + z[j/128, i] )
 *
 * where q is the integer code matrix of the reordered weight Wt [N, K] (N output features,
 * K input features), every 128 x 128 tile of Wt carries its own bit-width b in {2,3,4}
 * (the "bitmap"), and (s, z) is one fp16 scale / additive zero-point pair per row per
 * group of 128 reordered columns (other group lengths and bf16 storage: sfmp_layout_set_quant).
 *
 * Conventions
 *   - Every function returns SFMP_OK (0) or a negative SFMP_ERR_* code and never throws.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory on
 *     the current device.  All buffers are owned by the caller; the library allocates and
 *     frees no device memory and never synchronises the stream.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *   - N and K must be positive multiples of 128; M >= 1 is arbitrary.
 *
 * Packed format (what sfmp_pack writes and the kernels read)
 *   Three byte streams S2, S3, S4.  Stream S_b holds all tiles of width b in ascending
 *   (tile row, tile column) order; a tile of width b occupies exactly 2048*b bytes.
 *   A tile is 8 slabs of 256*b bytes; slab sigma holds the tile rows {8i + sigma}.  Inside a
 *   slab each of 64 lanes owns b consecutive little-endian 32-bit words: word w of lane l of
 *   slab sigma is at byte offset sigma*256*b + l*4*b + 4*w of the tile, so one load of 4*b
 *   bytes per lane of a 64-wide wavefront reads 256*b contiguous bytes, and a 16-row slab of
 *   a tile can be fetched on its own.
 *   Element (r, c) of the tile (r = row, c = column inside the tile) belongs to
 *       lane  l     = 16*((c%32)/8) + r/8
 *       slab  sigma = r%8
 *       step  kappa = c/32,  slot v = c%8,  reg = v/2,  half = v%2
 *   and its bits sit inside the lane's b words of that slab at
 *       b=4: word reg,     bits [16*half + 4*kappa, +4)
 *       b=2: word reg%2,   bits [16*half + 8*(reg/2) + 2*kappa, +2)
 *       b=3: every 16-bit half of a word holds five 3-bit fields j=0..4 at bits [3j, 3j+3) and
 *            one spare bit 15; (kappa, reg) -> (word, field):
 *                kappa 0: (0,0) (1,0) (2,0) (0,3)
 *                kappa 1: (0,1) (1,1) (2,1) (0,4)
 *                kappa 2: (0,2) (1,2) (2,2) SPARE
 *                kappa 3: (1,3) (2,3) (1,4) (2,4)
 *            SPARE: bit t of the code is the spare bit (bit 16*half + 15) of word t, t = 0,1,2.
 *   With this placement the two codes of a register (slots 2*reg, 2*reg+1) share one 32-bit
 *   mask and land inside the fp16 mantissa window of the two halves, the four registers of a
 *   k-step share one field position, and the 8 slots of a lane are exactly the 8 k-values that
 *   lane feeds to a 16x16x32 fp16 matrix instruction.
 *
 *   Block-index table (int32 words), replacing any run-time offset computation
 *   (Appendix G, "Comparison with LUT-based GEMM Family", attributes a <=3 % cost to computing block offsets at
 *   run time):
 *       [0,3)                 number of tiles of width 2, 3, 4
 *       [3, 3+nt)             tile_desc[tr*(K/128)+tc] = (slot << 2) | (b-2); slot = index of
 *                             the tile inside stream S_b
 *       3 x (N/128 + 1)       row_ptr_b for b = 2,3,4 (CSR over tile rows)
 *       count2+count3+count4  col_idx_b for b = 2,3,4 (tile column of each tile, stream order)
 */
#ifndef SFMP_H
#define SFMP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SFMP_TILE 128
#define SFMP_GROUP 128        /* default quantisation group length along K */
#define SFMP_SCALE_FP16 0     /* scales and zeros stored as IEEE fp16 */
#define SFMP_SCALE_BF16 1     /* ... as bfloat16 (the storage type of the paper's Table 1) */

#define SFMP_OK 0
#define SFMP_ERR_NULL (-1)        /* a required pointer is NULL */
#define SFMP_ERR_SHAPE (-2)       /* N or K not a positive multiple of 128, or M < 1 */
#define SFMP_ERR_BITWIDTH (-3)    /* a bitmap entry is not 2, 3 or 4 */
#define SFMP_ERR_CODE_RANGE (-4)  /* a code is >= 2^b for its tile */
#define SFMP_ERR_WORKSPACE (-5)   /* workspace missing, misaligned (256 B) or too small */
#define SFMP_ERR_HIP (-6)         /* a HIP call or kernel launch failed */
#define SFMP_ERR_PERM (-7)        /* sfmp_check_perm: not a permutation of 0..n-1 */
#define SFMP_ERR_LAYOUT (-8)      /* layout struct inconsistent with itself */
#define SFMP_ERR_ALIGN (-9)       /* a device pointer is not aligned as required (see sfmp_gemm) */
#define SFMP_ERR_TOO_LARGE (-10)  /* sfmp_gemm_static: the problem needs more scratch than the static buffer holds */

#define SFMP_LUT_TABLE_FP32 0  /* sfmp_lut_gemv: table entries held as fp32 */
#define SFMP_LUT_TABLE_FP16 1  /* ... as fp16, the 2-byte entries of Appendix F (fp32 sum of the 8 activations, rounded once) */

#define SFMP_STATIC_SCRATCH_BYTES (16 * 1024 * 1024)  /* scratch of sfmp_gemm_static, per GPU */

/* Sizes of a packed matrix.  Filled by sfmp_pack_query / sfmp_pack; passed by the caller,
 * unchanged, to the device entry points. */
typedef struct sfmp_layout {
  int32_t N, K;                    /* rows (output features) and columns (input features) of Wt */
  int32_t tile, group;             /* 128, 128 */
  int32_t count2, count3, count4;  /* tiles of each width */
  int32_t index_words;             /* length of the block-index table in int32 words */
  int64_t bytes_s2, bytes_s3, bytes_s4, bytes_index;
  int32_t scale_format;            /* SFMP_SCALE_FP16 (default) or SFMP_SCALE_BF16 */
  int32_t reserved;                /* 0 */
} sfmp_layout_t;

/* Text for an error code (static storage, never NULL).  For SFMP_ERR_HIP the text of the last
 * HIP error seen by the calling thread is appended. */
const char* sfmp_strerror(int code);

/* Host only.  Sizes of the three streams and of the index table for a bitmap
 * (int8 [N/128, K/128], row-major, host).  Section 4.2, paragraph "Extra Metadata": one int8 per block. */
int sfmp_pack_query(const int8_t* bitmap_host, int32_t N, int32_t K, sfmp_layout_t* out);

/* Host only.  Chooses the quantisation-parameter format of a layout filled by sfmp_pack_query / sfmp_pack
 * (which set group 128, fp16): group = 64, 128, 256 or 512 columns per (scale, zero) pair, K a multiple of it
 * (Appendix G "Effect of n_b": the block width n_b is also the group size); scale_format = SFMP_SCALE_FP16 or
 * SFMP_SCALE_BF16.  The packed streams and the index table do not depend on either.  scales and zeros are then
 * [K/group, N] arrays of 16-bit values in that format.  With group 64 a 128-column tile holds two groups, which share
 * the tile's bit-width (a bit-allocation block narrower than 128 columns is not expressible: the bitmap has one entry
 * per 128 x 128 tile).  SFMP_ERR_LAYOUT for any other value. */
int sfmp_layout_set_quant(sfmp_layout_t* layout, int32_t group, int32_t scale_format);

/* Host only.  Packs codes (uint8 [N, K] row-major, reordered coordinates, host) into the three
 * streams and writes the block-index table; all four outputs are host buffers of the sizes
 * sfmp_pack_query reports (a stream of size 0 may be NULL).  Every code is checked against
 * its tile's width.  The caller uploads the buffers (each to a 16-byte aligned device
 * address).  This is the offline packing step of Section 3.5 / Appendix F ("block-major
 * layout, contiguous within each block"), in the byte format described above. */
int sfmp_pack(const uint8_t* codes_host, const int8_t* bitmap_host, int32_t N, int32_t K,
              uint8_t* s2_host, uint8_t* s3_host, uint8_t* s4_host, int32_t* index_host,
              sfmp_layout_t* out);

/* Device.  Expands the packed streams back to codes_dev (uint8 [N, K] row-major, device) with
 * the same device unpack routines the GEMM kernels use.  Asynchronous on hip_stream.
 * Debug / parity entry point: unpacked codes must equal the packer's input bit for bit. */
int sfmp_unpack(const sfmp_layout_t* layout, const void* s2_dev, const void* s3_dev, const void* s4_dev,
                const int32_t* index_dev, uint8_t* codes_dev, void* hip_stream);

/* Host only.  Bytes of device workspace sfmp_gemm needs for this layout and M
 * (256-byte granularity; never 0). */
int sfmp_gemm_workspace(const sfmp_layout_t* layout, int32_t M, int64_t* bytes);

/* Device.  Zero-fills a workspace (a small fill kernel on hip_stream, safe under graph
 * capture).  Optional: sfmp_gemm writes every workspace byte it later reads (staged or gathered
 * activations, the product before the row un-permute), so an uninitialised workspace is fine.
 * One workspace serves one stream at a time: two calls that overlap on the same workspace
 * race. */
int sfmp_workspace_init(void* workspace_dev, int64_t bytes, void* hip_stream);

/* Device.  The mixed-precision product of Fig. 3(c):
 *   X         fp16 [M, K] row-major, ORIGINAL column order.
 *   col_perm  int32 [K]; the kernel reads X[m, col_perm[j]] for reordered column j
 *             (Section 3.4: the weight's column permutation applied to the activation);
 *             NULL = identity.
 *   layout, s2, s3, s4, index   a matrix packed by sfmp_pack, uploaded unchanged.
 *   scales, zeros  16-bit [K/group, N] (group-major; group and storage type from the layout, fp16 and 128
 *             unless sfmp_layout_set_quant said otherwise): w_hat = s*q + z (Appendix B Eq. 11).
 *   bitmap    int8 [N/128, K/128] (device), the bitmap the matrix was packed with, or NULL.  It is part of the
 *             operation's statement (Section 4.2 "Extra Metadata": one int8 per block) but no kernel reads it: the
 *             block-index table that sfmp_pack derived from it carries every tile's width and position, and is
 *             the authority.  A bitmap that disagrees with the index table is not detected.
 *   row_perm  int32 [N]; output feature i of the reordered product is stored at column
 *             row_perm[i] of Y (undoing P_row of Eq. 9); NULL = leave the rows reordered.
 *   Y         fp16 [M, N] row-major; fully overwritten.  fp32 accumulation, one
 *             round-to-nearest-even conversion at the end.  The order of the fp32 sums is fixed for a given
 *             (N, K, M, group length): the same call on the same inputs gives the same bits, on any stream
 *             (no floating-point atomics anywhere).
 *   workspace device memory of at least sfmp_gemm_workspace() bytes, 256-byte aligned; contents
 *             on entry are irrelevant, contents on return are unspecified.
 * Alignment (SFMP_ERR_ALIGN otherwise): X, col_perm, row_perm, s2, s3, s4, scales and zeros 16 bytes (the kernels
 * read them with 16-byte vector loads and direct global-to-LDS copies); index 4 bytes; Y 2 bytes for M <= 16 and
 * 16 bytes for M > 16 (whole 16-byte row segments are stored there).
 * Precision for M <= 16 (and the chunks of 16 rows): the codes go through the matrix cores as fp16 denormals, and
 * v_mfma_f32_16x16x32_f16 aligns its 32 products by nominal exponents (2^-14 for a denormal) and keeps 24 bits below the
 * largest: a product whose activation lies 2^4 or more below the largest activation of its 32 columns loses low-order
 * bits, less than |s| 2^(E-14) each (E = exponent of that largest activation) - of the order of 2^-14 of the largest
 * product of those 32 columns, above fp32 rounding and far below the fp16 rounding of the result unless the result is
 * a small difference of large terms.
 * Number range: for M <= 16 scales and zeros are widened to fp32 and never rounded.  For M > 16 on the matrix-core
 * path the dequantised weight s*q + z is formed and rounded ONCE in fp16 (bf16 parameters are converted to fp16 first,
 * which is exact inside fp16's normal range): scales, zeros and weights must lie within fp16's normal range,
 * 2^-14 <= |v| <= 65504 (or be 0), to keep full precision; below it a weight carries an absolute error of up to 2^-25,
 * above it it overflows.
 * M = 1 runs the bandwidth-bound GEMV kernel, 2 <= M <= 16 (and M = 1 with K above about 32k) the
 * same scheme with the activations staged per tile column, 16 < M <= 128 with K >= 4096 on matrices and
 * batch sizes where that measured faster (N <= 1024: M <= 128; K <= 8192: M <= 32 on any N, M <= 64 up to
 * 1536 tiles of 128 x 128, M <= 96 up to 1024 tiles; longer K: M <= 32 on N <= 4096) that kernel once more, on
 * chunks of 16 rows side by side in one launch, and everything else the MFMA prefill kernels (with K
 * cut into ranges and fp32 partial products in the workspace when there would be few workgroups;
 * SFMP_ERR_SHAPE there if K > 57344, or, with a row permutation or a split K, N > 81920; the kernels for
 * M <= 16 and for the chunked form return SFMP_ERR_SHAPE if N * K >= 2^33).
 * Asynchronous on hip_stream; re-entrant and thread-safe.  The only state kept between calls is a mutex-guarded
 * record, per device, of the kernels whose LDS limit has been raised.  The permutations are not checked for
 * being bijections (out-of-range entries are the caller's error; use sfmp_check_perm). */
int sfmp_gemm(const void* X_dev, int32_t M, const int32_t* col_perm_dev, const sfmp_layout_t* layout,
              const void* s2_dev, const void* s3_dev, const void* s4_dev, const int32_t* index_dev,
              const void* scales_dev, const void* zeros_dev, const int8_t* bitmap_dev,
              const int32_t* row_perm_dev, void* Y_dev, void* workspace_dev, int64_t workspace_bytes,
              void* hip_stream);

/* Device.  sfmp_gemm for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same arguments and the same result, bit for
 * bit, as sfmp_gemm, without the workspace: the scratch memory (staged or gathered activations, the product before the
 * row un-permute, partial products of a split K) is a 256-byte aligned array of SFMP_STATIC_SCRATCH_BYTES (16 MiB) that
 * is part of the library's device code, one copy per GPU, held from the moment the library is loaded on that GPU until
 * the process ends.  The call allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine); its
 * first call on a device looks the array's address up once (hipGetSymbolAddress) - make that first call outside any
 * graph capture.  SFMP_ERR_TOO_LARGE if sfmp_gemm_workspace(layout, M) exceeds SFMP_STATIC_SCRATCH_BYTES (for example
 * M = 2048 on K = 4096; every M <= 16 fits for K up to 1 Mi); other errors as sfmp_gemm.  Nothing in the scratch
 * has to start at zero: every call writes what it later reads, whatever the previous call left.  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads) race; order them. */
int sfmp_gemm_static(const void* X_dev, int32_t M, const int32_t* col_perm_dev, const sfmp_layout_t* layout,
                     const void* s2_dev, const void* s3_dev, const void* s4_dev, const int32_t* index_dev,
                     const void* scales_dev, const void* zeros_dev, const int8_t* bitmap_dev,
                     const int32_t* row_perm_dev, void* Y_dev, void* hip_stream);

/* One problem of a batched launch: the arguments of sfmp_gemm without M and workspace. */
typedef struct sfmp_gemv_problem {
  const void* X_dev;             /* fp16 [M, K] */
  const int32_t* col_perm_dev;   /* int32 [K] or NULL */
  const sfmp_layout_t* layout;   /* host pointer; read during the call only */
  const void* s2_dev;
  const void* s3_dev;
  const void* s4_dev;
  const int32_t* index_dev;
  const void* scales_dev;
  const void* zeros_dev;
  const int8_t* bitmap_dev;
  const int32_t* row_perm_dev;   /* int32 [N] or NULL */
  void* Y_dev;                   /* fp16 [M, N] */
} sfmp_gemv_problem_t;

/* Device.  Up to 8 independent M = 1 products (each exactly what sfmp_gemm computes, each with its
 * own weights, permutations, X and Y) in ONE kernel launch: the launch and first-touch latency that
 * bounds small decode layers is paid once for, say, the q, k and v projections of a decoder layer
 * (Section 4 measures decode at batch 1, where every projection is a GEMV).  problems_host is a host
 * array read during the call.  Needs no workspace.  SFMP_ERR_SHAPE if a problem cannot use the
 * GEMV kernel (K above about 32k) - call sfmp_gemm per problem then. */
int sfmp_gemv_batched(const sfmp_gemv_problem_t* problems_host, int32_t count, void* hip_stream);

/* The same for a small batch: up to 8 independent products with a common M, 1 <= M <= 16 (each exactly what
 * sfmp_gemm computes; X_dev of a problem is fp16 [M, K], Y_dev fp16 [M, N]), in one launch of the GEMM kernel plus,
 * for M >= 2, one launch of the activation staging kernel.  Problems that pass the same X_dev, col_perm_dev and K
 * (q, k and v; gate and up) share one staged copy of the activations.  M = 1 is sfmp_gemv_batched.
 * One launch runs one form of the kernel, chosen for the whole batch (by its largest K and its largest share of
 * slabs per workgroup), which may not be the form a single sfmp_gemm call takes for one of its problems: the operation
 * is the same, the order of the fp32 sums and hence the last bit of an output may differ from the single call.  The
 * same batch on the same inputs gives the same bits every time.
 * sfmp_gemm_batched_workspace (host only) gives the workspace size for these problems and this M (never 0);
 * the workspace is device memory, 256-byte aligned, contents irrelevant on entry and unspecified on return.
 * SFMP_ERR_SHAPE if M is outside 1..16, if a problem would put more than 16 slabs on a workgroup (N above about
 * 65536 times its share of the grid), or if some but not all problems have group length 64 (one launch runs one of
 * the two classes; sfmp_gemv_batched likewise) - call sfmp_gemm per problem then. */
int sfmp_gemm_batched_workspace(const sfmp_gemv_problem_t* problems_host, int32_t count, int32_t M, int64_t* bytes);
int sfmp_gemm_batched(const sfmp_gemv_problem_t* problems_host, int32_t count, int32_t M, void* workspace_dev,
                      int64_t workspace_bytes, void* hip_stream);

/* Host only.  SFMP_OK if perm_host[0..n) is a permutation of 0..n-1, else SFMP_ERR_PERM. */
int sfmp_check_perm(const int32_t* perm_host, int32_t n);

/* Host only.  Folds the row permutation of one matrix into the column permutation of the next, so that the
 * first product can stay in reordered row order (row_perm_dev = NULL: no un-permute pass) and the second
 * gathers from it directly (Section 3.4: the reordering is applied to activations and undone on outputs; the
 * reorder-overhead measurement of Section 4.2 counts exactly these two reorder operations per layer):
 *   folded[j] = inverse(row_perm_prev)[col_perm_next[j]],   j in [0, n)
 * so that  Xt[:, folded[j]] = X[:, col_perm_next[j]]  whenever  Xt[:, i] = X[:, row_perm_prev[i]],  which holds
 * for Xt = f(Yt), X = f(Y) with any element-wise f between the two matrices (a per-feature weight, as in a norm,
 * has to be reordered by the caller the same way).  col_perm_next_host = NULL stands for the identity.  n is
 * the first matrix' N and the second one's K.  SFMP_ERR_PERM if either input is not a permutation.
 * folded_host may not alias the inputs. */
int sfmp_fold_perms(const int32_t* row_perm_prev_host, const int32_t* col_perm_next_host, int32_t n,
                    int32_t* folded_host);

/* ---- One-bit lookup-table GEMV on a bit-plane format (the paper's own kernel scheme) ----------------------
 * Section 3.5 and Appendix F describe the unified kernel as a one-bit lookup-table GEMM: every block is
 * decomposed into one-bit matrices (Appendix B, Eq. 10), put into +-1 form (s^ = s/2, W^_i = 2 W_i - 1,
 * z^ = z + (2^b - 1) s / 2), packed 8 input features to a byte, and multiplied through tables of the signed
 * sums of 8 activations held in on-chip memory, of which half is stored (mirror storage).  The three calls
 * below are that scheme for M = 1, as a measured alternative to sfmp_gemm (which contracts on the matrix cores):
 * the same operation Y = X[col_perm] . (s q + z)^T with the same bitmap, scale / zero arrays (fp16, group
 * length 128 only) and permutations, on its own weight format.
 *
 * Bit-plane format B1: tiles of 128 x 128 codes in row-major order of (tile row, tile column); a tile of width b
 * holds b planes, lowest bit first; a plane is 128 rows x 16 bytes (2048 bytes); bit t of byte (r, g) is bit i of
 * the code at row 128 tr + r, column 128 tc + 8 g + t.  tile_off[t], t = tr * (K/128) + tc, is the start of tile
 * t in planes (units of 2048 bytes); tile_off[ntiles] is the total, so a tile's width is tile_off[t+1] - tile_off[t].
 *
 * sfmp_lut_pack_query: sizes of the two arrays for a bitmap [N/128, K/128] (host).  SFMP_ERR_SHAPE,
 * SFMP_ERR_BITWIDTH as for sfmp_pack_query.
 * sfmp_lut_pack: codes [N, K] uint8 (host, row-major, reordered coordinates) -> planes_host (plane_bytes bytes),
 * tile_off_host (table_words uint32), both caller-allocated; SFMP_ERR_CODE_RANGE if a code does not fit its tile.
 * sfmp_lut_gemv_workspace / sfmp_lut_gemv: device pointers throughout; X fp16 [K], col_perm int32 [K] or NULL,
 * planes and tile_off as packed (uploaded unchanged), scales / zeros fp16 [K/128, N], row_perm int32 [N] or NULL,
 * Y fp16 [N] fully overwritten; workspace of at least the queried bytes, 256-byte aligned, contents irrelevant
 * on entry and unspecified on return (fp32 partial sums of the K ranges).  table_format: SFMP_LUT_TABLE_FP32, or
 * SFMP_LUT_TABLE_FP16 for the 2-byte table entries of Appendix F (each entry = the fp32 signed sum of its 8
 * activations rounded once to fp16: a relative error of up to 2^-11 per looked-up value; SFMP_ERR_LAYOUT for any other
 * value).  Accumulation in fp32 either way, one round-to-nearest-even conversion at the end; results repeat bit for
 * bit.  Asynchronous on hip_stream; two launches; no global state.  Errors as for sfmp_gemm. */
int sfmp_lut_pack_query(const int8_t* bitmap_host, int32_t N, int32_t K, int64_t* plane_bytes, int64_t* table_words);
int sfmp_lut_pack(const uint8_t* codes_host, const int8_t* bitmap_host, int32_t N, int32_t K, uint8_t* planes_host,
                  uint32_t* tile_off_host);
int sfmp_lut_gemv_workspace(int32_t N, int32_t K, int64_t* bytes);
int sfmp_lut_gemv(const void* X_dev, const int32_t* col_perm_dev, int32_t N, int32_t K, const void* planes_dev,
                  const uint32_t* tile_off_dev, const void* scales_dev, const void* zeros_dev,
                  const int32_t* row_perm_dev, void* Y_dev, int32_t table_format, void* workspace_dev,
                  int64_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SFMP_H */
