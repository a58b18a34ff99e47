"""CPU oracle for the SFMP block-wise mixed-precision GEMM / GEMV.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module: only
the tests, the smoke check and the CPU-baseline leg of the benchmark call it.  It shares
no code, table or constant generator with the HIP library; it is plain numpy, float64,
and deliberately slow and literal.

What it computes (paper: Fig. 3(c); Section 3.4 Eq. 8-9; Appendix B Eq. 10-11;
Section 4 "group quantization is applied along the n_b dimension within each block"):

    b        = bitmap[n // 128, k // 128]                      bit-width of the tile, in {2,3,4}
    w_hat    = s[k // G, n] * q[n, k] + z[k // G, n]          z is an additive real zero-point; G = group
                                                               length along K (128 by default; the ablation
                                                               "Effect of n_b" also uses 256 and 512), read off
                                                               the shape of s: G = K / s.shape[0]
    Xp[m, j] = X[m, col_perm[j]]                               the same permutation on the activation
    Yt       = Xp @ w_hat^T                                    float64
    Y[:, row_perm[i]] = Yt[:, i]                               undo the row reordering of the weight

The method reaches exactly this definition (its kernels are re-associations of the same
sum), so the oracle *is* the definition.  Pinned by tests/test_oracle_*.py: every function
here has at least one pin that does not go through itself.  Nothing is "parity unpinned".

The second half implements, independently and bit by bit from the written format
description (include/sfmp.h, "Packed format"), the packed byte format that the library's
packer emits, so that packed bytes and unpacked codes can be compared bit-exactly.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np

TILE = 128  # tile edge (rows of Wt = output features, columns = input features)
GROUP = 128  # default quantisation group length along K
WIDTHS = (2, 3, 4)


# ======================================================================================
# Part 1 - the arithmetic definition
# ======================================================================================
def bit_plane(codes: np.ndarray, i: int) -> np.ndarray:
    """One-bit matrix W_i of the integer codes: bit i (i = 0 is the lowest bit).

    Appendix B: a q-bit integer matrix is decomposed into q one-bit matrices,
    W_int = sum_i 2^i W_i (Eq. 10).
    """
    return ((codes.astype(np.int64) >> i) & 1).astype(np.uint8)


def codes_from_bit_planes(planes: Sequence[np.ndarray]) -> np.ndarray:
    """Inverse of ``bit_plane``: W_int = sum_i 2^i W_i (Appendix B, Eq. 10)."""
    acc = np.zeros(planes[0].shape, dtype=np.int64)
    for i, p in enumerate(planes):
        acc += p.astype(np.int64) << i
    return acc.astype(np.uint8)


def group_length(K: int, scales: np.ndarray) -> int:
    """Group length G along K implied by a scale array of shape [K/G, N]."""
    ng = scales.shape[0]
    assert ng > 0 and K % ng == 0, (K, scales.shape)
    return K // ng


def dequant(codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray) -> np.ndarray:
    """w_hat[n, k] = s[k // G, n] * q[n, k] + z[k // G, n]   (Appendix B, Eq. 11; group quantisation along
    the n_b dimension, Section 4 and the "Effect of n_b" ablation).

    codes uint8 [N, K]; scales, zeros [K/G, N] in any float type whose values are the stored parameters
    (fp16, or float32 holding bf16-representable numbers).  Returns float64 [N, K].
    """
    N, K = codes.shape
    G = group_length(K, scales)
    ng = K // G
    assert scales.shape == (ng, N) and zeros.shape == (ng, N)
    w_hat = np.empty((N, K), dtype=np.float64)
    for g in range(ng):
        s = scales[g].astype(np.float64)[:, None]  # one scale per row for this group
        z = zeros[g].astype(np.float64)[:, None]
        q = codes[:, g * G:(g + 1) * G].astype(np.float64)
        w_hat[:, g * G:(g + 1) * G] = s * q + z
    return w_hat


def permute_activation(X: np.ndarray, col_perm: Optional[np.ndarray]) -> np.ndarray:
    """Xp[m, j] = X[m, col_perm[j]] in float64 (Section 3.4: the weight's column
    permutation is applied to the activation at inference)."""
    Xd = X.astype(np.float64)
    if col_perm is None:
        return Xd
    return Xd[:, np.asarray(col_perm, dtype=np.int64)]


def gemm(X: np.ndarray, col_perm: Optional[np.ndarray], codes: np.ndarray, scales: np.ndarray,
         zeros: np.ndarray, row_perm: Optional[np.ndarray] = None) -> np.ndarray:
    """Y = X[:, col_perm] . dequant(codes)^T, rows optionally un-permuted.  float64 [M, N].

    With Wt = P_row W P_col (Eq. 9), Xp Wt^T = (X W^T) P_row^T, so output feature
    ``row_perm[i]`` of the un-reordered layer is column i of the product.
    """
    w_hat = dequant(codes, scales, zeros)
    Xp = permute_activation(X, col_perm)
    Yt = Xp @ w_hat.T
    if row_perm is None:
        return Yt
    Y = np.empty_like(Yt)
    Y[:, np.asarray(row_perm, dtype=np.int64)] = Yt
    return Y


def gemm_rows(X: np.ndarray, col_perm: Optional[np.ndarray], codes: np.ndarray, scales: np.ndarray,
              zeros: np.ndarray, rows: np.ndarray) -> np.ndarray:
    """Columns ``rows`` of the reordered product Yt (before any row un-permutation).

    The same definition as ``gemm`` evaluated only for the sampled output features, so that
    full-size layers can be checked one output at a time.  Returns float64 [M, len(rows)].
    """
    rows = np.asarray(rows, dtype=np.int64)
    w_hat = dequant_rows(codes, scales, zeros, rows)
    Xp = permute_activation(X, col_perm)
    return Xp @ w_hat.T


def dequant_rows(codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray, rows: np.ndarray) -> np.ndarray:
    """``dequant`` restricted to the given rows of Wt.  float64 [len(rows), K]."""
    rows = np.asarray(rows, dtype=np.int64)
    K = codes.shape[1]
    G = group_length(K, scales)
    q = codes[rows].astype(np.float64)
    s = np.repeat(scales[:, rows].astype(np.float64).T, G, axis=1)
    z = np.repeat(zeros[:, rows].astype(np.float64).T, G, axis=1)
    return s * q + z


def fold_perms(row_perm_prev: np.ndarray, col_perm_next: Optional[np.ndarray]) -> np.ndarray:
    """The column permutation that lets a matrix read the previous product while it is still in reordered row
    order (Section 3.4; the two reorder operations per layer whose overhead Section 4.2 measures collapse into one gather).

    Written from its defining property, by search: folded[j] is the position i at which the reordered product
    holds the feature that the plain gather would fetch, i.e. the i with row_perm_prev[i] == col_perm_next[j]."""
    r = np.asarray(row_perm_prev).astype(np.int64)
    n = r.size
    c = np.arange(n, dtype=np.int64) if col_perm_next is None else np.asarray(col_perm_next).astype(np.int64)
    out = np.empty(n, dtype=np.int32)
    for j in range(n):
        (hits,) = np.nonzero(r == c[j])
        assert hits.size == 1, "row_perm_prev is not a permutation"
        out[j] = hits[0]
    return out


def rel_frobenius(Y: np.ndarray, Y_ref: np.ndarray) -> float:
    """||Y - Y_ref||_F / ||Y_ref||_F in float64 (the acceptance measure for fp16 outputs)."""
    Yd = np.asarray(Y, dtype=np.float64)
    Rd = np.asarray(Y_ref, dtype=np.float64)
    den = float(np.linalg.norm(Rd))
    num = float(np.linalg.norm(Yd - Rd))
    return num / den if den > 0 else num


# ======================================================================================
# Part 2 - the packed byte format, written from its description
# ======================================================================================
# A tile is 128 rows x 128 columns of b-bit codes and occupies exactly 2048*b bytes: 8 "slabs"
# of 256*b bytes.  Inside a slab each of 64 "lanes" owns b consecutive little-endian 32-bit
# words: word w of lane l of slab sigma sits at byte offset sigma*256*b + l*4*b + 4*w.
#
# Element (r, c) of the tile (r = row in tile, c = column in tile) belongs to
#     lane   l     = 16 * ((c % 32) // 8) + r // 8
#     slab   sigma = r % 8
#     step   kappa = c // 32             (4 steps of 32 columns)
#     slot   v     = c % 8,  reg = v // 2,  half = v % 2  (half selects bits 0-15 / 16-31 of a word)
# and its bits are placed inside the lane's b words of that slab as follows:
#     b = 4: word reg,      bits [16*half + 4*kappa, +4)
#     b = 2: word reg % 2,  bits [16*half + 8*(reg // 2) + 2*kappa, +2)
#     b = 3: each 16-bit half of a word has five 3-bit fields j = 0..4 at bits [3j, 3j+3) and one
#            spare bit 15.  (kappa, reg) -> (word, field j) by the table below; the entry SPARE
#            spreads the code over the three spare bits: bit t of the code is bit 16*half + 15 of
#            word t.
#                kappa 0: (0,0) (1,0) (2,0) (0,3)
#                kappa 1: (0,1) (1,1) (2,1) (0,4)
#                kappa 2: (0,2) (1,2) (2,2) SPARE
#                kappa 3: (1,3) (2,3) (1,4) (2,4)
_SPARE = None
_FIELD3 = (
    ((0, 0), (1, 0), (2, 0), (0, 3)),
    ((0, 1), (1, 1), (2, 1), (0, 4)),
    ((0, 2), (1, 2), (2, 2), _SPARE),
    ((1, 3), (2, 3), (1, 4), (2, 4)),
)


def tile_bytes(b: int) -> int:
    return 2048 * b


def code_bit_position(b: int, r: int, c: int, t: int) -> int:
    """Absolute bit index, inside the tile's byte string, of bit t of the code at (r, c).

    Bit index x means bit (x % 8) of byte (x // 8); words are little-endian, so bit j of the
    32-bit word at byte offset o is bit index 8*o + j.
    """
    assert b in WIDTHS and 0 <= r < TILE and 0 <= c < TILE and 0 <= t < b
    lane = 16 * ((c % 32) // 8) + r // 8
    slab = r % 8
    kappa = c // 32
    v = c % 8
    reg, half = v // 2, v % 2
    if b == 4:
        word, bit = reg, 16 * half + 4 * kappa + t
    elif b == 2:
        word, bit = reg % 2, 16 * half + 8 * (reg // 2) + 2 * kappa + t
    else:
        entry = _FIELD3[kappa][reg]
        if entry is _SPARE:
            word, bit = t, 16 * half + 15
        else:
            word, bit = entry[0], 16 * half + 3 * entry[1] + t
    byte_off = slab * 256 * b + lane * 4 * b + 4 * word
    return 8 * byte_off + bit


_POS_CACHE: Dict[int, np.ndarray] = {}


def tile_bit_positions(b: int) -> np.ndarray:
    """int64 [128, 128, b]: ``code_bit_position`` for every element and bit of a width-b tile."""
    if b not in _POS_CACHE:
        pos = np.empty((TILE, TILE, b), dtype=np.int64)
        for r in range(TILE):
            for c in range(TILE):
                for t in range(b):
                    pos[r, c, t] = code_bit_position(b, r, c, t)
        _POS_CACHE[b] = pos
    return _POS_CACHE[b]


def pack_tile(tile_codes: np.ndarray, b: int) -> np.ndarray:
    """uint8 [2048*b]: one tile's codes (uint8 [128,128], all < 2^b) in the packed format."""
    assert tile_codes.shape == (TILE, TILE)
    if int(tile_codes.max(initial=0)) >= (1 << b):
        raise ValueError("code out of range for the tile's bit-width")
    pos = tile_bit_positions(b)
    bits = np.zeros(tile_bytes(b) * 8, dtype=np.uint8)
    for t in range(b):
        bits[pos[:, :, t].ravel()] = bit_plane(tile_codes, t).ravel()
    return np.packbits(bits, bitorder="little")


def unpack_tile(tile: np.ndarray, b: int) -> np.ndarray:
    """uint8 [128,128]: the codes stored in one packed tile (uint8 [2048*b])."""
    assert tile.shape == (tile_bytes(b),)
    pos = tile_bit_positions(b)
    bits = np.unpackbits(tile, bitorder="little")
    planes = [bits[pos[:, :, t].ravel()].reshape(TILE, TILE) for t in range(b)]
    return codes_from_bit_planes(planes)


def index_words(ntr: int, ntc: int) -> int:
    """Length, in int32 words, of the block-index table of an ntr x ntc tile grid."""
    nt = ntr * ntc
    return 3 + nt + 3 * (ntr + 1) + nt


def build_index(bitmap: np.ndarray) -> np.ndarray:
    """Block-index table (int32) for a bitmap, written from the format description.

    words [0,3)            number of tiles of width 2, 3, 4
    words [3, 3+nt)        tile_desc[tr*ntc + tc] = (slot << 2) | (b - 2); slot = rank of the tile among
                           the tiles of its width in ascending (tr, tc) order = its position in that stream
    then, for b = 2,3,4    row_ptr_b[ntr + 1]  (CSR over tile rows, counting tiles of width b)
    then, for b = 2,3,4    col_idx_b[count_b]  (tile column of every width-b tile, stream order)
    """
    ntr, ntc = bitmap.shape
    nt = ntr * ntc
    idx = np.zeros(index_words(ntr, ntc), dtype=np.int32)
    counts = {b: 0 for b in WIDTHS}
    row_ptr = {b: [0] for b in WIDTHS}
    col_idx = {b: [] for b in WIDTHS}
    for tr in range(ntr):
        for tc in range(ntc):
            b = int(bitmap[tr, tc])
            if b not in WIDTHS:
                raise ValueError("bit-width must be 2, 3 or 4")
            idx[3 + tr * ntc + tc] = (counts[b] << 2) | (b - 2)
            counts[b] += 1
            col_idx[b].append(tc)
        for b in WIDTHS:
            row_ptr[b].append(counts[b])
    idx[0:3] = [counts[2], counts[3], counts[4]]
    o = 3 + nt
    for b in WIDTHS:
        idx[o:o + ntr + 1] = row_ptr[b]
        o += ntr + 1
    for b in WIDTHS:
        idx[o:o + counts[b]] = col_idx[b]
        o += counts[b]
    assert o == idx.size
    return idx


def pack(codes: np.ndarray, bitmap: np.ndarray) -> Dict[str, np.ndarray]:
    """Pack a whole code matrix: three per-width tile streams + the block-index table.

    Stream S_b holds the tiles of width b in ascending (tile row, tile column) order, each
    tile as ``pack_tile`` writes it.  Returns {"s2","s3","s4": uint8 arrays, "index": int32}.
    """
    N, K = codes.shape
    ntr, ntc = N // TILE, K // TILE
    assert bitmap.shape == (ntr, ntc)
    index = build_index(bitmap)
    streams = {b: np.zeros(int(index[b - 2]) * tile_bytes(b), dtype=np.uint8) for b in WIDTHS}
    for tr in range(ntr):
        for tc in range(ntc):
            desc = int(index[3 + tr * ntc + tc])
            b, slot = (desc & 3) + 2, desc >> 2
            tile = codes[tr * TILE:(tr + 1) * TILE, tc * TILE:(tc + 1) * TILE]
            streams[b][slot * tile_bytes(b):(slot + 1) * tile_bytes(b)] = pack_tile(tile, b)
    return {"s2": streams[2], "s3": streams[3], "s4": streams[4], "index": index}


def unpack(N: int, K: int, s2: np.ndarray, s3: np.ndarray, s4: np.ndarray, index: np.ndarray) -> np.ndarray:
    """Inverse of ``pack``: uint8 [N, K] codes from the three streams and the index table."""
    ntr, ntc = N // TILE, K // TILE
    streams = {2: s2, 3: s3, 4: s4}
    codes = np.empty((N, K), dtype=np.uint8)
    for tr in range(ntr):
        for tc in range(ntc):
            desc = int(index[3 + tr * ntc + tc])
            b, slot = (desc & 3) + 2, desc >> 2
            tile = streams[b][slot * tile_bytes(b):(slot + 1) * tile_bytes(b)]
            codes[tr * TILE:(tr + 1) * TILE, tc * TILE:(tc + 1) * TILE] = unpack_tile(tile, b)
    return codes


def gemm_packed(X, col_perm, N, K, s2, s3, s4, index, scales, zeros, row_perm=None) -> np.ndarray:
    """``gemm`` on packed weights: unpack with this module's own ``unpack``, then the definition."""
    return gemm(X, col_perm, unpack(N, K, s2, s3, s4, index), scales, zeros, row_perm)
