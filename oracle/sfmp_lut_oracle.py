"""CPU oracle for the one-bit lookup-table GEMV (the paper's own kernel scheme, Appendix B and Appendix F).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module: only the tests, the
smoke check and the benchmark's CPU leg call it.  It shares no code, table or constant generator
with the HIP library; plain numpy, float64, deliberately slow and literal.

What it computes, in the paper's order and notation (Appendix B, Eq. 10-13; Appendix F):

  1. the b-bit codes of a block are decomposed into b one-bit matrices W_i in {0,1} (Eq. 10);
  2. the linear change of variables  s^ = s/2,  W^_i = 2 W_i - 1,  z^ = z + (1/2) sum_i 2^i s
     turns  w = sum_i 2^i s W_i + z  into  w = sum_i 2^i s^ W^_i + z^  with W^_i in {-1,+1};
  3. the activations are taken 8 at a time; for every group of 8 a table of the 256 signed sums
     sum_t (+-) x_t is needed, of which only 128 are built (those whose top sign is minus): the
     other half is the negation of a stored entry (mirror storage);
  4. a packed byte of W_i (8 consecutive input features of one output feature) indexes the table;
     the looked-up values are added over the groups, weighted by 2^i over the bit planes, scaled
     by s^ per quantisation group, and z^ times the sum of the group's activations is added.

The result equals the plain definition  y = (x[col_perm]) . (s q + z)^T  (that identity is what
pins this module: tests/test_lut_oracle.py compares it with the definition written out separately,
and with a brute-force enumeration of the table).  Nothing here is "parity unpinned".

The bit-plane byte format ("format B1") is described in include/sfmp.h; this module implements it
independently, from that description:

  tiles of 128 x 128 codes in row-major order of (tile row, tile column); a tile of width b holds
  b planes, lowest bit first; a plane is 128 rows x 16 bytes; bit t of byte (r, g) is bit i of the
  code at row 128 tr + r, column 128 tc + 8 g + t.  tile_off[t] is the start of tile t in units
  of 2048 bytes (one plane), tile_off[ntiles] the total.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

TILE = 128
GROUP = 128
PLANE_BYTES = TILE * TILE // 8  # 2048


def lut_pack(codes: np.ndarray, bitmap: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """codes [N, K] uint8, bitmap [N/128, K/128] -> (plane bytes uint8 [total], tile_off uint32 [ntiles + 1])."""
    N, K = codes.shape
    ntr, ntc = N // TILE, K // TILE
    tile_off = np.zeros(ntr * ntc + 1, dtype=np.uint32)
    chunks = []
    for tr in range(ntr):
        for tc in range(ntc):
            b = int(bitmap[tr, tc])
            tile = codes[tr * TILE:(tr + 1) * TILE, tc * TILE:(tc + 1) * TILE].astype(np.uint8)
            for i in range(b):
                bits = (tile >> i) & 1                                   # W_i of this tile, [128, 128]
                grouped = bits.reshape(TILE, TILE // 8, 8)               # [row, group of 8 columns, t]
                weights = (1 << np.arange(8)).astype(np.uint16)          # bit t of the byte <- column 8g + t
                chunks.append((grouped * weights).sum(axis=2).astype(np.uint8).reshape(-1))
            tile_off[tr * ntc + tc + 1] = tile_off[tr * ntc + tc] + b
    planes = np.concatenate(chunks) if chunks else np.zeros(0, dtype=np.uint8)
    return planes, tile_off


def lut_unpack(N: int, K: int, planes: np.ndarray, tile_off: np.ndarray) -> np.ndarray:
    """Inverse of lut_pack: the codes [N, K] (the width of a tile is tile_off[t+1] - tile_off[t])."""
    ntr, ntc = N // TILE, K // TILE
    codes = np.zeros((N, K), dtype=np.uint8)
    for tr in range(ntr):
        for tc in range(ntc):
            t = tr * ntc + tc
            b = int(tile_off[t + 1]) - int(tile_off[t])
            acc = np.zeros((TILE, TILE), dtype=np.uint8)
            for i in range(b):
                start = (int(tile_off[t]) + i) * PLANE_BYTES
                plane = planes[start:start + PLANE_BYTES].reshape(TILE, TILE // 8)
                bits = (plane[:, :, None] >> np.arange(8)) & 1            # [row, group, t]
                acc |= (bits.reshape(TILE, TILE).astype(np.uint8) << i)
            codes[tr * TILE:(tr + 1) * TILE, tc * TILE:(tc + 1) * TILE] = acc
    return codes


def half_table(x8: np.ndarray) -> np.ndarray:
    """The 128 stored entries of the table of one group of 8 activations (Appendix B, mirror storage):
    entry p (0 <= p < 128) = sum_t sign_t(p) x_t with sign_t = +1 if bit t of p is set, else -1; bit 7 of p is 0,
    so x_7 always enters with a minus sign."""
    x8 = np.asarray(x8, dtype=np.float64)
    table = np.zeros(128, dtype=np.float64)
    for p in range(128):
        acc = 0.0
        for t in range(8):
            acc += x8[t] if (p >> t) & 1 else -x8[t]
        table[p] = acc
    return table


def table_lookup(table: np.ndarray, byte: np.ndarray) -> np.ndarray:
    """Value of the full 256-entry table at `byte`, from the stored half: an index with bit 7 set is the negation
    of the entry at the complemented index."""
    byte = byte.astype(np.int64)
    high = byte >= 128
    idx = np.where(high, 255 - byte, byte)
    val = table[idx]
    return np.where(high, -val, val)


def lut_gemv(x: np.ndarray, col_perm: Optional[np.ndarray], N: int, K: int, planes: np.ndarray,
             tile_off: np.ndarray, scales: np.ndarray, zeros: np.ndarray,
             row_perm: Optional[np.ndarray] = None, table_dtype=None) -> np.ndarray:
    """y [N] float64 from the bit-plane format, by table lookups (steps 1-4 of the module header).

    x [K]; col_perm [K] or None; scales, zeros [K/128, N] (group length 128); row_perm [N] or None.
    table_dtype=np.float16: the table entries are rounded to fp16 before they are looked up (the 2-byte entries of
    Appendix F; every activation then enters the result through a rounded entry, the sum of a column's activations
    included: it is minus the sum of the entries whose signs are all negative); everything else stays float64."""
    ntr, ntc = N // TILE, K // TILE
    xp = np.asarray(x, dtype=np.float64).reshape(-1)
    if col_perm is not None:
        xp = xp[np.asarray(col_perm, dtype=np.int64)]
    s = np.asarray(scales, dtype=np.float64)
    z = np.asarray(zeros, dtype=np.float64)
    yt = np.zeros(N, dtype=np.float64)
    for tc in range(ntc):
        xs = xp[tc * TILE:(tc + 1) * TILE]
        tables = [half_table(xs[8 * g:8 * g + 8]) for g in range(TILE // 8)]
        sum_x = xs.sum()
        if table_dtype is not None:
            tables = [tb.astype(table_dtype).astype(np.float64) for tb in tables]
            sum_x = -sum(tb[0] for tb in tables)
        for tr in range(ntr):
            t = tr * ntc + tc
            b = int(tile_off[t + 1]) - int(tile_off[t])
            rows = slice(tr * TILE, (tr + 1) * TILE)
            s_hat = s[tc, rows] / 2.0
            z_hat = z[tc, rows] + 0.5 * sum((2.0 ** i) for i in range(b)) * s[tc, rows]
            acc = np.zeros(TILE, dtype=np.float64)
            for i in range(b):
                start = (int(tile_off[t]) + i) * PLANE_BYTES
                plane = planes[start:start + PLANE_BYTES].reshape(TILE, TILE // 8)
                one_bit = np.zeros(TILE, dtype=np.float64)               # x . W^_i for the 128 rows
                for g in range(TILE // 8):
                    one_bit += table_lookup(tables[g], plane[:, g])
                acc += (2.0 ** i) * one_bit
            yt[rows] += s_hat * acc + z_hat * sum_x
    if row_perm is None:
        return yt
    y = np.zeros(N, dtype=np.float64)
    y[np.asarray(row_perm, dtype=np.int64)] = yt
    return y
