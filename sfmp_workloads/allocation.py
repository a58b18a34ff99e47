"""The offline side of the method on synthetic salience: reordering and block-wise bit allocation.

Inputs only: this module produces the bitmaps and permutations that the GEMM consumes, so that benches and
tests can run on bitmaps with the structure the method creates (high-salience rows and columns first, wide
tiles clustered in the top-left corner) instead of shuffled ones.  Nothing here runs on the GPU.

Paper: Section 3.2 (objective sum_i F_ii / (2^{b_i} - 1)^2 under an average-bit budget; Case 1: two widths,
sort and split; Case 2 / Algorithm 1: three widths, one-dimensional grid over the share of the lowest width),
Section 3.3 (blocks of m_b x n_b weights as the allocation unit, block salience = sum of its F_ii),
Section 3.4 (row / column salience = sums of F_ii over a row / column, permutations = descending argsort).
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence, Tuple

import numpy as np

TILE = 128


def synthetic_salience(N: int, K: int, rng: np.random.Generator, row_sigma: float = 1.0, col_sigma: float = 1.5,
                       noise_sigma: float = 0.5) -> np.ndarray:
    """A positive [N, K] map with strong row and column structure (a stand-in for the Fisher diagonal, whose
    values the paper shows to be organised along rows and columns): log-normal row factor x log-normal column
    factor x log-normal noise.  float32."""
    r = np.exp(row_sigma * rng.standard_normal(N)).astype(np.float32)
    c = np.exp(col_sigma * rng.standard_normal(K)).astype(np.float32)
    F = np.exp(noise_sigma * rng.standard_normal((N, K)).astype(np.float32))
    F *= r[:, None]
    F *= c[None, :]
    return F


def reorder(F: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(row_perm, col_perm) that sort rows and columns by aggregated salience, largest first (Section 3.4).

    Convention of this code base: the reordered matrix is ``Wt[i, j] = W[row_perm[i], col_perm[j]]``.
    Ties keep their original order (stable sort)."""
    s_row = F.sum(axis=1, dtype=np.float64)
    s_col = F.sum(axis=0, dtype=np.float64)
    row_perm = np.argsort(-s_row, kind="stable").astype(np.int32)
    col_perm = np.argsort(-s_col, kind="stable").astype(np.int32)
    return row_perm, col_perm


def block_salience(Ft: np.ndarray, mb: int, nb: int) -> np.ndarray:
    """Sum of the (reordered) salience over every mb x nb block (Section 3.3).  float64 [N/mb, K/nb]."""
    N, K = Ft.shape
    assert N % mb == 0 and K % nb == 0
    return Ft.reshape(N // mb, mb, K // nb, nb).sum(axis=(1, 3), dtype=np.float64)


def allocation_loss(sal: np.ndarray, bits: np.ndarray) -> float:
    """sum_j F_j / (2^{b_j} - 1)^2, the bit-allocation objective."""
    return float((sal.astype(np.float64) / (2.0 ** bits.astype(np.float64) - 1.0) ** 2).sum())


def allocate_two(sal: np.ndarray, widths: Sequence[int], target: float) -> np.ndarray:
    """Case 1: two widths b1 < b2.  The shares are fixed by the budget; the floor(alpha_1 n) units of lowest
    salience get b1, the rest b2.  Returns the width of every unit (same shape as ``sal``)."""
    b1, b2 = widths
    assert b1 < b2 and b1 <= target <= b2
    flat = sal.ravel()
    n = flat.size
    alpha1 = (b2 - target) / (b2 - b1)
    n1 = int(np.floor(alpha1 * n + 1e-9))
    order = np.argsort(flat, kind="stable")
    out = np.full(n, b2, dtype=np.int8)
    out[order[:n1]] = b1
    return out.reshape(sal.shape)


def allocate_three(sal: np.ndarray, widths: Sequence[int], target: float, step: float = 0.01) -> np.ndarray:
    """Case 2 (Algorithm 1): three widths b1 < b2 < b3.  For every share alpha_1 of the lowest width on a grid of
    the given step, the budget fixes alpha_2 and alpha_3; units sorted by ascending salience receive b1, b2, b3
    in that order with n_k = floor(alpha_k n) (the remainder goes to b3); the assignment of least loss wins."""
    b1, b2, b3 = widths
    assert b1 < b2 < b3 and b1 <= target <= b3
    flat = sal.ravel().astype(np.float64)
    n = flat.size
    order = np.argsort(flat, kind="stable")
    sorted_sal = flat[order]
    prefix = np.concatenate([[0.0], np.cumsum(sorted_sal)])
    w = [1.0 / (2.0 ** b - 1.0) ** 2 for b in (b1, b2, b3)]
    best = None
    steps = int(round(1.0 / step))
    for i in range(steps + 1):
        alpha1 = i * step
        alpha2 = (target - b3 - (b1 - b3) * alpha1) / (b2 - b3)
        alpha3 = 1.0 - alpha1 - alpha2
        if alpha2 < -1e-12 or alpha3 < -1e-12:
            continue
        n1 = int(np.floor(alpha1 * n + 1e-9))
        n2 = int(np.floor(max(alpha2, 0.0) * n + 1e-9))
        if n1 + n2 > n:
            continue
        loss = w[0] * prefix[n1] + w[1] * (prefix[n1 + n2] - prefix[n1]) + w[2] * (prefix[n] - prefix[n1 + n2])
        if best is None or loss < best[0]:
            best = (loss, n1, n2)
    assert best is not None, "the target is outside the range of the candidate widths"
    _, n1, n2 = best
    out = np.full(n, b3, dtype=np.int8)
    out[order[:n1]] = b1
    out[order[n1:n1 + n2]] = b2
    return out.reshape(sal.shape)


def allocated_layout(N: int, K: int, target: float, rng: np.random.Generator, widths: Sequence[int] = (2, 3, 4),
                     block: Tuple[int, int] = (4, 1), step: float = 0.01,
                     F: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Salience -> permutations -> block salience -> widths -> tile bitmap, for one [N, K] matrix.

    ``block`` = (rows, columns) of an allocation block in 128x128 tiles ((4, 1) = the paper's (512, 128)).
    Returns dict(bitmap int8 [N/128, K/128], row_perm, col_perm int32, block_bits int8)."""
    if F is None:
        F = synthetic_salience(N, K, rng)
    row_perm, col_perm = reorder(F)
    Ft = F[row_perm][:, col_perm]
    sal = block_salience(Ft, TILE * block[0], TILE * block[1])
    bits = allocate_two(sal, widths, target) if len(widths) == 2 else allocate_three(sal, widths, target, step)
    bitmap = np.repeat(np.repeat(bits, block[0], axis=0), block[1], axis=1).astype(np.int8)
    return dict(bitmap=bitmap, row_perm=row_perm, col_perm=col_perm, block_bits=bits)
