"""Seeded generators for SFMP GEMM/GEMV test and bench inputs (inputs only).

Conventions (they follow the paper's Section 3.4, Eq. 8-9, with the reading
that a weight matrix is stored [N, K] = [output features, input features]):

* ``W``        original-coordinate weight, fp16 ``[N, K]``.
* ``row_perm`` int32 ``[N]``, ``col_perm`` int32 ``[K]``: the reordered weight is
  ``Wt[i, j] = W[row_perm[i], col_perm[j]]``.
* ``bitmap``   int8 ``[N/128, K/128]`` holding the literal bit-width 2, 3 or 4 of
  every 128x128 tile of ``Wt`` (Section 3.3 block-wise allocation; one int8
  per block as in the "Extra Metadata" paragraph of Section 4.2).
* ``codes``    uint8 ``[N, K]`` integer codes of ``Wt``; ``scales`` / ``zeros``
  ``[K/G, N]``: one (s, z) pair per row per group of G reordered columns (G = 128 by
  default; 64, 256 and 512 as in the paper's ablation of the block width n_b, which is also its
  group size), stored as fp16, or as bf16 (the paper's storage type) held in float32 arrays.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Iterator, List, Optional, Sequence, Tuple

import numpy as np

TILE = 128
GROUP = 128

# (K, N) = (in features, out features) of the seven projections of one layer.
SHAPES_8B: Dict[str, Tuple[int, int]] = {
    "q": (4096, 4096),
    "k": (4096, 1024),
    "v": (4096, 1024),
    "o": (4096, 4096),
    "gate": (4096, 14336),
    "up": (4096, 14336),
    "down": (14336, 4096),
}
SHAPES_70B: Dict[str, Tuple[int, int]] = {
    "q": (8192, 8192),
    "k": (8192, 1024),
    "v": (8192, 1024),
    "o": (8192, 8192),
    "gate": (8192, 28672),
    "up": (8192, 28672),
    "down": (28672, 8192),
}
LAYER_8B: List[str] = ["q", "k", "v", "o", "gate", "up", "down"]
LAYER_70B: List[str] = ["q", "k", "v", "o", "gate", "up", "down"]


@dataclass(frozen=True)
class ConfigSpec:
    """One of the five benchmark configurations."""

    cid: int
    name: str
    shapes: Tuple[Tuple[str, int, int], ...]  # (label, K, N)
    Ms: Tuple[int, ...]
    w_std: Tuple[float, ...]  # one per shape
    fractions: Optional[Dict[int, float]]  # width -> fraction; None = i.i.d. uniform
    outliers: bool
    row_perm: Tuple[bool, ...]  # one per shape
    col_perm: bool = True


def _layer(shapes: Dict[str, Tuple[int, int]], prefix: str):
    return tuple((f"{prefix}.{n}", shapes[n][0], shapes[n][1]) for n in LAYER_8B)


_PREFILL_SHAPES = (
    ("8b.q", 4096, 4096),
    ("8b.k", 4096, 1024),
    ("8b.gate", 4096, 14336),
    ("8b.down", 14336, 4096),
    ("70b.gate", 8192, 28672),
    ("70b.down", 28672, 8192),
)

CONFIGS: Dict[int, ConfigSpec] = {
    1: ConfigSpec(1, "tiny", (("tiny", 512, 512),), (1,), (0.02,), None, False, (False,)),
    2: ConfigSpec(2, "8b-decode-3.0b", _layer(SHAPES_8B, "8b"), (1,), (0.02,) * 7,
                  {2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, False, (True,) * 7),
    3: ConfigSpec(3, "8b-fractional-2.5b", _layer(SHAPES_8B, "8b"), (1, 4, 16, 64), (0.02,) * 7,
                  {2: 0.5, 3: 0.5}, True, (True,) * 7),
    4: ConfigSpec(4, "70b-decode-3.25b", _layer(SHAPES_70B, "70b"), (1, 8), (0.015,) * 7,
                  {2: 0.25, 3: 0.25, 4: 0.5}, False, (True,) * 7),
    5: ConfigSpec(5, "prefill-3.5b", _PREFILL_SHAPES, (2048,), (0.02, 0.02, 0.02, 0.02, 0.015, 0.015),
                  {3: 0.5, 4: 0.5}, True, (True, True, True, True, False, False)),
}


# --------------------------------------------------------------------------------------
# elementary generators
# --------------------------------------------------------------------------------------
def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def _rng_x(seed: int, M: int) -> np.random.Generator:
    """Activations come from their own stream, so problems that differ only in M share weights."""
    return np.random.Generator(np.random.PCG64([int(seed), int(M), 0x5F3]))


def make_bitmap(ntr: int, ntc: int, fractions: Optional[Dict[int, float]], rng: np.random.Generator) -> np.ndarray:
    """Bit-width of every tile.

    ``fractions`` None: i.i.d. uniform over {2,3,4}.  Otherwise exact counts
    ``floor(f_b * nt)`` per width; the few remainder tiles get the middle width of
    the set (the lower one for a two-width mix); a seeded shuffle places them.
    """
    nt = ntr * ntc
    if fractions is None:
        return rng.integers(2, 5, size=(ntr, ntc)).astype(np.int8)
    widths = sorted(fractions)
    counts = {b: int(np.floor(fractions[b] * nt + 1e-9)) for b in widths}
    rest = nt - sum(counts.values())
    filler = widths[(len(widths) - 1) // 2]
    counts[filler] += rest
    flat = np.concatenate([np.full(counts[b], b, dtype=np.int8) for b in widths])
    rng.shuffle(flat)
    return flat.reshape(ntr, ntc)


def block_bitmap(ntr: int, ntc: int, fractions: Optional[Dict[int, float]], rng: np.random.Generator,
                 mb_tiles: int = 4, nb_tiles: int = 1) -> np.ndarray:
    """A bitmap whose widths are constant on blocks of (128*mb_tiles) x (128*nb_tiles) weights.

    The paper allocates bit-widths per (m_b, n_b) block, (512, 128) in its experiments; a block is
    a run of equal-width 128x128 tiles.  ``ntr`` and ``ntc`` must be multiples of the block.
    """
    assert ntr % mb_tiles == 0 and ntc % nb_tiles == 0
    coarse = make_bitmap(ntr // mb_tiles, ntc // nb_tiles, fractions, rng)
    return np.repeat(np.repeat(coarse, mb_tiles, axis=0), nb_tiles, axis=1).astype(np.int8)


def to_bf16(x: np.ndarray) -> np.ndarray:
    """Rounds to the nearest bf16 value (ties to even); returns float32 holding those values."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) >> 16
    return (bits.astype(np.uint32) << 16).view(np.float32).reshape(np.shape(x))


def param_bits(a: np.ndarray) -> np.ndarray:
    """The 16 stored bits of every scale / zero: fp16 arrays as they are, bf16-in-float32 arrays by their top half."""
    if a.dtype == np.float16:
        return np.ascontiguousarray(a).view(np.uint16)
    assert a.dtype == np.float32
    return (np.ascontiguousarray(a).view(np.uint32) >> 16).astype(np.uint16)


def _store(x: np.ndarray, scale_format: str) -> np.ndarray:
    if scale_format == "fp16":
        return x.astype(np.float16)
    assert scale_format == "bf16"
    return to_bf16(x.astype(np.float32))


def _group_widths(bitmap: np.ndarray, group: int) -> np.ndarray:
    """Width of every (tile row, group): all tiles under a group must agree; a group shorter than a tile (64)
    has the width of the tile that holds it."""
    if group < TILE:
        assert TILE % group == 0
        return np.repeat(bitmap, TILE // group, axis=1)
    tpg = group // TILE
    assert group % TILE == 0 and bitmap.shape[1] % tpg == 0
    bg = bitmap.reshape(bitmap.shape[0], bitmap.shape[1] // tpg, tpg)
    assert (bg == bg[:, :, :1]).all(), "tiles that share a quantisation group must have one width"
    return bg[:, :, 0]


def clustered_bitmap(ntr: int, ntc: int, fractions: Dict[int, float]) -> np.ndarray:
    """Widths sorted so that the widest tiles sit in the top-left corner.

    This mimics what a salience-sorted row/column reordering (Section 3.4) produces:
    high-salience rows and columns come first and receive the larger bit-widths.
    """
    nt = ntr * ntc
    widths = sorted(fractions, reverse=True)
    counts = [int(np.floor(fractions[b] * nt + 1e-9)) for b in widths]
    counts[-1] += nt - sum(counts)
    order = np.argsort((np.arange(ntr)[:, None] / ntr + np.arange(ntc)[None, :] / ntc).ravel(), kind="stable")
    flat = np.empty(nt, dtype=np.int8)
    pos = 0
    for b, c in zip(widths, counts):
        flat[order[pos:pos + c]] = b
        pos += c
    return flat.reshape(ntr, ntc)


def make_weights(N: int, K: int, std: float, rng: np.random.Generator) -> np.ndarray:
    return (rng.standard_normal((N, K), dtype=np.float32) * np.float32(std)).astype(np.float16)


def make_activations(M: int, K: int, rng: np.random.Generator, outliers: bool = False,
                     outlier_frac: float = 0.01, outlier_scale: float = 20.0) -> np.ndarray:
    x = rng.standard_normal((M, K), dtype=np.float32)
    if outliers:
        n_out = int(np.floor(outlier_frac * K))
        cols = rng.choice(K, size=n_out, replace=False)
        x[:, cols] *= np.float32(outlier_scale)
    return x.astype(np.float16)


def make_perm(n: int, rng: np.random.Generator) -> np.ndarray:
    return rng.permutation(n).astype(np.int32)


# --------------------------------------------------------------------------------------
# test-data quantiser (harness only; both the oracle and the HIP path consume its output)
# --------------------------------------------------------------------------------------
def quantize_minmax(Wt: np.ndarray, bitmap: np.ndarray, group: int = GROUP,
                    scale_format: str = "fp16") -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Asymmetric min-max group quantisation of the reordered weight ``Wt`` [N, K].

    Per row n and per group g of ``group`` consecutive reordered columns, at the width b of
    the tiles that hold the group: step ``s = store((max - min) / (2^b - 1))`` (the
    uniform-quantiser step of the paper's Eq. 5), ``z = store(min)`` and
    ``q = clip(rint((w - z) / s), 0, 2^b - 1)`` evaluated in float64 with the
    stored (fp16- or bf16-rounded) s and z.  A group whose step rounds to zero gets ``s = 1, q = 0``.
    Returns (codes uint8 [N,K], scales [K/group,N], zeros [K/group,N]).
    """
    N, K = Wt.shape
    assert N % TILE == 0 and K % group == 0
    ng = K // group
    gw = _group_widths(bitmap, group)
    sdt = np.float16 if scale_format == "fp16" else np.float32
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((ng, N), dtype=sdt)
    zeros = np.empty((ng, N), dtype=sdt)
    rows_per_step = TILE * max(1, (1 << 22) // (K * TILE) or 1)
    for r0 in range(0, N, rows_per_step):
        r1 = min(N, r0 + rows_per_step)
        w = Wt[r0:r1].astype(np.float64).reshape(r1 - r0, ng, group)
        b = np.repeat(gw[r0 // TILE:(r1 + TILE - 1) // TILE].astype(np.int64), TILE, axis=0)[: r1 - r0]
        levels = (2.0 ** b - 1.0)  # [rows, ng]
        lo = w.min(axis=2)
        hi = w.max(axis=2)
        s16 = _store((hi - lo) / levels, scale_format)
        z16 = _store(lo, scale_format)
        degenerate = (s16 == 0) | ~np.isfinite(s16)
        s16 = np.where(degenerate, sdt(1.0), s16)
        s = s16.astype(np.float64)[:, :, None]
        z = z16.astype(np.float64)[:, :, None]
        q = np.clip(np.rint((w - z) / s), 0.0, levels[:, :, None])
        q = np.where(degenerate[:, :, None], 0.0, q)
        codes[r0:r1] = q.reshape(r1 - r0, K).astype(np.uint8)
        scales[:, r0:r1] = s16.T
        zeros[:, r0:r1] = z16.T
    return codes, scales, zeros


def random_quantized(N: int, K: int, bitmap: np.ndarray, std: float, rng: np.random.Generator,
                     group: int = GROUP, scale_format: str = "fp16") -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Codes / scales / zeros with the value ranges of ``quantize_minmax`` but drawn directly.

    Used only where building and quantising a float weight would dominate the run
    (timing loops); codes are uniform in [0, 2^b), the group range is about 5 sigma.
    """
    ng = K // group
    gw = _group_widths(bitmap, group)
    bm = np.repeat(np.repeat(bitmap.astype(np.uint8), TILE, axis=0), TILE, axis=1)
    raw = rng.integers(0, 256, size=(N, K), dtype=np.uint8)
    codes = (raw & ((np.uint8(1) << bm) - np.uint8(1))).astype(np.uint8)
    span = (5.0 * std) * (1.0 + 0.1 * rng.standard_normal((ng, N)))
    lv = (2.0 ** np.repeat(gw.astype(np.float64), TILE, axis=0).T - 1.0)  # [ng, N]
    scales = _store(span / lv, scale_format)
    zeros = _store(-0.5 * span * (1.0 + 0.05 * rng.standard_normal((ng, N))), scale_format)
    return codes, scales, zeros


# --------------------------------------------------------------------------------------
# whole problems
# --------------------------------------------------------------------------------------
@dataclass
class Problem:
    """Everything one ``Y = X[:, col_perm] . dequant(Wq)^T`` call consumes."""

    label: str
    N: int
    K: int
    M: int
    X: np.ndarray  # fp16 [M, K], original column order
    bitmap: np.ndarray  # int8 [N/128, K/128]
    codes: np.ndarray  # uint8 [N, K], reordered coordinates
    scales: np.ndarray  # [K/group, N]: fp16, or float32 holding bf16 values
    zeros: np.ndarray  # same
    col_perm: Optional[np.ndarray]  # int32 [K] or None (identity)
    row_perm: Optional[np.ndarray]  # int32 [N] or None (leave rows reordered)
    W: Optional[np.ndarray] = None  # fp16 [N, K] original coordinates, if materialised
    Wt: Optional[np.ndarray] = None  # fp16 [N, K] reordered, if kept
    seed: int = 0
    meta: dict = field(default_factory=dict)
    group: int = GROUP  # quantisation group length along K (64, 128, 256 or 512)
    scale_format: str = "fp16"  # storage type of scales and zeros: "fp16" or "bf16"

    @property
    def avg_bits(self) -> float:
        return float(self.bitmap.astype(np.float64).mean())


def make_problem(label: str, K: int, N: int, M: int, seed: int, *, w_std: float = 0.02,
                 fractions: Optional[Dict[int, float]] = None, outliers: bool = False,
                 use_col_perm: bool = True, use_row_perm: bool = True, bitmap: Optional[np.ndarray] = None,
                 keep_weights: bool = False, from_original: bool = False, fast_codes: bool = False,
                 group: int = GROUP, scale_format: str = "fp16", block: Tuple[int, int] = (1, 1)) -> Problem:
    """Build one seeded problem.

    ``from_original`` draws W in original coordinates and reorders it with the two
    permutations (what the offline pipeline does); otherwise the reordered weight is drawn
    directly (an i.i.d. Gaussian matrix has the same law either way).  ``fast_codes`` skips
    the float weight and draws codes / scales / zeros directly (timing runs only).
    """
    rng = _rng(seed)
    ntr, ntc = N // TILE, K // TILE
    if bitmap is None:
        # ``block`` = (rows, columns) of a bit-allocation block in tiles; a group never spans blocks
        nb = max(block[1], group // TILE)
        bitmap = make_bitmap(ntr, ntc, fractions, rng) if (block[0], nb) == (1, 1) else \
            block_bitmap(ntr, ntc, fractions, rng, block[0], nb)
    col_perm = make_perm(K, rng) if use_col_perm else None
    row_perm = make_perm(N, rng) if use_row_perm else None
    X = make_activations(M, K, _rng_x(seed, M), outliers=outliers)
    W = Wt = None
    if fast_codes:
        codes, scales, zeros = random_quantized(N, K, bitmap, w_std, rng, group, scale_format)
    else:
        if from_original:
            W = make_weights(N, K, w_std, rng)
            Wt = W
            if row_perm is not None:
                Wt = Wt[row_perm]
            if col_perm is not None:
                Wt = Wt[:, col_perm]
            Wt = np.ascontiguousarray(Wt)
        else:
            Wt = make_weights(N, K, w_std, rng)
        codes, scales, zeros = quantize_minmax(Wt, bitmap, group, scale_format)
    return Problem(label=label, N=N, K=K, M=M, X=X, bitmap=bitmap, codes=codes, scales=scales, zeros=zeros,
                   col_perm=col_perm, row_perm=row_perm, W=W if keep_weights else None,
                   Wt=Wt if keep_weights else None, seed=seed, group=group, scale_format=scale_format)


def with_activations(p: "Problem", M: int, outliers: bool) -> "Problem":
    """The same weights, bitmap and permutations with a fresh activation block of M rows."""
    import dataclasses
    return dataclasses.replace(p, M=M, X=make_activations(M, p.K, _rng_x(p.seed, M), outliers=outliers))


def config_cases(cid: int) -> Iterator[Tuple[str, int, int, int, int, dict]]:
    """Yield (label, K, N, M, seed, kwargs-for-make_problem) for every (shape, M) of a config.

    The seed is ``1000 * config + shape_index`` so that all M values of one shape share the
    same weights, bitmap and permutations.
    """
    spec = CONFIGS[cid]
    for si, (label, K, N) in enumerate(spec.shapes):
        for M in spec.Ms:
            yield (label, K, N, M, 1000 * cid + si,
                   dict(w_std=spec.w_std[si], fractions=spec.fractions, outliers=spec.outliers,
                        use_col_perm=spec.col_perm, use_row_perm=spec.row_perm[si]))


# --------------------------------------------------------------------------------------
# byte accounting (what the method itself has to move)
# --------------------------------------------------------------------------------------
def algorithmic_bytes(N: int, K: int, M: int, bitmap: np.ndarray, *, col_perm: bool = True,
                      row_perm: bool = True, index_words: int = 0, group: int = GROUP) -> int:
    """Bytes one GEMM call must move at minimum.

    codes: N*K*b/8 summed over tiles; 16-bit scale+zero: 4 bytes per row per group;
    X and Y in fp16; the two int32 permutation vectors; the int8 bitmap; optionally the
    block-index table words that replace a run-time offset computation.
    """
    code_bytes = int(bitmap.astype(np.int64).sum()) * (TILE * TILE // 8)
    sz_bytes = N * (K // group) * 4
    xy = 2 * M * K + 2 * M * N
    perms = 4 * K * int(col_perm) + 4 * N * int(row_perm)
    return code_bytes + sz_bytes + xy + perms + bitmap.size + 4 * index_words


def metadata_bits_per_weight(shapes: Sequence[Tuple[int, int]], block_rows: int = 512, block_cols: int = 128) -> float:
    """Bit-width map + reorder vectors, in bits per weight (Section 4.2, paragraph "Extra Metadata").

    One int8 per (block_rows x block_cols) block and two 16-bit reorder vectors per matrix.
    """
    meta_bytes = 0
    weights = 0
    for K, N in shapes:
        meta_bytes += (N // block_rows) * (K // block_cols) * 1 + (N + K) * 2
        weights += N * K
    return 8.0 * meta_bytes / weights
