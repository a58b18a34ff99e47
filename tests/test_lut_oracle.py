"""Pins for the CPU oracle of the one-bit lookup-table GEMV (no GPU).

Each test checks the oracle against something that is not the oracle: the worked example the
paper prints, the plain definition of the product written out here with loops, a brute-force
enumeration of the 256 signed sums, exact integer arithmetic."""
import itertools

import numpy as np
import pytest

from oracle import sfmp_lut_oracle as L
import sfmp_workloads as W


def _problem(seed=3, N=256, K=384, fractions=None):
    return W.make_problem("lut", K, N, 1, seed, fractions=fractions, keep_weights=True)


# ---- the bit-plane byte format ---------------------------------------------------------------
def test_plane_bytes_of_the_papers_worked_example(golden):
    g = golden("lut_bitplane_bytes.txt")
    codes = np.zeros((128, 128), dtype=np.uint8)
    codes[0, :4] = g["integers"]
    planes, tile_off = L.lut_pack(codes, np.array([[4]], dtype=np.int8))
    assert tile_off.tolist() == [0, 4]
    assert planes.size == 4 * 2048
    assert [int(planes[i * 2048]) for i in range(4)] == g["plane_bytes"]
    assert int(planes.astype(np.int64).sum()) == sum(g["plane_bytes"])  # every other byte is zero


def test_pack_places_every_bit_where_the_format_says():
    rng = np.random.default_rng(5)
    bitmap = np.array([[2, 4, 3], [3, 2, 4]], dtype=np.int8)
    N, K = 256, 384
    codes = np.zeros((N, K), dtype=np.uint8)
    for tr in range(2):
        for tc in range(3):
            codes[tr * 128:(tr + 1) * 128, tc * 128:(tc + 1) * 128] = rng.integers(0, 1 << bitmap[tr, tc], (128, 128))
    planes, tile_off = L.lut_pack(codes, bitmap)
    assert tile_off.tolist() == [0, 2, 6, 9, 12, 14, 18]
    assert planes.size == 18 * 2048
    for _ in range(400):  # sampled bits, located by the format's formula written out here
        n, k = int(rng.integers(N)), int(rng.integers(K))
        tr, tc, r, c = n // 128, k // 128, n % 128, k % 128
        b = int(bitmap[tr, tc])
        i = int(rng.integers(b))
        byte = planes[(int(tile_off[tr * 3 + tc]) + i) * 2048 + r * 16 + c // 8]
        assert (int(byte) >> (c % 8)) & 1 == (int(codes[n, k]) >> i) & 1
    assert np.array_equal(L.lut_unpack(N, K, planes, tile_off), codes)


# ---- the table (Appendix B: mirror storage) ---------------------------------------------------
def test_half_table_and_mirror_against_all_256_sign_patterns():
    rng = np.random.default_rng(9)
    x8 = rng.integers(-50, 51, size=8).astype(np.float64)  # integers: every sum is exact
    table = L.half_table(x8)
    for signs in itertools.product((0, 1), repeat=8):  # signs[t] = 1: +x_t, 0: -x_t
        byte = sum(s << t for t, s in enumerate(signs))
        direct = sum(x8[t] if s else -x8[t] for t, s in enumerate(signs))
        assert L.table_lookup(table, np.array([byte]))[0] == direct
    assert table[0] == -x8.sum() and table[127] == x8[:7].sum() - x8[7]


# ---- the whole product against the plain definition -------------------------------------------
@pytest.mark.parametrize("seed,N,K,fractions", [(1, 128, 128, {2: 1.0}), (2, 256, 384, None), (3, 384, 256, {3: 0.5, 4: 0.5}),
                                                (4, 128, 512, {2: 0.5, 4: 0.5})])
def test_lut_gemv_equals_the_definition(seed, N, K, fractions):
    p = _problem(seed, N, K, fractions)
    planes, tile_off = L.lut_pack(p.codes, p.bitmap)
    y = L.lut_gemv(p.X[0], p.col_perm, N, K, planes, tile_off, p.scales, p.zeros, p.row_perm)
    # the definition, with loops over the output features and quantisation groups
    xp = p.X[0].astype(np.float64)[p.col_perm.astype(np.int64)] if p.col_perm is not None else p.X[0].astype(np.float64)
    s, z = p.scales.astype(np.float64), p.zeros.astype(np.float64)
    ref_t = np.zeros(N)
    for n in range(N):
        for g in range(K // 128):
            q = p.codes[n, g * 128:(g + 1) * 128].astype(np.float64)
            ref_t[n] += np.dot(s[g, n] * q + z[g, n], xp[g * 128:(g + 1) * 128])
    ref = np.zeros(N)
    if p.row_perm is not None:
        ref[p.row_perm.astype(np.int64)] = ref_t
    else:
        ref = ref_t
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-11 * np.abs(ref).max())


def test_lut_gemv_exact_on_integers():
    # integer activations, unit scales, zero offsets: every step is exact in float64
    rng = np.random.default_rng(12)
    N, K = 128, 256
    bitmap = np.array([[3, 4]], dtype=np.int8)
    codes = np.zeros((N, K), dtype=np.uint8)
    codes[:, :128] = rng.integers(0, 8, (N, 128))
    codes[:, 128:] = rng.integers(0, 16, (N, 128))
    x = rng.integers(-9, 10, size=K).astype(np.float64)
    planes, tile_off = L.lut_pack(codes, bitmap)
    y = L.lut_gemv(x, None, N, K, planes, tile_off, np.ones((2, N)), np.zeros((2, N)))
    assert np.array_equal(y, codes.astype(np.int64) @ x.astype(np.int64))


def test_a_dropped_plane_weight_or_mirror_sign_is_caught():
    # the pins above fail for plausible mistakes: check two of them on a copy of the arithmetic
    p = _problem(6, 128, 128, {4: 1.0})
    planes, tile_off = L.lut_pack(p.codes, p.bitmap)
    good = L.lut_gemv(p.X[0], p.col_perm, 128, 128, planes, tile_off, p.scales, p.zeros, p.row_perm)
    flipped = planes.copy()
    flipped[3 * 2048:] ^= 0x80  # top sign of every byte of the highest plane
    bad = L.lut_gemv(p.X[0], p.col_perm, 128, 128, flipped, tile_off, p.scales, p.zeros, p.row_perm)
    assert not np.allclose(good, bad, rtol=1e-6, atol=0)


# ---- table entries rounded to fp16 (the 2-byte entries of Appendix F) -------------------------------------
def test_fp16_tables_change_nothing_when_every_entry_is_representable():
    # small integer activations: every signed sum of 8 of them is an integer below 2048, exact in fp16
    rng = np.random.default_rng(14)
    N, K = 128, 256
    bitmap = np.array([[2, 4]], dtype=np.int8)
    codes = np.zeros((N, K), dtype=np.uint8)
    codes[:, :128] = rng.integers(0, 4, (N, 128))
    codes[:, 128:] = rng.integers(0, 16, (N, 128))
    x = rng.integers(-100, 101, size=K).astype(np.float64)
    planes, tile_off = L.lut_pack(codes, bitmap)
    s, z = rng.uniform(0.5, 2.0, (2, N)), rng.normal(size=(2, N))
    y = L.lut_gemv(x, None, N, K, planes, tile_off, s, z)
    y16 = L.lut_gemv(x, None, N, K, planes, tile_off, s, z, table_dtype=np.float16)
    assert np.array_equal(y, y16)


def test_fp16_tables_stay_within_the_rounding_bound_and_do_round():
    # |y16 - y| <= 2^-11 * sum over the looked-up entries of |entry| * (their weight s^ 2^i), plus the same for the
    # entries that make up the column sums (weight |z^|); written out here with loops over the plain definition
    p = _problem(9, 128, 256, {3: 0.5, 4: 0.5})
    planes, tile_off = L.lut_pack(p.codes, p.bitmap)
    y = L.lut_gemv(p.X[0], p.col_perm, p.N, p.K, planes, tile_off, p.scales, p.zeros, p.row_perm)
    y16 = L.lut_gemv(p.X[0], p.col_perm, p.N, p.K, planes, tile_off, p.scales, p.zeros, p.row_perm, table_dtype=np.float16)
    assert not np.array_equal(y, y16)  # Gaussian activations: the entries do get rounded
    xp = p.X[0].astype(np.float64)[p.col_perm]
    s, z = p.scales.astype(np.float64), p.zeros.astype(np.float64)
    bound_t = np.zeros(p.N)
    for n in range(p.N):
        for tc in range(p.K // 128):
            b = int(p.bitmap[n // 128, tc])
            s_hat = abs(s[tc, n]) / 2
            z_hat = abs(z[tc, n] + 0.5 * (2 ** b - 1) * s[tc, n])
            for g in range(16):
                xs = xp[tc * 128 + 8 * g:tc * 128 + 8 * g + 8]
                q = p.codes[n, tc * 128 + 8 * g:tc * 128 + 8 * g + 8].astype(np.int64)
                for i in range(b):
                    signs = 2.0 * ((q >> i) & 1) - 1.0
                    bound_t[n] += s_hat * (2 ** i) * abs(float(signs @ xs))
                bound_t[n] += z_hat * abs(float(xs.sum()))
    bound = np.zeros(p.N)
    bound[p.row_perm] = bound_t
    assert np.all(np.abs(y16 - y) <= 2.0 ** -11 * bound * (1 + 1e-9))
    assert np.linalg.norm(y16 - y) / np.linalg.norm(y) < 1e-3
