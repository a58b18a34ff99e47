"""Pins for the arithmetic half of the CPU oracle (no GPU).

Each test checks the oracle against something that is not the oracle: a value the paper
prints, an identity the paper states, a brute-force loop, an exact sum, or a closed form.
"""
import math

import numpy as np
import pytest

from oracle import sfmp_oracle as O
import sfmp_workloads as W


def _small_problem(seed=7, N=256, K=384, M=3, fractions=None, **kw):
    return W.make_problem("small", K, N, M, seed, fractions=fractions, keep_weights=True, **kw)


# ---- Appendix B worked example and Eq. 10 (bit-plane decomposition) -----------------------
def test_bit_plane_worked_example(golden):
    g = golden("bitplane_example.txt")
    ints = np.array(g["integers"], dtype=np.uint8)
    assert O.bit_plane(ints, 0).tolist() == g["lowest_bit"]
    assert O.bit_plane(ints, 3).tolist() == g["highest_bit"]
    assert O.codes_from_bit_planes([O.bit_plane(ints, i) for i in range(4)]).tolist() == g["integers"]


def test_bit_plane_linearity_eq10():
    rng = np.random.default_rng(1)
    for q in (2, 3, 4):
        Wint = rng.integers(0, 1 << q, size=(24, 40)).astype(np.uint8)
        X = rng.integers(-8, 9, size=(5, 40)).astype(np.int64)  # integers: both sides exact
        lhs = X @ Wint.astype(np.int64).T
        rhs = sum((1 << i) * (X @ O.bit_plane(Wint, i).astype(np.int64).T) for i in range(q))
        assert np.array_equal(lhs, rhs)


# ---- dequant (Appendix B Eq. 11; groups along K inside a tile) -----------------------------
def test_dequant_matches_bruteforce_loops():
    p = _small_problem(seed=11, N=128, K=256, M=1)
    w_hat = O.dequant(p.codes, p.scales, p.zeros)
    for n in range(0, p.N, 7):
        for k in range(0, p.K, 5):
            g = k // 128
            expect = float(p.scales[g, n]) * int(p.codes[n, k]) + float(p.zeros[g, n])
            assert w_hat[n, k] == expect


def test_dequant_catches_transposed_scale_layout():
    # scales are [K/128, N]; a [N, K/128] reading must not give the same result
    p = _small_problem(seed=12, N=256, K=256, M=1)
    w_hat = O.dequant(p.codes, p.scales, p.zeros)
    wrong = (p.scales.astype(np.float64).reshape(p.N, -1).repeat(128, axis=1) * p.codes
             + p.zeros.astype(np.float64).reshape(p.N, -1).repeat(128, axis=1))
    assert not np.allclose(w_hat, wrong)


@pytest.mark.parametrize("b", [2, 4])
def test_uniform_bitmap_reduces_to_plain_group_quantisation(b):
    N, K = 256, 512
    bitmap = np.full((N // 128, K // 128), b, dtype=np.int8)
    p = W.make_problem("u", K, N, 2, 21 + b, bitmap=bitmap)
    ng = K // 128
    # independent expression of uniform per-row group quantisation, group 128
    indep = (p.scales.T.astype(np.float64).reshape(N, ng, 1) * p.codes.reshape(N, ng, 128).astype(np.float64)
             + p.zeros.T.astype(np.float64).reshape(N, ng, 1)).reshape(N, K)
    assert np.array_equal(O.dequant(p.codes, p.scales, p.zeros), indep)
    assert int(p.codes.max()) == (1 << b) - 1  # min-max quantiser reaches the top level


def test_mirror_identity_eq12():
    # s^ = s/2, W^_i = 2 W_i - 1, z^ = z + 1/2 sum_i 2^i s  ==>  sum_i 2^i s^ W^_i + z^ == s q + z
    p = _small_problem(seed=31, N=128, K=256, M=1)
    w_hat = O.dequant(p.codes, p.scales, p.zeros)
    bm = np.repeat(np.repeat(p.bitmap, 128, axis=0), 128, axis=1).astype(np.int64)
    s = np.repeat(p.scales.astype(np.float64).T, 128, axis=1)
    z = np.repeat(p.zeros.astype(np.float64).T, 128, axis=1)
    acc = np.zeros_like(w_hat)
    zhat = z.copy()
    for i in range(4):
        active = (i < bm)
        mirrored = 2.0 * O.bit_plane(p.codes, i) - 1.0
        acc += np.where(active, (2.0 ** i) * (s / 2.0) * mirrored, 0.0)
        zhat += np.where(active, 0.5 * (2.0 ** i) * s, 0.0)
    assert np.allclose(acc + zhat, w_hat, rtol=0, atol=1e-12)


@pytest.mark.parametrize("b", [2, 3, 4])
def test_quantiser_error_variance_is_step_squared_over_12(b):
    # Eq. 5: a uniform quantiser with step delta has E[(w - w')^2] = delta^2 / 12.
    N, K = 512, 512
    bitmap = np.full((N // 128, K // 128), b, dtype=np.int8)
    p = W.make_problem("v", K, N, 1, 40 + b, bitmap=bitmap, keep_weights=True)
    err = O.dequant(p.codes, p.scales, p.zeros) - p.Wt.astype(np.float64)
    s = np.repeat(p.scales.astype(np.float64).T, 128, axis=1)
    ratio = float(np.mean(err ** 2) / np.mean(s ** 2 / 12.0))
    assert 0.85 < ratio < 1.15, ratio
    assert float(np.max(np.abs(err) / s)) <= 0.5 + 2e-2  # never more than half a step (+ fp16 rounding of z)


# ---- matmul ----------------------------------------------------------------------------
def test_gemm_matches_triple_loop_and_exact_sum():
    p = _small_problem(seed=51, N=128, K=128, M=3, use_col_perm=True, use_row_perm=True)
    Y = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)
    assert Y.shape == (3, 128) and Y.dtype == np.float64
    for m in range(3):
        for i in range(0, 128, 9):
            terms = []
            for j in range(p.K):
                w = float(p.scales[j // 128, i]) * int(p.codes[i, j]) + float(p.zeros[j // 128, i])
                terms.append(float(p.X[m, p.col_perm[j]]) * w)
            exact = math.fsum(terms)
            assert abs(Y[m, p.row_perm[i]] - exact) <= 1e-12 * max(1.0, abs(exact))


def test_gemm_rows_agrees_with_full_product():
    p = _small_problem(seed=52, N=256, K=256, M=2)
    rows = np.array([0, 5, 130, 255])
    Yt = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, None)
    part = O.gemm_rows(p.X, p.col_perm, p.codes, p.scales, p.zeros, rows)
    assert np.allclose(part, Yt[:, rows], rtol=1e-13, atol=1e-13)


# ---- permutations (Section 3.4, Eq. 8-9) ---------------------------------------------------
def test_permutation_equivalence_in_original_coordinates():
    p = W.make_problem("perm", 384, 256, 4, 61, from_original=True, keep_weights=True)
    w_hat = O.dequant(p.codes, p.scales, p.zeros)  # reordered coordinates
    # scatter the dequantised weight back to original coordinates without using the oracle's gather
    W_orig = np.zeros_like(w_hat)
    for i in range(p.N):
        W_orig[p.row_perm[i], p.col_perm] = w_hat[i]
    Y_direct = p.X.astype(np.float64) @ W_orig.T
    Y = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)
    assert np.allclose(Y, Y_direct, rtol=1e-12, atol=1e-12)
    # gathering X beforehand and passing the identity gives the same product
    Xg = p.X[:, p.col_perm]
    Y2 = O.gemm(Xg, None, p.codes, p.scales, p.zeros, p.row_perm)
    assert np.array_equal(Y, Y2)
    # leaving rows reordered, then un-permuting by hand
    Yt = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, None)
    assert np.array_equal(Yt, Y[:, p.row_perm])
    # the reordered weight really is W[row_perm][:, col_perm]
    assert np.array_equal(p.Wt, p.W[p.row_perm][:, p.col_perm])


def test_identity_permutations_are_noops():
    p = _small_problem(seed=62, N=128, K=256, M=2)
    ident_c = np.arange(p.K, dtype=np.int32)
    ident_r = np.arange(p.N, dtype=np.int32)
    a = O.gemm(p.X, None, p.codes, p.scales, p.zeros, None)
    b = O.gemm(p.X, ident_c, p.codes, p.scales, p.zeros, ident_r)
    assert np.array_equal(a, b)


def test_wrong_permutation_direction_is_detected():
    # the inverse permutation on the activation must NOT reproduce the product (guards the gather direction)
    p = W.make_problem("perm", 256, 128, 2, 63, from_original=True, keep_weights=True)
    inv = np.argsort(p.col_perm).astype(np.int32)
    good = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)
    bad = O.gemm(p.X, inv, p.codes, p.scales, p.zeros, p.row_perm)
    ref = p.X.astype(np.float64) @ p.W.astype(np.float64).T
    assert O.rel_frobenius(good, ref) < 0.5 * O.rel_frobenius(bad, ref)


# ---- end-to-end sanity: the quantised product sits where the quantisation noise predicts -----
def test_quantised_product_noise_band():
    N, K, M = 512, 1024, 8
    p = W.make_problem("band", K, N, M, 71, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, from_original=True,
                       keep_weights=True)
    Y = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)
    Y_fp = p.X.astype(np.float64) @ p.W.astype(np.float64).T
    # independent noise with variance s^2/12 per weight -> E||dY||^2 = sum_m sum_n sum_k x^2 s^2/12
    s = np.repeat(p.scales.astype(np.float64).T, 128, axis=1)  # [N, K] reordered
    x2 = (p.X.astype(np.float64)[:, p.col_perm]) ** 2  # [M, K] reordered
    predicted = math.sqrt(float((x2 @ (s ** 2 / 12.0).T).sum()))
    observed = float(np.linalg.norm(Y - Y_fp))
    assert 0.8 < observed / predicted < 1.25, (observed, predicted)


def test_rel_frobenius_definition():
    a = np.array([[3.0, 4.0]])
    b = np.array([[3.0, 0.0]])
    assert O.rel_frobenius(a, b) == pytest.approx(4.0 / 3.0)
    assert O.rel_frobenius(b, b) == 0.0


# ---- group lengths beyond 128 and bf16 parameters ("Effect of n_b" ablation; Table 1 caption) -----------
@pytest.mark.parametrize("group", [256, 512])
def test_longer_groups_match_bruteforce_and_reduce_to_group_128(group):
    p = _small_problem(seed=21, N=256, K=1024, fractions={2: 0.5, 4: 0.5}, group=group)
    assert p.scales.shape == (p.K // group, p.N)
    w_hat = O.dequant(p.codes, p.scales, p.zeros)
    # brute force on a sample of elements, straight from the definition
    rng = np.random.default_rng(3)
    for n, k in zip(rng.integers(0, p.N, 200), rng.integers(0, p.K, 200)):
        g = k // group
        assert w_hat[n, k] == float(p.scales[g, n]) * float(p.codes[n, k]) + float(p.zeros[g, n])
    # a parameter shared by `group` columns is the same as that parameter repeated for every 128 columns
    rep = group // 128
    w_128 = O.dequant(p.codes, np.repeat(p.scales, rep, axis=0), np.repeat(p.zeros, rep, axis=0))
    assert np.array_equal(w_hat, w_128)
    rows = np.array([0, 5, 130, 255])
    assert np.array_equal(O.dequant_rows(p.codes, p.scales, p.zeros, rows), w_hat[rows])
    # the quantiser used one width per group: its error stays within half a step
    err = np.abs(w_hat - p.Wt.astype(np.float64))
    step = np.repeat(p.scales.astype(np.float64).T, group, axis=1)
    assert (err <= 0.5 * step * (1 + 1e-2) + 1e-3 * np.abs(p.Wt.astype(np.float64)) + 1e-6).all()


def test_group_64_matches_bruteforce_and_reduces_to_group_128():
    # "Effect of n_b" (Appendix G): 64 columns per (scale, zero) pair, two groups inside every 128-column tile
    p = _small_problem(seed=23, N=256, K=512, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, group=64)
    assert p.scales.shape == (p.K // 64, p.N) and O.group_length(p.K, p.scales) == 64
    w_hat = O.dequant(p.codes, p.scales, p.zeros)
    rng = np.random.default_rng(4)
    for n, k in zip(rng.integers(0, p.N, 300), rng.integers(0, p.K, 300)):
        g = k // 64
        assert w_hat[n, k] == float(p.scales[g, n]) * float(p.codes[n, k]) + float(p.zeros[g, n])
    # columns 64..127 of a tile use the second pair: swapping the two pairs of a tile changes exactly those tiles
    sw_s, sw_z = p.scales.copy(), p.zeros.copy()
    sw_s[[0, 1]], sw_z[[0, 1]] = p.scales[[1, 0]], p.zeros[[1, 0]]
    w_sw = O.dequant(p.codes, sw_s, sw_z)
    assert np.array_equal(w_sw[:, 128:], w_hat[:, 128:]) and not np.array_equal(w_sw[:, :128], w_hat[:, :128])
    # a group-128 parameter set repeated for both halves of its group is the group-128 result
    q = _small_problem(seed=23, N=256, K=512, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3})
    assert np.array_equal(O.dequant(q.codes, np.repeat(q.scales, 2, axis=0), np.repeat(q.zeros, 2, axis=0)),
                          O.dequant(q.codes, q.scales, q.zeros))
    rows = np.array([0, 77, 255])
    assert np.array_equal(O.dequant_rows(p.codes, p.scales, p.zeros, rows), w_hat[rows])
    # the quantiser used the tile's width for both of its groups: the error stays within half a step
    err = np.abs(w_hat - p.Wt.astype(np.float64))
    step = np.repeat(p.scales.astype(np.float64).T, 64, axis=1)
    assert (err <= 0.5 * step * (1 + 1e-2) + 1e-3 * np.abs(p.Wt.astype(np.float64)) + 1e-6).all()
    # and the product follows: gemm on these parameters equals the triple loop on a few outputs
    Y = O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)
    for m, i in ((0, 3), (2, 200)):
        acc = math.fsum(float(p.X[m, p.col_perm[k]]) * float(w_hat[i, k]) for k in range(p.K))
        assert Y[m, p.row_perm[i]] == pytest.approx(acc, rel=1e-12)
    # byte accounting: 0.5 bit per weight of parameters at group 64 (the ablation's overhead column)
    extra = W.algorithmic_bytes(p.N, p.K, 1, p.bitmap, group=64) - W.algorithmic_bytes(p.N, p.K, 1, p.bitmap, group=128)
    assert extra * 8 == p.N * p.K // 4  # 0.5 - 0.25 bit per weight


def test_bf16_storage_values_and_bits():
    # bf16 keeps the top 16 bits of the float32 pattern, rounded to nearest even
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.14159, -2.5e-3, 0.0], dtype=np.float32)
    y = W.to_bf16(x)
    assert y.tolist() == [1.0, 1.0, 1.015625, 3.140625, -0.00250244140625, 0.0]
    assert W.param_bits(y).tolist() == [0x3F80, 0x3F80, 0x3F82, 0x4049, 0xBB24, 0x0000]
    assert W.param_bits(np.array([1.0, -2.0], dtype=np.float16)).tolist() == [0x3C00, 0xC000]
    p = _small_problem(seed=22, N=128, K=512, scale_format="bf16")
    assert p.scales.dtype == np.float32 and np.array_equal(W.to_bf16(p.scales), p.scales)
    w_hat = O.dequant(p.codes, p.scales, p.zeros)
    assert w_hat[3, 200] == float(p.scales[1, 3]) * float(p.codes[3, 200]) + float(p.zeros[1, 3])
    # the quantised weight tracks the original to within half a step plus the bf16 rounding of the zero-point
    err = np.abs(w_hat - p.Wt.astype(np.float64))
    step = np.repeat(p.scales.astype(np.float64).T, 128, axis=1)
    zmag = np.repeat(np.abs(p.zeros.astype(np.float64)).T, 128, axis=1)
    assert (err <= 0.5 * step * (1 + 1e-2) + zmag * 2.0 ** -8 + 1e-6).all()


def test_block_bitmap_is_constant_on_blocks():
    bm = W.block_bitmap(8, 6, {2: 0.5, 3: 0.25, 4: 0.25}, np.random.default_rng(0), mb_tiles=4, nb_tiles=2)
    assert bm.shape == (8, 6)
    for i in range(0, 8, 4):
        for j in range(0, 6, 2):
            assert (bm[i:i + 4, j:j + 2] == bm[i, j]).all()
    assert sorted(np.unique(bm).tolist()) == [2, 3, 4]
