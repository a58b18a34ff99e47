"""The comparison the GPU parity tests apply (tests/gpu_util.py) checked on the CPU: an output that is the oracle's
product rounded to fp16 passes; planted mistakes (one wrong 16-row slab of one tile, a handful of wrong outputs in a
large product, a transposed permutation) are rejected.  The mistakes are planted in copies of the oracle's inputs."""
import dataclasses
import os
import sys

import numpy as np
import pytest

import sfmp_workloads as W
from oracle import sfmp_oracle as O

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from gpu_util import check_against_oracle, elementwise_tolerance  # noqa: E402


def _fp16_of_oracle(p):
    return O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm).astype(np.float16)


@pytest.mark.parametrize("M", [1, 5, 40])
def test_rounded_oracle_output_passes(M):
    p = W.make_problem("chk", 1024, 512, M, 11, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, outliers=True)
    err = check_against_oracle(p, _fp16_of_oracle(p))
    assert err < 5e-4  # fp16 rounding of the output alone: about 2^-11 / sqrt(3)
    rows = np.random.default_rng(0).choice(p.N, 97, replace=False)
    check_against_oracle(p, _fp16_of_oracle(p), feature_rows=rows, m_rows=[0, M - 1])


def test_wrong_codes_in_one_slab_of_one_tile_are_rejected():
    # the lowest bit of four columns of one 16-row slab of one tile flipped: the norm over all outputs stays under
    # the acceptance bound (the mistake hides there), the norm over the slab's tile row does not
    p = W.make_problem("slab", 8192, 2048, 1, 12, fractions={2: 1 / 3, 3: 1 / 3, 4: 1 / 3}, fast_codes=True)
    bad = p.codes.copy()
    rows = 128 * 3 + 8 * np.arange(16) + 5  # slab 5 of tile row 3
    bad[np.ix_(rows, np.arange(128 * 7, 128 * 7 + 4))] ^= 1
    Y = _fp16_of_oracle(dataclasses.replace(p, codes=bad))
    assert O.rel_frobenius(Y, O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)) < 2e-3
    with pytest.raises(AssertionError):
        check_against_oracle(p, Y)


def test_a_few_entirely_wrong_outputs_are_rejected():
    p = W.make_problem("few", 1024, 4096, 48, 13, fractions={3: 0.5, 4: 0.5}, fast_codes=True)
    Y = _fp16_of_oracle(p)
    good = check_against_oracle(p, Y)
    Y2 = Y.copy()
    idx = np.random.default_rng(1).choice(Y.size, 20, replace=False)
    Y2.flat[idx] = -Y2.flat[idx]
    assert O.rel_frobenius(Y2, Y.astype(np.float64)) < 2e-2  # small in the norm of 196608 outputs
    with pytest.raises(AssertionError):
        check_against_oracle(p, Y2)
    assert good < 5e-4


def test_wrong_permutation_direction_is_rejected():
    p = W.make_problem("perm", 512, 256, 2, 14)
    inv = np.empty_like(p.row_perm)
    inv[p.row_perm] = np.arange(p.N, dtype=np.int32)
    Y = _fp16_of_oracle(dataclasses.replace(p, row_perm=inv))
    with pytest.raises(AssertionError):
        check_against_oracle(p, Y)


def test_tolerance_formula_values():
    # the bound at a hand-computed point: K = 4096, M = 1: D = 2 * 128 + 20 + 4 roundings (the 128 products inside the
    # matrix instructions count twice), plus the alignment term T as given
    ref, A, B, X1 = np.array([[2.0]]), np.array([[100.0]]), np.array([[300.0]]), np.array([[3000.0]])
    u16, u32 = 2.0 ** -11, 2.0 ** -24
    g = 280 * u32 / (1 - 280 * u32)
    want = u16 * 2.0 + 2.0 ** -25 + (1 + u16) * g * 300.0
    assert elementwise_tolerance(1, 4096, ref, A, B, X1)[0, 0] == pytest.approx(want, rel=1e-12)
    assert elementwise_tolerance(1, 4096, ref, A, B, X1, T=0.25)[0, 0] == pytest.approx(want + (1 + u16) * 0.25, rel=1e-12)
    gk = 8200 * u32 / (1 - 8200 * u32)
    pre = u16 * 2.0 + 2.0 ** -25 + (1 + u16) * ((u16 + u32 + gk) * 100.0 + 2.0 ** -25 * 3000.0)
    assert elementwise_tolerance(64, 4096, ref, A, B, X1)[0, 0] == pytest.approx(max(want, pre), rel=1e-12)


def test_alignment_loss_counts_by_hand():
    # one row, 64 columns = two k-steps of 32.  First: largest |x| = 40 (exponent 5), three values with exponent <= 1
    # (1.5, 0.75, -2^-20 counted at exponent -14... all <= 5 - 4), zeros ignored -> 3 * 2^(5-14).  Second: all ones
    # (exponent 0 everywhere): nothing at or below -4 -> 0.
    from gpu_util import mfma_alignment_loss
    x = np.zeros((1, 64))
    x[0, :32] = 0.0
    x[0, 0], x[0, 1], x[0, 2], x[0, 3], x[0, 4] = 40.0, 1.5, -0.75, 5.0, -(2.0 ** -20)   # 5.0: exponent 2 > 1, not counted
    x[0, 32:] = 1.0
    V = mfma_alignment_loss(x)
    assert V.shape == (1, 1)
    assert V[0, 0] == 3 * 2.0 ** (5 - 14)
    x[0, 33] = 64.0   # second k-step: exponent 6, the 31 ones left (exponent 0 <= 2) now count
    assert mfma_alignment_loss(x)[0, 0] == 3 * 2.0 ** (5 - 14) + 31 * 2.0 ** (6 - 14)
