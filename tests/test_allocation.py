"""Pins for the offline reordering / bit-allocation helpers (no GPU): brute force on tiny inputs, closed forms."""
import itertools

import numpy as np
import pytest

from sfmp_workloads import allocation as A


def _brute_force(sal, widths, counts):
    """Least loss over ALL assignments with the given number of units per width."""
    n = sal.size
    best = None
    for lo in itertools.combinations(range(n), counts[0]):
        rest = [i for i in range(n) if i not in lo]
        if len(widths) == 2:
            bits = np.full(n, widths[1])
            bits[list(lo)] = widths[0]
            loss = A.allocation_loss(sal, bits)
            best = loss if best is None else min(best, loss)
            continue
        for mid in itertools.combinations(rest, counts[1]):
            bits = np.full(n, widths[2])
            bits[list(lo)] = widths[0]
            bits[list(mid)] = widths[1]
            loss = A.allocation_loss(sal, bits)
            best = loss if best is None else min(best, loss)
    return best


def test_two_widths_worked_example_and_bruteforce():
    # salience 1, 2, 3, 4 at an average of 3 bits from {2, 4}: half the units, the two least salient, get 2 bits
    sal = np.array([3.0, 1.0, 4.0, 2.0])
    bits = A.allocate_two(sal, (2, 4), 3.0)
    assert bits.tolist() == [4, 2, 4, 2]
    assert A.allocation_loss(sal, bits) == pytest.approx(1 / 9 + 2 / 9 + 3 / 225 + 4 / 225)
    rng = np.random.default_rng(0)
    for _ in range(5):
        sal = rng.lognormal(size=9)
        bits = A.allocate_two(sal, (2, 3), 2.0 + 4 / 9)  # 5 of 9 units at 2 bits
        assert int((bits == 2).sum()) == 5
        assert A.allocation_loss(sal, bits) == pytest.approx(_brute_force(sal, (2, 3), (5, 4)))


def test_three_widths_matches_bruteforce_over_the_same_grid():
    rng = np.random.default_rng(1)
    for trial in range(4):
        n = 8
        sal = rng.lognormal(sigma=1.5, size=n)
        target, step = 3.0, 0.125  # the grid alpha_1 = k/8 makes every n_k an integer
        bits = A.allocate_three(sal, (2, 3, 4), target, step=step)
        assert bits.astype(np.float64).mean() == pytest.approx(target)
        best = None
        for n1 in range(n + 1):  # n1 two-bit units force n3 = n1 four-bit units at an average of 3 bits
            n2 = n - 2 * n1
            if n2 < 0:
                continue
            loss = _brute_force(sal, (2, 3, 4), (n1, n2, n1))
            best = loss if best is None else min(best, loss)
        assert A.allocation_loss(sal, bits) == pytest.approx(best)
        # higher salience never gets fewer bits
        order = np.argsort(sal)
        assert (np.diff(bits[order].astype(int)) >= 0).all()


def test_three_widths_budget_and_degenerate_targets():
    rng = np.random.default_rng(2)
    sal = rng.lognormal(size=(28, 32))
    for target in (2.25, 2.5, 3.0, 3.25, 3.5):
        bits = A.allocate_three(sal, (2, 3, 4), target)
        avg = bits.astype(np.float64).mean()
        # floors can only push units to the widest width: the budget is met from above by less than one step per unit
        assert target - 1e-9 <= avg <= target + 3.0 / sal.size + 0.02
    assert (A.allocate_three(sal, (2, 3, 4), 2.0) == 2).all()
    assert (A.allocate_three(sal, (2, 3, 4), 4.0) == 4).all()


def test_reordering_sorts_row_and_column_salience():
    rng = np.random.default_rng(3)
    F = A.synthetic_salience(256, 384, rng)
    rp, cp = A.reorder(F)
    assert sorted(rp.tolist()) == list(range(256)) and sorted(cp.tolist()) == list(range(384))
    Ft = F[rp][:, cp]
    assert (np.diff(Ft.sum(axis=1, dtype=np.float64)) <= 1e-6).all()
    assert (np.diff(Ft.sum(axis=0, dtype=np.float64)) <= 1e-6).all()
    # block salience adds up
    sal = A.block_salience(Ft, 128, 128)
    assert sal.shape == (2, 3) and sal.sum() == pytest.approx(float(F.sum(dtype=np.float64)), rel=1e-6)
    assert sal[0, 0] == pytest.approx(float(Ft[:128, :128].sum(dtype=np.float64)), rel=1e-6)


def test_allocated_layout_clusters_wide_tiles_top_left():
    rng = np.random.default_rng(4)
    lay = A.allocated_layout(2048, 1024, 3.0, rng, block=(4, 1))
    bm = lay["bitmap"]
    assert bm.shape == (16, 8) and set(np.unique(bm).tolist()) <= {2, 3, 4}
    for i in range(0, 16, 4):  # constant on (512, 128) blocks
        assert (bm[i:i + 4] == bm[i]).all()
    assert abs(bm.astype(np.float64).mean() - 3.0) <= 0.15
    # salient rows / columns come first, so the mean width falls from the top-left to the bottom-right quadrant
    assert bm[:8, :4].mean() > bm[8:, 4:].mean()
