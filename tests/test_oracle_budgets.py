"""Pins of the oracle's budget allocation to what Sec. 4.2.1 (Eq. budget) fixes:
top = k_total/(beta*m), bottom + top = 2*k_total/m, arithmetic sequence, sum = k_total,
monotonically decreasing from the bottom layer to the top layer."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import pkv_oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _grid():
    vals = {}
    with open(os.path.join(HERE, "golden", "paper_hyperparams.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            vals[k] = [int(x) for x in v]
    return vals


GRID = _grid()


def test_paper_grid_sum_monotone_endpoints():
    for L in GRID["layers"] + [4]:
        for avg in GRID["kv_size"]:
            for beta in GRID["beta"]:
                for alpha in GRID["alpha"]:
                    if alpha > avg:
                        continue
                    k = pkv_oracle.budgets(L, avg, beta, alpha).astype(np.int64)
                    A = avg - alpha
                    # total budget is spent exactly (k_total = L*A on top of the window)
                    assert k.sum() == L * avg
                    # decreasing from bottom to top layer
                    assert np.all(np.diff(k) <= 0)
                    # top layer k^{m-1} = k_total/(beta*m) = A/beta, up to the rounding unit
                    top = Fraction(A, beta)
                    assert abs(Fraction(int(k[-1] - alpha)) - top) < 1
                    # bottom layer k^0 = 2*k_total/m - k^{m-1}
                    assert abs(Fraction(int(k[0] - alpha)) - (2 * A - top)) < 1
                    # arithmetic sequence: every layer within one unit of the exact line
                    for l in range(L):
                        exact = (2 * A - top) - (2 * A - 2 * top) * Fraction(l, L - 1)
                        assert abs(Fraction(int(k[l] - alpha)) - exact) < 1
                    # window tokens are inside every layer's budget
                    assert np.all(k >= alpha)


def test_exact_when_no_rounding_needed():
    # beta | A and (L-1) | the span: the real-valued sequence is already integral.
    k = pkv_oracle.budgets(4, 128, 20, 8)
    assert list(k) == [242, 166, 90, 14]          # A=120: top 6, bottom 234, step 76
    k = pkv_oracle.budgets(3, 100, 7, 5)
    # A=95: top 95/7=13.571, bottom 176.43, middle 95 -> floors 176,95,13 (+2 units by largest remainder)
    assert k.sum() == 300 and list(k) == [181, 100, 19]
    k = pkv_oracle.budgets(5, 60, 5, 10)           # A=50: top 10, bottom 90, step 20
    assert list(k) == [100, 80, 60, 40, 20]


def test_degenerate_cases():
    assert list(pkv_oracle.budgets(1, 77, 20, 8)) == [77]          # single layer
    assert list(pkv_oracle.budgets(5, 40, 1, 8)) == [40] * 5       # beta = 1: uniform
    assert list(pkv_oracle.budgets(7, 8, 20, 8)) == [8] * 7        # nothing beyond the window
    for bad in [(0, 10, 20, 8), (4, 10, 0, 8), (4, 7, 20, 8), (4, 10, 20, -1)]:
        with pytest.raises(ValueError):
            pkv_oracle.budgets(*bad)


def test_largest_remainder_ties_go_to_lower_layers():
    # L=3, A=1, beta=2: r = [1.5, 1.0, 0.5]; floors 1,1,0 leave one unit; largest fraction is .5 at
    # layers 0 and 2 -> the lower layer takes it.
    k = pkv_oracle.budgets(3, 1, 2, 0)
    assert list(k) == [2, 1, 0]


def test_golden_file_is_what_the_oracle_gives():
    with open(os.path.join(HERE, "golden", "budget_cases.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            head, tail = line.split(":")
            L, avg, beta, alpha = (int(x) for x in head.split())
            want = [int(x) for x in tail.split()]
            assert list(pkv_oracle.budgets(L, avg, beta, alpha)) == want


# ---- other allocation strategies (appendix "Allocation Strategies") -------------------------------------


def test_geometric_schedule_ratio_sum_and_monotone():
    for (L, avg, beta, alpha) in [(32, 128, 20, 8), (32, 2048, 20, 32), (80, 512, 14, 16), (4, 128, 20, 8), (2, 64, 5, 8)]:
        k = pkv_oracle.budgets_schedule(L, avg, beta, alpha, pkv_oracle.SCHEDULE_GEOMETRIC).astype(np.int64)
        assert k.sum() == L * avg
        assert np.all(np.diff(k) <= 0) and np.all(k >= alpha)
        r = (k - alpha).astype(float)
        # top / bottom as in the linear pyramid: 1 / (2 beta - 1), up to the integer rounding of each end
        lo, hi = (r[-1] - 1) / (r[0] + 1), (r[-1] + 1) / max(r[0] - 1, 1)
        assert lo <= 1.0 / (2 * beta - 1) <= hi
        # constant ratio between neighbouring layers wherever the values are large enough to show it
        big = r[:-1] > 200
        if big.sum() > 3:
            ratios = r[1:][big] / r[:-1][big]
            assert ratios.max() - ratios.min() < 0.02


def test_geometric_schedule_is_more_bottom_heavy_than_linear():
    L, avg, beta, alpha = 32, 128, 20, 8
    lin = pkv_oracle.budgets(L, avg, beta, alpha)
    geo = pkv_oracle.budgets_schedule(L, avg, beta, alpha, pkv_oracle.SCHEDULE_GEOMETRIC)
    assert geo[0] > lin[0] and geo[L // 2] < lin[L // 2] and geo.sum() == lin.sum()


def test_uniform_schedule_and_degenerate_cases():
    assert pkv_oracle.budgets_schedule(7, 100, 20, 8, pkv_oracle.SCHEDULE_UNIFORM).tolist() == [100] * 7
    assert pkv_oracle.budgets_schedule(7, 100, 1, 8, pkv_oracle.SCHEDULE_GEOMETRIC).tolist() == [100] * 7   # beta = 1
    assert pkv_oracle.budgets_schedule(1, 100, 20, 8, pkv_oracle.SCHEDULE_GEOMETRIC).tolist() == [100]
    np.testing.assert_array_equal(pkv_oracle.budgets_schedule(32, 128, 20, 8, pkv_oracle.SCHEDULE_LINEAR),
                                  pkv_oracle.budgets(32, 128, 20, 8))
    with pytest.raises(ValueError):
        pkv_oracle.budgets_schedule(4, 100, 20, 8, 3)
