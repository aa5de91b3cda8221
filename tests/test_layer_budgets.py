"""Sensitivity-aware layer budgets (Sec. 3.2, Eq. 6): oracle pins and the host entry point.  CPU only."""
import ctypes

import numpy as np
import pytest

from oracle import epicache_oracle as orc
from paper_2509_17396_amd import binding as ep


def test_oracle_closed_forms():
    # alpha = 1, s = 1..4, L*M = 40: shares are exact integers 4, 8, 12, 16
    assert orc.layer_budgets([1, 2, 3, 4], 1.0, 10) == [4, 8, 12, 16]
    np.testing.assert_allclose(orc.layer_budgets_real([1, 2, 3, 4], 1.0, 10), [4, 8, 12, 16], rtol=1e-15)
    # alpha = 2: quotas 4/3, 16/3, 12, 64/3 -> floors 1, 5, 12, 21 (39); the spare row goes to the
    # largest remainder, three tie at 1/3 -> lowest layer
    assert orc.layer_budgets([1, 2, 3, 4], 2.0, 10) == [2, 5, 12, 21]
    # alpha = 0 or equal sensitivities: uniform
    assert orc.layer_budgets([0.3, 0.9, 0.1], 0.0, 7) == [7, 7, 7]
    assert orc.layer_budgets([0.25] * 5, 3.0, 11) == [11] * 5
    # a dead layer still keeps one row, taken from the largest
    assert orc.layer_budgets([0.0, 1.0, 1.0], 1.0, 4) == [1, 5, 6]
    assert orc.layer_budgets([0.0, 0.0], 2.0, 9) == [9, 9]


def test_oracle_invariants_random():
    rng = np.random.default_rng(41)
    for _ in range(200):
        L = int(rng.integers(1, 40))
        M = int(rng.integers(1, 5000))
        alpha = float(rng.choice([0.5, 1.0, 2.0, 4.0, 8.0]))
        s = rng.random(L) * 0.5 + 0.01
        got = orc.layer_budgets(s, alpha, M)
        real = orc.layer_budgets_real(s, alpha, M)
        assert sum(got) == L * M and min(got) >= 1                 # Eq. 6: budgets sum to L * M
        n_fixed = int((real < 1.0).sum())                          # layers lifted to one row, paid by the largest
        assert (np.abs(np.array(got) - real) < 1.0 + n_fixed).all()  # otherwise within one row of Eq. 6
        order = np.argsort(s, kind="stable")
        assert (np.diff(np.array(got)[order]) >= -1 - n_fixed).all()  # monotone in the sensitivity (up to rounding)


def test_larger_alpha_sharpens_the_allocation():
    s = [0.1, 0.2, 0.4, 0.8]
    spreads = [max(orc.layer_budgets(s, a, 1000)) - min(orc.layer_budgets(s, a, 1000)) for a in (1, 2, 4, 8)]
    assert spreads == sorted(spreads) and spreads[0] < spreads[-1]


def test_library_matches_oracle():
    rng = np.random.default_rng(43)
    for _ in range(300):
        L = int(rng.integers(1, 48))
        M = int(rng.integers(1, 20000))
        alpha = float(rng.choice([0.0, 0.5, 1.0, 2.0, 4.0, 8.0]))
        s = np.round(rng.random(L), 3)          # ties and exact zeros happen
        assert ep.epicache_layer_budgets(s, alpha, M) == orc.layer_budgets(s, alpha, M)
    assert ep.epicache_layer_budgets([1, 2, 3, 4], 2.0, 10) == [2, 5, 12, 21]


@pytest.mark.parametrize("sens,alpha,budget", [([0.1, -0.2], 1.0, 8), ([0.1, float("nan")], 1.0, 8),
                                               ([0.1, 0.2], -1.0, 8), ([0.1, 0.2], 1.0, 0), ([], 1.0, 8)])
def test_library_rejects_bad_arguments(sens, alpha, budget):
    n = len(sens)
    arr = (ctypes.c_double * max(n, 1))(*sens)
    out = (ctypes.c_int32 * max(n, 1))()
    assert ep.load().epicache_layer_budgets(arr, n, alpha, budget, out) == ep.ERR_INVALID_ARG
    assert ep.load().epicache_layer_budgets(None, 2, 1.0, 8, out) == ep.ERR_INVALID_ARG
