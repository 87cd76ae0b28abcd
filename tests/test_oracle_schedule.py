"""Pins of the estimator updates and the scheduling oracle (Section III-C)."""
import numpy as np
import pytest

from oracle import schedule as sch


def test_ema_hand_arithmetic():
    a = sch.update_alpha_hat([0.5, 0.5, 0.9], [1.0, 0.0, 0.123], [4, 2, 0], eta=0.2)
    np.testing.assert_allclose(a, [0.6, 0.4, 0.9])              # gamma = 0 keeps its estimate
    X = sch.update_goodput([1.0, 4.0], [3, 0], beta=0.5)
    np.testing.assert_allclose(X, [2.5, 2.5])                   # x = accepted + 1


def test_hand_worked_allocations():
    # gains (1/X) a^(S+1): server 1 offers 0.8, 0.64, 0.512, all above server 0's first 0.5
    np.testing.assert_array_equal(sch.schedule_greedy([0.5, 0.8], [1.0, 1.0], 3), [0, 3])
    # with X = (1, 2): server 0 offers 0.5, 0.25; server 1 offers 0.4, 0.32, 0.256
    np.testing.assert_array_equal(sch.schedule_greedy([0.5, 0.8], [1.0, 2.0], 3), [1, 2])
    # symmetric servers share the budget equally (the fixed split C/N)
    np.testing.assert_array_equal(sch.schedule_greedy([0.7] * 4, [2.0] * 4, 12), [3, 3, 3, 3])
    # ties go to the lowest index
    np.testing.assert_array_equal(sch.schedule_greedy([0.7] * 3, [2.0] * 3, 4), [2, 1, 1])


def test_objective_is_the_stated_sum():
    val = sch.objective([0.5, 0.8], [1.0, 2.0], [1, 2])
    assert val == pytest.approx(1.0 * (1 + 0.5) + 0.5 * (1 + 0.8 + 0.64))


@pytest.mark.parametrize("seed", range(12))
def test_greedy_attains_the_exhaustive_optimum(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 5))
    C = int(rng.integers(0, 11))
    a = rng.uniform(0.05, 0.98, n)
    X = rng.uniform(0.5, 6.0, n)
    best, _ = sch.schedule_exhaustive(a, X, C)
    S = sch.schedule_greedy(a, X, C)
    assert S.sum() == C and np.all(S >= 0)
    assert sch.objective(a, X, S) == pytest.approx(best, rel=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_greedy_with_box_bounds_attains_the_bounded_optimum(seed):
    rng = np.random.default_rng(50 + seed)
    n, C, lo, hi = 3, 9, 1, 4
    a = rng.uniform(0.05, 0.98, n)
    X = rng.uniform(0.5, 6.0, n)
    best, _ = sch.schedule_exhaustive(a, X, C, lo, hi)
    S = sch.schedule_greedy(a, X, C, lo, hi)
    assert np.all(S >= lo) and np.all(S <= hi) and S.sum() == min(C, n * hi)
    assert sch.objective(a, X, S) == pytest.approx(best, rel=1e-12)


def test_monotonicity_invariants():
    rng = np.random.default_rng(7)
    for _ in range(30):
        n, C = 5, 20
        a = rng.uniform(0.2, 0.95, n)
        X = rng.uniform(0.5, 5.0, n)
        S = sch.schedule_greedy(a, X, C)
        X2 = X.copy(); X2[2] *= 0.5                     # a server that has received less gets no fewer slots
        assert sch.schedule_greedy(a, X2, C)[2] >= S[2]
        Xe = np.ones(n)
        Se = sch.schedule_greedy(a, Xe, C)
        a2 = a.copy(); a2[1] = min(0.99, a2[1] + 0.04)   # a better-aligned draft model gets no fewer slots
        assert sch.schedule_greedy(a2, Xe, C)[1] >= Se[1]


def test_degenerate_alpha_is_clamped_not_divided_by_zero():
    S = sch.schedule_greedy([1.0, 0.0], [1.0, 1.0], 5)
    np.testing.assert_array_equal(S, [5, 0])
    assert np.isfinite(sch.objective([1.0, 0.0], [1.0, 1.0], S))


def test_round_updates_before_solving():
    a, X, g = sch.schedule_round([3, 0], [1.0, 0.0], [3, 3], [0.5, 0.5], [1.0, 1.0], 0.2, 0.5, 4)
    np.testing.assert_allclose(a, [0.6, 0.4]); np.testing.assert_allclose(X, [2.5, 1.0])
    # gains with the *updated* state: s0: 0.24, 0.144, ... ; s1: 0.4, 0.16, 0.064
    np.testing.assert_array_equal(g, [2, 2])
