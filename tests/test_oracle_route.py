"""Pins for the oracle's three-way routing (Section 3.2, Steps 1 and 3)."""
import itertools
import math

import numpy as np
import pytest
from scipy.stats import norm

from oracle import vector_oracle as vo


def _check_invariants(score, eps, n_pool, n_approx, tier, idx_r, idx_a):
    h_, n = score.shape
    for h in range(h_):
        t = tier[h]
        assert (t == vo.APPROX).sum() == n_approx
        assert (t == vo.RETAIN).sum() == n_pool - n_approx
        assert (t == vo.EVICT).sum() == n - n_pool
        assert np.all(np.diff(idx_r[h]) > 0) and np.all(np.diff(idx_a[h]) > 0)
        np.testing.assert_array_equal(np.flatnonzero(t == vo.RETAIN), idx_r[h])
        np.testing.assert_array_equal(np.flatnonzero(t == vo.APPROX), idx_a[h])
        pool = np.flatnonzero(t != vo.EVICT)
        ev = np.flatnonzero(t == vo.EVICT)
        if len(pool) and len(ev):
            worst_in = min((float(score[h, i]), -int(i)) for i in pool)
            best_out = max((float(score[h, i]), -int(i)) for i in ev)
            assert worst_in > best_out
        if n_approx and n_pool > n_approx:
            worst_apx = max((float(eps[h, i]), int(i)) for i in idx_a[h])
            best_ret = min((float(eps[h, i]), int(i)) for i in idx_r[h])
            assert worst_apx < best_ret


def test_invariants_random_with_ties():
    rng = np.random.default_rng(0)
    for trial in range(20):
        n = int(rng.integers(5, 200))
        n_pool = int(rng.integers(0, n + 1))
        n_approx = int(rng.integers(0, n_pool + 1))
        # few distinct values => many ties in both keys
        score = rng.integers(0, 4, size=(3, n)).astype(np.float32)
        eps = rng.integers(0, 3, size=(3, n)).astype(np.float32)
        out = vo.route(score, eps, n_pool, n_approx)
        _check_invariants(score, eps, n_pool, n_approx, *out)


def test_budget_never_exceeded():
    # keys stored = n_pool, values stored = n_retain; together they never
    # exceed the footprint of (1 - p_c) n full pairs (Section 3.2).
    rng = np.random.default_rng(1)
    n = 1000
    for p_c in (0.25, 0.5, 0.75, 0.9):
        p_a = vo.pa_deploy(p_c)
        n_pool, n_approx = vo.budget_counts(n, p_c, p_a)
        tier, idx_r, idx_a = vo.route(rng.random((2, n)).astype(np.float32),
                                      rng.random((2, n)).astype(np.float32), n_pool, n_approx)
        keys = (tier != vo.EVICT).sum(axis=1)
        vals = (tier == vo.RETAIN).sum(axis=1)
        assert (keys + vals <= 2 * (1 - p_c) * n + 1e-9).all()
        assert (keys == n_pool).all() and (vals == n_pool - n_approx).all()


@pytest.mark.parametrize("seed", range(6))
def test_exhaustive_tiny(seed):
    # enumerate every pool and every split: the chosen pool maximises the score
    # sum, the chosen approx set minimises the eps sum inside it, and among the
    # optima the chosen index set is the lexicographically smallest.
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(6, 11))
    n_pool = int(rng.integers(1, n))
    n_approx = int(rng.integers(0, n_pool + 1))
    score = rng.integers(0, 3, size=(1, n)).astype(np.float32)
    eps = rng.integers(0, 3, size=(1, n)).astype(np.float32)
    tier, idx_r, idx_a = vo.route(score, eps, n_pool, n_approx)
    best = max(sum(score[0, list(c)]) for c in itertools.combinations(range(n), n_pool))
    optimal_pools = [c for c in itertools.combinations(range(n), n_pool) if sum(score[0, list(c)]) == best]
    pool = tuple(np.flatnonzero(tier[0] != vo.EVICT))
    assert pool == min(optimal_pools)
    best_a = min(sum(eps[0, list(c)]) for c in itertools.combinations(pool, n_approx))
    optimal_a = [c for c in itertools.combinations(pool, n_approx) if sum(eps[0, list(c)]) == best_a]
    assert tuple(idx_a[0]) == min(optimal_a)
    assert tuple(idx_r[0]) == tuple(sorted(set(pool) - set(idx_a[0])))


def test_all_equal_keys_take_lowest_indices():
    n, w = 40, 4
    score = np.full((1, n), 0.5, dtype=np.float32)
    score[0, n - w:] = np.inf                 # window columns
    eps = np.full((1, n), 2.0, dtype=np.float32)
    tier, idx_r, idx_a = vo.route(score, eps, 10, 3)
    pool = np.flatnonzero(tier[0] != vo.EVICT)
    np.testing.assert_array_equal(pool, list(range(6)) + list(range(n - w, n)))
    np.testing.assert_array_equal(idx_a[0], [0, 1, 2])


def test_direction_of_both_selections():
    score = np.array([[0.1, 0.9, 0.5, 0.7, 0.3]], dtype=np.float32)
    eps = np.array([[9.0, 5.0, 1.0, 3.0, 0.0]], dtype=np.float32)
    tier, idx_r, idx_a = vo.route(score, eps, 3, 1)
    # pool = highest score {1,3,2}; approx = lowest eps inside the pool = {2}
    np.testing.assert_array_equal(tier[0], [0, 2, 1, 2, 0])
    np.testing.assert_array_equal(idx_r[0], [1, 3])
    np.testing.assert_array_equal(idx_a[0], [2])


def test_infinite_scores_always_pooled():
    rng = np.random.default_rng(3)
    n, w = 64, 8
    score = rng.random((2, n)).astype(np.float32)
    score[:, n - w:] = np.inf
    tier, _, _ = vo.route(score, rng.random((2, n)).astype(np.float32), 12, 6)
    assert (tier[:, n - w:] != vo.EVICT).all()


def test_truncated_gaussian_closed_form():
    # Example 1 of Section 4 and its proof: with one-dimensional values and
    # signed residuals r ~ N(0, sigma^2) independent of importance, the mean
    # eps over the approximated tokens is
    #   sigma^2 * (1 - 2 z phi(z) / q),  q = n_a / n_p,  z = Phi^{-1}(1/2 + q/2).
    rng = np.random.default_rng(4)
    n, sigma = 400_000, 0.7
    p_c, p_a = 0.5, 0.25                      # pool 0.75, approx 0.5 of tokens
    n_pool, n_approx = vo.budget_counts(n, p_c, p_a)
    k = rng.standard_normal((1, n, 1))
    w_map = np.array([[[1.3]]])
    r = sigma * rng.standard_normal((1, n, 1))
    v = k @ w_map + r
    eps = vo.residual(k, v, w_map)
    score = rng.random((1, n)).astype(np.float32)
    tier, idx_r, idx_a = vo.route(score, eps, n_pool, n_approx)
    q = n_approx / n_pool
    z = norm.ppf(0.5 + q / 2)
    expect = sigma ** 2 * (1 - 2 * z * norm.pdf(z) / q)
    got = eps[0, idx_a[0]].astype(np.float64).mean()
    # standard error of the mean of r^2 over ~2e5 samples is ~ sigma^2 * 1e-3
    assert got == pytest.approx(expect, rel=0.01)
    # the paper's eta threshold: the largest |r| approximated is sigma * z
    assert math.sqrt(eps[0, idx_a[0]].max()) == pytest.approx(sigma * z, rel=0.01)
