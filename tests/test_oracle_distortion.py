"""Pins for the distortion measure and the quantities of Proposition 1 (Section 4)."""
import numpy as np

from oracle import vector_oracle as vo


def _case(seed, H=2, n=40, d=6):
    rng = np.random.default_rng(seed)
    w = rng.random((H, n)); w /= w.sum(axis=1, keepdims=True)
    v = rng.standard_normal((H, n, d))
    eps = rng.random((H, n)) * (v ** 2).sum(-1) * 0.5
    return w, v, eps


def test_extremes():
    w, v, eps = _case(0)
    n = w.shape[1]
    keep = np.full(w.shape, vo.RETAIN)
    r = vo.distortion_report(w, keep, eps, v)
    assert np.allclose(r["E"], 0) and np.allclose(r["w_bar"], 1.0) and np.all(r["w_star"] == 0)
    drop = np.full(w.shape, vo.EVICT)
    drop[:, 0] = vo.RETAIN
    r = vo.distortion_report(w, drop, eps, v)
    np.testing.assert_allclose(r["E"], 1 - w[:, 0], rtol=1e-12)
    # everything approximated with exact reconstruction costs nothing; with eps = ||v||^2 it costs as much as eviction
    ap = np.full(w.shape, vo.APPROX)
    assert np.allclose(vo.distortion_report(w, ap, np.zeros_like(eps), v)["E"], 0)
    r = vo.distortion_report(w, ap, (v ** 2).sum(-1), v)
    np.testing.assert_allclose(r["E"], 1.0, rtol=1e-12)
    np.testing.assert_allclose(r["r2_approx"], 0.0, atol=1e-12)


def test_matches_term_by_term_sum_and_older_function():
    w, v, eps = _case(1)
    tier = np.random.default_rng(2).integers(0, 3, w.shape)
    r = vo.distortion_report(w, tier, eps, v)
    for h in range(w.shape[0]):
        E = 0.0
        rels = []
        for t in range(w.shape[1]):
            if tier[h, t] == vo.EVICT:
                E += w[h, t]
            elif tier[h, t] == vo.APPROX:
                rel = eps[h, t] / float(v[h, t] @ v[h, t])
                E += w[h, t] * rel
                rels.append(rel)
        assert abs(r["E"][h] - E) < 1e-12
        assert abs(r["mu_approx"][h] - np.mean(rels)) < 1e-12
        assert abs(r["w_star"][h] - w.shape[1] * max(w[h, t] for t in range(w.shape[1]) if tier[h, t] == vo.EVICT)) < 1e-12
    np.testing.assert_allclose(r["E"], vo.distortion(w, tier, eps, (v ** 2).sum(-1)), rtol=1e-12)


def test_proposition_1_predicts_the_sign_of_the_change():
    """One head, equal weights inside the pool (so the mean pool weight is exact for the token that
    leaves the retention tier) and a constant relative error mu on every token.  Growing the
    approximation tier by one step moves the heaviest evicted token (weight w*) into the pool and
    approximates two more tokens; E falls exactly when 1 - mu exceeds w_bar / (w* + w_bar)."""
    n, n_pool, n_apx = 20, 10, 4
    for w_star_rel, mu in [(0.5, 0.2), (0.5, 0.45), (0.05, 0.2), (0.05, 0.02), (1.0, 0.49), (1.0, 0.51)]:
        w = np.empty(n)
        w[:n_pool] = 1.0                       # pool tokens, equal weight
        w[n_pool] = w_star_rel                 # the evicted token at the boundary
        w[n_pool + 1:] = 0.01 * w_star_rel     # the rest of the evicted tokens: lighter
        w /= w.sum()
        v = np.ones((1, n, 4))
        vsq = 4.0
        eps = np.full((1, n), mu * vsq)
        eps[0, :n_pool] += 1e-9 * np.arange(n_pool)         # a definite order inside the pool
        eps[0, n_pool] = mu * vsq - 1e-6                    # the newcomer is the easiest to rebuild: it is approximated
        score = w[None, :].copy()
        t0, _, _ = vo.route(score.astype(np.float32), eps.astype(np.float32), n_pool, n_apx)
        t1, _, _ = vo.route(score.astype(np.float32), eps.astype(np.float32), n_pool + 1, n_apx + 2)
        r0 = vo.distortion_report(w[None], t0, eps, v)
        r1 = vo.distortion_report(w[None], t1, eps, v)
        assert t1[0, n_pool] == vo.APPROX and (t1[0] == vo.APPROX).sum() == n_apx + 2
        improves = r1["E"][0] < r0["E"][0]
        predicted = r0["r2_approx"][0] > r0["threshold"][0]
        assert improves == predicted, (w_star_rel, mu, r0["E"][0], r1["E"][0], r0["threshold"][0])
        # and the size of the change is the proposition's: -w*(1 - mu) + mu * (pool weight)
        delta = -w[n_pool] * (1 - mu) + mu * w[0]
        assert abs((r1["E"][0] - r0["E"][0]) - delta) < 1e-6      # up to the tie-breaking perturbations above
