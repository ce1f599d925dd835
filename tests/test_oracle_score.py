"""Pins for the oracle's base scorer (observation-window attention mass + pooling).

None of these re-type the oracle's own code path: they use closed forms, a
library softmax, a scalar pure-Python brute force, and invariants.
"""
import math

import numpy as np
import pytest
from scipy.special import softmax

from oracle import vector_oracle as vo


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_mass_sums_to_one_per_head():
    q = _rand(0, 6, 5, 8)          # Hq=6, w=5
    k = _rand(1, 2, 40, 8)         # Hkv=2, n=40
    mass = vo.attention_mass(q, k)
    assert mass.shape == (2, 40)
    np.testing.assert_allclose(mass.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    assert (mass >= 0).all()


def test_zero_query_closed_form():
    # q = 0: every causal row is uniform over the keys it may see, so
    # mass[t < n-w] = (1/w) sum_r 1/(n-w+r+1); pooling of a constant keeps it
    # in the interior and scales the edges by (kernel - missing)/kernel.
    n, w, kern, d = 50, 4, 7, 8
    q = np.zeros((2, w, d))
    k = _rand(2, 1, n, d)
    mass = vo.attention_mass(q, k)
    c = sum(1.0 / (n - w + r + 1) for r in range(w)) / w
    np.testing.assert_allclose(mass[0, : n - w], c, rtol=1e-13)
    # window column n-w+j is seen by rows r >= j only
    for j in range(w):
        cj = sum(1.0 / (n - w + r + 1) for r in range(j, w)) / w
        assert mass[0, n - w + j] == pytest.approx(cj, rel=1e-13)
    sc = vo.pool_scores(mass, w, kern)
    half = kern // 2
    n_prefix = n - w
    for t in range(n_prefix):
        missing = max(0, half - t) + max(0, t + half - (n_prefix - 1))
        assert sc[0, t] == pytest.approx(c * (kern - missing) / kern, rel=1e-12)
    assert np.isposinf(sc[0, n_prefix:]).all()


def test_single_row_reduces_to_textbook_softmax():
    n, d = 33, 16
    q = _rand(3, 1, 1, d)
    k = _rand(4, 1, n, d)
    mass = vo.attention_mass(q, k)
    ref = softmax((k[0] @ q[0, 0]) / math.sqrt(d))
    np.testing.assert_allclose(mass[0], ref, rtol=1e-12, atol=1e-15)
    sc = vo.score(q, k, window=1, pool_kernel=1)
    np.testing.assert_allclose(sc[0, : n - 1], ref[: n - 1].astype(np.float32), rtol=1e-6)
    assert np.isposinf(sc[0, n - 1])


def test_kernel_one_is_identity_on_prefix():
    q = _rand(5, 4, 3, 8)
    k = _rand(6, 2, 30, 8)
    mass = vo.attention_mass(q, k)
    sc = vo.pool_scores(mass, 3, 1)
    np.testing.assert_array_equal(sc[:, :27], mass[:, :27])


def test_brute_force_scalar_loops():
    # scalar re-derivation: every probability computed one by one
    n, w, d, hq, hkv, kern = 12, 3, 4, 4, 2, 3
    q = _rand(7, hq, w, d)
    k = _rand(8, hkv, n, d)
    g = hq // hkv
    mass = [[0.0] * n for _ in range(hkv)]
    for h in range(hkv):
        for gi in range(g):
            for r in range(w):
                pos = n - w + r
                logits = []
                for t in range(pos + 1):
                    dot = 0.0
                    for i in range(d):
                        dot += q[h * g + gi, r, i] * k[h, t, i]
                    logits.append(dot / math.sqrt(d))
                z = sum(math.exp(x) for x in logits)
                for t in range(pos + 1):
                    mass[h][t] += math.exp(logits[t]) / z / (g * w)
    got = vo.attention_mass(q, k)
    np.testing.assert_allclose(got, np.array(mass), rtol=1e-12, atol=1e-15)
    # pooled: brute-force neighbourhood sums over prefix columns only
    sc = vo.score(q, k, w, kern)
    for h in range(hkv):
        for t in range(n - w):
            acc = 0.0
            for j in range(-(kern // 2), kern // 2 + 1):
                if 0 <= t + j < n - w:
                    acc += mass[h][t + j]
            assert sc[h, t] == pytest.approx(acc / kern, rel=1e-6)


def test_causal_mask_last_column():
    # the last key is visible to the last window row only
    n, w, d = 20, 4, 8
    q = _rand(9, 1, w, d)
    k = _rand(10, 1, n, d)
    mass = vo.attention_mass(q, k)
    p_last = softmax((k[0] @ q[0, w - 1]) / math.sqrt(d))[n - 1]
    assert mass[0, n - 1] == pytest.approx(p_last / w, rel=1e-12)
    # and the first window row ignores keys after its own position
    p0 = softmax((k[0, : n - w + 1] @ q[0, 0]) / math.sqrt(d))
    only_row0 = vo.attention_mass(q[:, :1], k[:, : n - w + 1])
    np.testing.assert_allclose(only_row0[0], p0, rtol=1e-12)


def test_one_hot_limit():
    n, w, d = 64, 4, 8
    q = np.abs(_rand(11, 2, w, d)) + 0.5
    k = _rand(12, 1, n, d) * 0.01
    k[0, 17] = 1e3                      # aligned with every (positive) query
    mass = vo.attention_mass(q, k)
    assert mass[0, 17] == pytest.approx(1.0, abs=1e-12)


def test_group_and_row_permutation_invariance():
    q = _rand(13, 4, 5, 8)
    k = _rand(14, 2, 25, 8)
    base = vo.attention_mass(q, k)
    perm = q[[1, 0, 3, 2]]              # swap heads inside each group
    np.testing.assert_allclose(vo.attention_mass(perm, k), base, rtol=1e-13, atol=1e-16)


def test_scale_is_inverse_sqrt_d():
    # doubling d by zero-padding must change logits only through 1/sqrt(d)
    n, d = 10, 4
    q = _rand(15, 1, 1, d)
    k = _rand(16, 1, n, d)
    qp = np.concatenate([q, np.zeros_like(q)], axis=-1)
    kp = np.concatenate([k, np.zeros_like(k)], axis=-1)
    ref = softmax((k[0] @ q[0, 0]) / math.sqrt(2 * d))
    np.testing.assert_allclose(vo.attention_mass(qp, kp)[0], ref, rtol=1e-12)


def test_pooling_matches_library_convolution():
    rng = np.random.default_rng(17)
    mass = rng.random((3, 41))
    w, kern = 6, 5
    sc = vo.pool_scores(mass, w, kern)
    for h in range(3):
        ref = np.convolve(mass[h, : 41 - w], np.ones(kern) / kern, mode="same")
        np.testing.assert_allclose(sc[h, : 41 - w], ref, rtol=1e-13)
    assert np.isposinf(sc[:, 41 - w:]).all()


# ---- the maximum-pooling variant ----
def test_max_pooling_matches_library_filter_and_hand_values():
    from scipy.ndimage import maximum_filter1d
    rng = np.random.default_rng(19)
    mass = rng.random((3, 41))
    w = 6
    for kern in (1, 3, 5, 7, 13):
        sc = vo.pool_scores(mass, w, kern, "max")
        for h in range(3):
            ref = maximum_filter1d(mass[h, : 41 - w], size=kern, mode="constant", cval=0.0)
            np.testing.assert_array_equal(sc[h, : 41 - w], ref)
        assert np.isposinf(sc[:, 41 - w:]).all()
    # by hand: kernel 3 over the prefix (2, 9, 4, 1, 7), one window column that must not leak in
    hand = vo.pool_scores(np.array([[2.0, 9.0, 4.0, 1.0, 7.0, 100.0]]), 1, 3, "max")
    assert hand[0, :5].tolist() == [9.0, 9.0, 9.0, 7.0, 7.0] and np.isposinf(hand[0, 5])


def test_max_pooling_closed_forms():
    n, w, kern = 30, 4, 7
    half = kern // 2
    # a unit impulse spreads over the kernel's width at full height (average pooling: height 1/k)
    imp = np.zeros((1, n)); imp[0, 11] = 1.0
    mx = vo.pool_scores(imp, w, kern, "max")[0, : n - w]
    av = vo.pool_scores(imp, w, kern, "avg")[0, : n - w]
    want = np.zeros(n - w); want[11 - half: 11 + half + 1] = 1.0
    np.testing.assert_array_equal(mx, want)
    np.testing.assert_allclose(av, want / kern, rtol=1e-15)
    # an increasing sequence is shifted by half a kernel and clamped at the prefix's end
    ramp = np.arange(n, dtype=np.float64)[None, :]
    mx = vo.pool_scores(ramp, w, kern, "max")[0, : n - w]
    np.testing.assert_array_equal(mx, np.minimum(np.arange(n - w) + half, n - w - 1))
    # kernel 1 is the identity; the maximum dominates the average everywhere
    rng = np.random.default_rng(23)
    mass = rng.random((2, n))
    np.testing.assert_array_equal(vo.pool_scores(mass, w, 1, "max")[:, : n - w], mass[:, : n - w])
    assert (vo.pool_scores(mass, w, kern, "max")[:, : n - w] >= vo.pool_scores(mass, w, kern, "avg")[:, : n - w]).all()


def test_score_passes_the_pool_mode_through():
    q = _rand(41, 2, 3, 4)
    k = _rand(42, 1, 20, 4)
    mass = vo.attention_mass(q, k)
    np.testing.assert_array_equal(vo.score(q, k, 3, 5, "max"), vo.pool_scores(mass, 3, 5, "max").astype(np.float32))
    np.testing.assert_array_equal(vo.score(q, k, 3, 5), vo.pool_scores(mass, 3, 5, "avg").astype(np.float32))


# ---- the query-agnostic key-diversity score ----
def test_key_diversity_brute_force_and_invariances():
    rng = np.random.default_rng(31)
    k = rng.standard_normal((2, 50, 8)) + 1.5                       # a common direction plus spread
    got = vo.score_key_diversity(k)
    for h in range(2):
        unit = [row / np.sqrt((row * row).sum()) for row in k[h]]
        a = np.sum(unit, axis=0)
        a = a / np.sqrt((a * a).sum())
        for t in range(50):
            assert abs(got[h, t] + float(unit[t] @ a)) < 1e-6
    # positive rescaling of single keys changes nothing; a common rotation changes nothing
    scale = rng.random((2, 50, 1)) * 10 + 0.1
    np.testing.assert_allclose(vo.score_key_diversity(k * scale), got, atol=1e-6)
    qmat, _ = np.linalg.qr(rng.standard_normal((8, 8)))
    np.testing.assert_allclose(vo.score_key_diversity(k @ qmat), got, atol=1e-6)


def test_key_diversity_extremes_and_minority_cluster():
    same = np.tile(np.array([1.0, 2.0, -1.0, 0.5]), (1, 20, 1))
    np.testing.assert_allclose(vo.score_key_diversity(same), -1.0, atol=1e-6)   # all along the anchor
    k = np.tile(np.array([1.0, 0.0, 0.0, 0.0]), (1, 20, 1))
    k[0, 7] = [-3.0, 0.0, 0.0, 0.0]                                           # one key points the other way
    s = vo.score_key_diversity(k)
    assert abs(s[0, 7] - 1.0) < 1e-6 and np.allclose(np.delete(s[0], 7), -1.0, atol=1e-6)
    rng = np.random.default_rng(32)
    big = rng.standard_normal((1, 90, 6)) * 0.1 + np.array([3.0, 0, 0, 0, 0, 0])
    small = rng.standard_normal((1, 10, 6)) * 0.1 + np.array([0, 3.0, 0, 0, 0, 0])
    s = vo.score_key_diversity(np.concatenate([big, small], axis=1))
    assert s[0, 90:].min() > s[0, :90].max()                                  # the minority direction ranks highest
