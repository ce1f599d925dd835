"""Pins for the oracle's decode attention over the packed cache."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import vector_oracle as vo


def _case(seed, b=2, hq=4, hkv=2, d=8, n_r=9, n_a=7, cap=12):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((b, hq, d))
    k_ret = rng.standard_normal((b, hkv, cap, d))
    v_ret = rng.standard_normal((b, hkv, cap, d))
    k_apx = rng.standard_normal((b, hkv, n_a, d))
    w = rng.standard_normal((hkv, d, d)) / np.sqrt(d)
    length = np.full(b, n_r, dtype=np.int32)
    return q, k_ret, v_ret, length, k_apx, w


def test_no_approx_is_textbook_attention():
    q, k_ret, v_ret, length, k_apx, w = _case(0, n_a=0)
    out = vo.decode_attn(q, k_ret, v_ret, length, k_apx, w, 0.3)
    for b in range(2):
        for qh in range(4):
            h = qh // 2
            p = softmax(k_ret[b, h, :9] @ q[b, qh] * 0.3)
            np.testing.assert_allclose(out[b, qh], p @ v_ret[b, h, :9], rtol=1e-12)


def test_lossless_when_values_are_exactly_linear():
    # if the approximated tokens' true values equal k @ W, the result is
    # full attention over all pool tokens with their true values
    q, k_ret, v_ret, length, k_apx, w = _case(1)
    out = vo.decode_attn(q, k_ret, v_ret, length, k_apx, w, 0.35)
    for b in range(2):
        for qh in range(4):
            h = qh // 2
            keys = np.concatenate([k_ret[b, h, :9], k_apx[b, h]])
            vals = np.concatenate([v_ret[b, h, :9], k_apx[b, h] @ w[h]])
            p = softmax(keys @ q[b, qh] * 0.35)
            np.testing.assert_allclose(out[b, qh], p @ vals, rtol=1e-12)


def test_zero_query_gives_plain_mean():
    q, k_ret, v_ret, length, k_apx, w = _case(2)
    out = vo.decode_attn(np.zeros_like(q), k_ret, v_ret, length, k_apx, w, 1.0)
    for h in range(2):
        vals = np.concatenate([v_ret[0, h, :9], k_apx[0, h] @ w[h]])
        np.testing.assert_allclose(out[0, 2 * h], vals.mean(axis=0), rtol=1e-12)


def test_single_token():
    q, k_ret, v_ret, length, k_apx, w = _case(3, n_a=0)
    length[:] = 1
    out = vo.decode_attn(q, k_ret, v_ret, length, k_apx, w, 1.0)
    np.testing.assert_allclose(out[1, 3], v_ret[1, 1, 0], rtol=1e-13)
    # a single approximated token and no retained one: the rebuilt value itself
    q, k_ret, v_ret, length, k_apx, w = _case(4, n_a=1)
    length[:] = 0
    out = vo.decode_attn(q, k_ret, v_ret, length, k_apx, w, 1.0)
    np.testing.assert_allclose(out[0, 0], k_apx[0, 0, 0] @ w[0], rtol=1e-13)


def test_rows_beyond_length_are_ignored_and_lengths_are_per_sequence():
    q, k_ret, v_ret, length, k_apx, w = _case(5)
    length = np.array([9, 4], dtype=np.int32)
    base = vo.decode_attn(q, k_ret, v_ret, length, k_apx, w, 0.4)
    k2, v2 = k_ret.copy(), v_ret.copy()
    k2[0, :, 9:] = 1e6
    v2[0, :, 9:] = -1e6
    k2[1, :, 4:] = 1e6
    np.testing.assert_array_equal(vo.decode_attn(q, k2, v2, length, k_apx, w, 0.4), base)


def test_permutation_invariance_within_segments():
    q, k_ret, v_ret, length, k_apx, w = _case(6)
    base = vo.decode_attn(q, k_ret, v_ret, length, k_apx, w, 0.4)
    pr = np.random.default_rng(0).permutation(9)
    pa = np.random.default_rng(1).permutation(7)
    k2, v2 = k_ret.copy(), v_ret.copy()
    k2[:, :, :9], v2[:, :, :9] = k_ret[:, :, pr], v_ret[:, :, pr]
    out = vo.decode_attn(q, k2, v2, length, k_apx[:, :, pa], w, 0.4)
    np.testing.assert_allclose(out, base, rtol=1e-12, atol=1e-14)


def test_reassociation_identity():
    # sum_t p_t (k_t W) = (sum_t p_t k_t) W : checks the oracle's literal form
    q, k_ret, v_ret, length, k_apx, w = _case(7)
    out = vo.decode_attn(q, k_ret, v_ret, length, k_apx, w, 0.4)
    b, qh, h = 1, 2, 1
    keys = np.concatenate([k_ret[b, h, :9], k_apx[b, h]])
    p = softmax(keys @ q[b, qh] * 0.4)
    alt = p[:9] @ v_ret[b, h, :9] + (p[9:] @ k_apx[b, h]) @ w[h]
    np.testing.assert_allclose(out[b, qh], alt, rtol=1e-12)


def test_group_mapping_uses_consecutive_query_heads():
    # query heads 2h and 2h+1 read KV head h: zeroing KV head 1's values must
    # change query heads 2,3 only
    q, k_ret, v_ret, length, k_apx, w = _case(8, n_a=0)
    base = vo.decode_attn(q, k_ret, v_ret, length, k_apx, w, 0.4)
    v2 = v_ret.copy()
    v2[:, 1] = 0
    out = vo.decode_attn(q, k_ret, v2, length, k_apx, w, 0.4)
    np.testing.assert_array_equal(out[:, :2], base[:, :2])
    assert np.abs(out[:, 2:]).max() == 0.0


def test_compact_round_trip():
    rng = np.random.default_rng(9)
    k = rng.integers(0, 65535, size=(2, 30, 4)).astype(np.uint16)
    v = rng.integers(0, 65535, size=(2, 30, 4)).astype(np.uint16)
    score = rng.random((2, 30)).astype(np.float32)
    eps = rng.random((2, 30)).astype(np.float32)
    tier, idx_r, idx_a = vo.route(score, eps, 12, 5)
    k_ret, v_ret, k_apx = vo.compact(k, v, idx_r, idx_a)
    assert k_ret.shape == (2, 7, 4) and k_apx.shape == (2, 5, 4) and k_ret.dtype == np.uint16
    back_k = np.zeros_like(k)
    back_v = np.zeros_like(v)
    for h in range(2):
        back_k[h, idx_r[h]] = k_ret[h]
        back_k[h, idx_a[h]] = k_apx[h]
        back_v[h, idx_r[h]] = v_ret[h]
        pool = tier[h] != vo.EVICT
        assert np.array_equal(back_k[h][pool], k[h][pool])
        assert np.array_equal(back_v[h][tier[h] == vo.RETAIN], v[h][tier[h] == vo.RETAIN])
        assert not back_k[h][~pool].any()


def test_distortion_measure_prefers_three_way_routing_on_planted_data():
    # Section 4: with well-predicted values the importance-weighted loss of the
    # three-way split is below that of binary eviction at equal memory
    rng = np.random.default_rng(10)
    n, d, p_c, p_a = 2000, 16, 0.75, 0.125
    k = rng.standard_normal((1, n, d))
    w_true = rng.standard_normal((1, d, d)) / np.sqrt(d)
    v = k @ w_true + 0.05 * rng.standard_normal((1, n, d))
    wts = rng.dirichlet(np.full(n, 0.3))[None]
    eps = vo.residual(k, v, w_true)
    vsq = (v ** 2).sum(-1)
    n_pool, n_approx = vo.budget_counts(n, p_c, p_a)
    tier3, _, _ = vo.route(wts.astype(np.float32), eps, n_pool, n_approx)
    n_keep = int((1 - p_c) * n)
    tier2, _, _ = vo.route(wts.astype(np.float32), eps, n_keep, 0)
    assert vo.distortion(wts, tier3, eps, vsq)[0] < vo.distortion(wts, tier2, eps, vsq)[0]
