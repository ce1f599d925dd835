"""Pins for the rotary un-rotation that precedes the value map on post-RoPE keys
(Section 3.1, "RoPE Decoupling")."""
import math

import numpy as np
import pytest

from oracle import vector_oracle as vo
from paper_2605_23258_amd import datagen as dg


def _inv_freq(d, theta=10000.0):
    return theta ** (-np.arange(d // 2) * 2.0 / d)


def _dense_rotation(pos, inv_freq, d, interleaved):
    """R_m as a dense d x d matrix, one 2 x 2 block per pair, built with math.cos / math.sin."""
    R = np.zeros((d, d))
    for i, f in enumerate(inv_freq):
        ia, ib = (2 * i, 2 * i + 1) if interleaved else (i, i + d // 2)
        c, s = math.cos(pos * f), math.sin(pos * f)
        R[ia, ia], R[ia, ib], R[ib, ia], R[ib, ib] = c, -s, s, c
    return R


def test_quarter_turn_by_hand():
    # one pair, angle pi/2 at position 1: the forward rotation sends (1, 0) to (0, 1), so the
    # cached row (0, 1) comes back as (1, 0)
    out = vo.rope_unrotate(np.array([[0.0, 1.0]]), np.array([1]), np.array([math.pi / 2]))
    np.testing.assert_allclose(out, [[1.0, 0.0]], atol=1e-15)
    out = vo.rope_unrotate(np.array([[0.0, 1.0]]), np.array([3]), np.array([math.pi / 2]))   # three quarter turns
    np.testing.assert_allclose(out, [[-1.0, 0.0]], atol=1e-15)


@pytest.mark.parametrize("interleaved", [False, True])
def test_matches_inverse_of_dense_block_rotation(interleaved):
    d, n = 8, 6
    rng = np.random.default_rng(0)
    k_pre = rng.standard_normal((n, d))
    pos = np.array([0, 1, 5, 17, 1000, 31999])
    f = _inv_freq(d)
    k_post = np.stack([_dense_rotation(m, f, d, interleaved) @ k_pre[t] for t, m in enumerate(pos)])
    back = vo.rope_unrotate(k_post, pos, f, interleaved)
    np.testing.assert_allclose(back, k_pre, atol=1e-9)
    for t, m in enumerate(pos):                      # and it is the matrix inverse, not merely a transpose guess
        ref = np.linalg.solve(_dense_rotation(m, f, d, interleaved), k_post[t])
        np.testing.assert_allclose(back[t], ref, atol=1e-9)


def test_position_zero_is_identity_and_norms_are_kept():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 10, 16))
    f = _inv_freq(16)
    np.testing.assert_array_equal(vo.rope_unrotate(x, np.zeros((3, 10), int), f), x)
    y = vo.rope_unrotate(x, rng.integers(0, 5000, (3, 10)), f)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)


def test_rotated_dot_products_depend_on_position_difference_only():
    # <R_m a, R_n b> = <a, R_{n-m} b>: un-rotating both sides by a common shift leaves it unchanged
    rng = np.random.default_rng(2)
    a, b = rng.standard_normal((1, 12)), rng.standard_normal((1, 12))
    f = _inv_freq(12)
    fwd = lambda x, m: vo.rope_unrotate(x, np.array([-m]), f)          # turning back by -m is turning forward by m
    d1 = fwd(a, 7)[0] @ fwd(b, 19)[0]
    d2 = fwd(a, 107)[0] @ fwd(b, 119)[0]
    assert abs(d1 - d2) < 1e-10
    assert abs(d1 - a[0] @ b[0]) > 1e-3                                # and it is not position-free


def test_interleaved_is_half_split_under_the_pair_permutation():
    rng = np.random.default_rng(3)
    d = 16
    x = rng.standard_normal((5, d))
    pos = np.array([3, 9, 27, 81, 243])
    f = _inv_freq(d)
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])    # interleaved -> half-split order
    a = vo.rope_unrotate(x, pos, f, interleaved=True)[:, perm]
    b = vo.rope_unrotate(x[:, perm], pos, f, interleaved=False)
    np.testing.assert_allclose(a, b, atol=1e-14)


def test_residual_on_rotated_keys_equals_residual_on_plain_keys():
    # values are linear in the pre-RoPE keys; the cache holds post-RoPE keys
    rng = np.random.default_rng(4)
    H, n, d = 2, 40, 8
    k_pre = rng.standard_normal((H, n, d))
    w = rng.standard_normal((H, d, d)) / 3
    v = k_pre @ w + 0.1 * rng.standard_normal((H, n, d))
    f = _inv_freq(d, 500000.0)
    pos = np.arange(n) + 100
    k_post = np.stack([[_dense_rotation(m, f, d, False) @ k_pre[h, t] for t, m in enumerate(pos)] for h in range(H)])
    plain = vo.residual(k_pre, v, w)
    np.testing.assert_allclose(vo.residual(k_post, v, w, pos=pos, inv_freq=f), plain, rtol=1e-6)
    assert np.abs(vo.residual(k_post, v, w) - plain).max() > 1e-2       # skipping the un-rotation is visible
    # default positions are the row indices
    k_post0 = np.stack([[_dense_rotation(t, f, d, False) @ k_pre[h, t] for t in range(n)] for h in range(H)])
    np.testing.assert_allclose(vo.residual(k_post0, v, w, inv_freq=f), plain, rtol=1e-6)


def test_decode_rebuilds_values_from_unrotated_keys_but_scores_with_cached_keys():
    rng = np.random.default_rng(5)
    B, Hq, H, d, n_r, n_a = 2, 4, 2, 8, 5, 7
    f = _inv_freq(d)
    q = rng.standard_normal((B, Hq, d))
    k_ret, v_ret = rng.standard_normal((B, H, n_r, d)), rng.standard_normal((B, H, n_r, d))
    k_pre = rng.standard_normal((B, H, n_a, d))
    pos = rng.integers(0, 3000, (B, H, n_a))
    k_post = np.empty_like(k_pre)
    for b in range(B):
        for h in range(H):
            for t in range(n_a):
                k_post[b, h, t] = _dense_rotation(pos[b, h, t], f, d, False) @ k_pre[b, h, t]
    w = rng.standard_normal((H, d, d)) / 3
    got = vo.decode_attn(q, k_ret, v_ret, np.full(B, n_r), k_post, w, 0.3, pos_apx=pos, inv_freq=f)
    # by hand: logits from the cached keys, values of approximated tokens from the plain keys
    for b in range(B):
        for qh in range(Hq):
            h = qh // (Hq // H)
            keys = np.concatenate([k_ret[b, h], k_post[b, h]])
            vals = np.concatenate([v_ret[b, h], k_pre[b, h] @ w[h]])
            s = keys @ q[b, qh] * 0.3
            p = np.exp(s - s.max()); p /= p.sum()
            np.testing.assert_allclose(got[b, qh], p @ vals, atol=1e-9)
    # all positions zero: identical to the call without rotary arguments
    z = vo.decode_attn(q, k_ret, v_ret, np.full(B, n_r), k_post, w, 0.3, pos_apx=np.zeros_like(pos), inv_freq=f)
    np.testing.assert_allclose(z, vo.decode_attn(q, k_ret, v_ret, np.full(B, n_r), k_post, w, 0.3), atol=1e-12)
