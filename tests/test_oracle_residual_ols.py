"""Pins for the reconstruction residual (Section 3.2, Step 2) and the
least-squares value map (Section 3.1)."""
import numpy as np
import pytest

from oracle import vector_oracle as vo
from paper_2605_23258_amd import datagen as dg
import workloads as wl


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_zero_noise_planted_map_gives_zero_residual():
    k = _rand(0, 2, 50, 16)
    w = _rand(1, 2, 16, 16) / 4
    v = np.einsum("hti,hij->htj", k, w)
    assert vo.residual(k, v, w).max() <= 1e-24


def test_zero_map_gives_value_norm():
    k, v = _rand(2, 1, 30, 8), _rand(3, 1, 30, 8)
    eps = vo.residual(k, v, np.zeros((1, 8, 8)))
    np.testing.assert_allclose(eps[0], np.linalg.norm(v[0], axis=1) ** 2, rtol=1e-6)


def test_identity_map():
    k = _rand(4, 1, 30, 8)
    assert vo.residual(k, k, np.eye(8)[None]).max() == 0.0


def test_row_convention_not_transposed():
    # an asymmetric map: k @ W and k @ W.T differ; eps must vanish for the first only
    k = _rand(5, 1, 20, 6)
    w = _rand(6, 1, 6, 6)
    v = k @ w
    assert vo.residual(k, v, w).max() < 1e-24
    assert vo.residual(k, v, np.swapaxes(w, 1, 2)).min() > 1e-3


def test_single_entry_by_hand():
    k = np.array([[[1.0, 2.0]]])
    v = np.array([[[0.5, -1.0]]])
    w = np.array([[[1.0, 0.0], [0.5, 2.0]]])      # k @ w = [2, 4]
    assert vo.residual(k, v, w)[0, 0] == pytest.approx((0.5 - 2) ** 2 + (-1 - 4) ** 2)


def test_quadratic_scaling():
    k, v, w = _rand(7, 1, 25, 8), _rand(8, 1, 25, 8), _rand(9, 1, 8, 8)
    np.testing.assert_allclose(vo.residual(3 * k, 3 * v, w), 9 * vo.residual(k, v, w), rtol=1e-6)


def test_chi_square_mean():
    # with the true map, eps_t / sigma_t^2 is chi-square with d degrees of freedom
    n, d = 20000, 16
    rng = np.random.default_rng(10)
    k = rng.standard_normal((1, n, d))
    w = rng.standard_normal((1, d, d)) / 4
    sig = 10.0 ** (-3 * rng.random((1, n)))
    v = k @ w + sig[..., None] * rng.standard_normal((1, n, d))
    ratio = vo.residual(k, v, w)[0] / (sig[0] ** 2 * d)
    assert ratio.mean() == pytest.approx(1.0, abs=5 * np.sqrt(2.0 / (n * d)))


def test_ols_recovers_planted_map_without_noise():
    k = _rand(11, 3, 4096, 32)
    w_true = _rand(12, 3, 32, 32) / np.sqrt(32)
    v = np.einsum("hti,hij->htj", k, w_true)
    assert np.abs(vo.ols_fit(k, v) - w_true).max() < 1e-10


def test_ols_normal_equations_orthogonality():
    k = _rand(13, 1, 500, 12)
    v = _rand(14, 1, 500, 12)
    w = vo.ols_fit(k, v)
    resid = v[0] - k[0] @ w[0]
    assert np.abs(k[0].T @ resid).max() < 1e-9 * np.abs(k[0].T @ v[0]).max()


def test_ols_is_a_minimum():
    k, v = _rand(15, 1, 200, 6), _rand(16, 1, 200, 6)
    w = vo.ols_fit(k, v)
    base = vo.residual(k, v, w).astype(np.float64).sum()
    rng = np.random.default_rng(17)
    for _ in range(5):
        pert = w + 1e-3 * rng.standard_normal(w.shape)
        assert vo.residual(k, v, pert).astype(np.float64).sum() > base


def test_generator_calibration_agrees_with_oracle_fit():
    # the input generator fits W with a library least-squares call; the oracle's
    # normal-equation fit on the same draw must give the same map
    cfg = dg.scaled(dg.CONFIGS["cfg1"], seq_len=256, cal_tokens=1024)
    w_true = np.random.default_rng(0).standard_normal((1, 64, 64)) / 8
    k_cal, v_cal, _, _ = dg._draw_kv(cfg, 0, cfg.cal_tokens, w_true, dg._TAG_CAL)
    np.testing.assert_allclose(wl.fit_w(k_cal, v_cal), vo.ols_fit(k_cal, v_cal), rtol=0, atol=1e-9)


def test_generator_recipe_shapes_and_planted_structure():
    cfg = dg.scaled(dg.CONFIGS["cfg2"], seq_len=512, n_kv_heads=2, n_q_heads=8)
    li = wl.make_layer(cfg, 0)
    assert li.k.dtype == np.uint16 and li.k.shape == (2, 512, 128)
    assert li.q_win.shape == (8, 32, 128) and li.w_cal.shape == (2, 128, 128)
    k, v = dg.widen(li.k), dg.widen(li.v)
    # residual under the true map ~ sigma^2 d (+ bf16 rounding noise of the stored tensors)
    eps = vo.residual(k, v, li.w_true).astype(np.float64)
    big = li.sigma > 0.3
    assert np.median(eps[big] / (li.sigma[big] ** 2 * 128)) == pytest.approx(1.0, abs=0.15)
    # heavy hitters: key norms about 4x
    norms = np.linalg.norm(k, axis=-1)
    assert norms[li.heavy].mean() / norms[~li.heavy].mean() == pytest.approx(4.0, rel=0.05)
    # regenerating gives identical bits
    li2 = wl.make_layer(cfg, 0)
    assert np.array_equal(li.k, li2.k) and np.array_equal(li.w_cal, li2.w_cal)
    assert not np.array_equal(li.k, wl.make_layer(cfg, 1).k)


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40], dtype=np.float32)
    bits = dg.f32_to_bf16_bits(x)
    back = dg.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to even (1.0);
    # 1 + 3*2^-8 is a tie between 1+2^-7 (odd) and 1+2^-6 (even)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    assert np.all(np.abs(back[:4] - x[:4]) <= np.abs(x[:4]) * 2.0 ** -8)


def test_r2_global_against_library_and_limits():
    from sklearn.metrics import r2_score
    k, w = _rand(20, 2, 200, 12), _rand(21, 2, 12, 12) / 3
    v = np.einsum("hti,hij->htj", k, w) + 0.5 * _rand(22, 2, 200, 12) + 3.0      # an offset: centring matters
    r = vo.r2_global(k, v, w)
    for h in range(2):
        lib = r2_score(v[h], k[h] @ w[h], multioutput="variance_weighted")
        assert abs(r["r2_centered"][h] - lib) < 1e-12
    assert (r["r2_uncentered"] > r["r2_centered"]).all()                        # the offset inflates the raw total
    exact = vo.r2_global(k, np.einsum("hti,hij->htj", k, w), w)
    assert np.allclose(exact["r2_centered"], 1.0) and np.allclose(exact["r2_uncentered"], 1.0)
    none = vo.r2_global(k, v, np.zeros_like(w))
    assert np.allclose(none["r2_uncentered"], 0.0)
    np.testing.assert_allclose(r["sse"], vo.residual(k, v, w).astype(np.float64).sum(axis=1), rtol=1e-6)
