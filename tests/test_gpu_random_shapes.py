"""Seeded sweep over small random shapes: the whole compression pass and decode attention
against the oracle, to reach corners the hand-picked cases miss (odd head counts, windows that
are not multiples of 32, tails of every length, pools of all sizes)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
import workloads as wl
from paper_2605_23258_amd import pipeline as pl
from parity_util import decode_check

pytestmark = pytest.mark.gpu
ATOL, RTOL = 1e-3, 2e-3


def _close(got, ref, what):
    err = np.abs(np.asarray(got, np.float64) - np.asarray(ref, np.float64))
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


def _compress_shapes():
    rng = np.random.default_rng(2024)
    out = []
    for i in range(28):
        d = int(rng.choice([64, 128]))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        hkv = int(rng.integers(1, 4))
        g = int(rng.choice([1, 2, 3, 4, 8]))
        n = int(rng.integers(40, 2600))
        w = int(rng.integers(1, min(n, 64 // max(1, g // 4)) + 1))
        pool = int(rng.choice([1, 3, 5, 7, 9]))
        f_r, f_a = float(rng.random() * 0.4), float(rng.random() * 0.4)
        out.append((i, dtype, d, hkv, g, n, w, pool, f_r, f_a))
    return out


@pytest.mark.parametrize("case", _compress_shapes(), ids=lambda c: f"{c[0]}-{c[1]}-d{c[2]}-h{c[3]}g{c[4]}-n{c[5]}-w{c[6]}-k{c[7]}")
def test_compression_pass_on_random_shape(case):
    i, dtype, d, hkv, g, n, w, pool, f_r, f_a = case
    base = dg.CONFIGS["cfg2" if dtype == "bf16" else "cfg1"]
    cfg = dg.scaled(base, head_dim=d, n_kv_heads=hkv, n_q_heads=hkv * g, seq_len=n, window=w, pool_kernel=pool,
                    f_retain=f_r, f_approx=f_a, cal_tokens=512, heavy_frac=0.05)
    li = wl.make_layer(cfg, i)
    n_r, n_a, n_p = cfg.counts()
    if n_p < 1:
        n_r, n_a, n_p = 1, 0, 1
    shape = pl.shape_of(cfg)
    dev = {k: pl.to_device(getattr(li, k)) for k in ("q_win", "k", "v", "w_cal")}
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    out = pl.alloc_outputs(shape, n_p, n_a, n_r + 2, torch.bfloat16 if dtype == "bf16" else torch.float32)
    pl.compress_layer(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], n_p, n_a, out, ws)
    torch.cuda.synchronize()
    wide = {k: dg.widen(getattr(li, k)) for k in ("q_win", "k", "v", "w_cal")}
    g_score, g_eps = out.score.cpu().numpy(), out.eps.cpu().numpy()
    assert np.isposinf(g_score[:, n - w:]).all()
    _close(g_score[:, : n - w].astype(np.float64) * n, vo.score(wide["q_win"], wide["k"], w, pool)[:, : n - w].astype(np.float64) * n, "n*score")
    _close(g_eps, vo.residual(wide["k"], wide["v"], wide["w_cal"]), "eps")
    tier, idx_r, idx_a = vo.route(g_score, g_eps, n_p, n_a)
    assert np.array_equal(out.tier.cpu().numpy(), tier)
    if n_r:
        assert np.array_equal(out.idx_retain.cpu().numpy()[:, :n_r], idx_r)
    if n_a:
        assert np.array_equal(out.idx_approx.cpu().numpy()[:, :n_a], idx_a)
    rk, rv, ra = vo.compact(li.k, li.v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(out.k_ret)[:, :n_r], rk) and np.array_equal(pl.to_host(out.v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(out.k_apx)[:, :n_a], ra)


def _decode_shapes():
    rng = np.random.default_rng(77)
    out = []
    for i in range(24):
        d = int(rng.choice([64, 128]))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        B = int(rng.integers(1, 4))
        hkv = int(rng.integers(1, 5))
        g = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8]))
        cap = int(rng.integers(1, 700))
        n_a = int(rng.integers(0, 700))
        out.append((i, dtype, d, B, hkv, g, cap, n_a))
    return out


@pytest.mark.parametrize("case", _decode_shapes(), ids=lambda c: f"{c[0]}-{c[1]}-d{c[2]}-b{c[3]}h{c[4]}g{c[5]}-r{c[6]}-a{c[7]}")
def test_decode_on_random_shape(case):
    i, dtype, d, B, hkv, g, cap, n_a = case
    rng = np.random.default_rng(1000 + i)
    hq = hkv * g
    is_bf = dtype == "bf16"
    store = (lambda x: dg.f32_to_bf16_bits(np.asarray(x, np.float32))) if is_bf else (lambda x: np.asarray(x, np.float32))
    k_ret, v_ret = store(rng.standard_normal((B, hkv, cap, d))), store(rng.standard_normal((B, hkv, cap, d)))
    k_apx = store(rng.standard_normal((B, hkv, max(n_a, 1), d)))[:, :, :n_a]
    W = store(rng.standard_normal((hkv, d, d)) / np.sqrt(d))
    q = store(rng.standard_normal((B, hq, d)) * 2.0)
    lens = rng.integers(0, cap + 1, size=B).astype(np.int32)
    if n_a == 0:
        lens = np.maximum(lens, 1)
    t = dict(k_ret=pl.to_device(np.ascontiguousarray(k_ret)), v_ret=pl.to_device(np.ascontiguousarray(v_ret)),
             k_apx=pl.to_device(np.ascontiguousarray(k_apx)) if n_a else None, W=pl.to_device(W), q=pl.to_device(q),
             lens=pl.to_device(lens))
    cache = vb.Cache(batch=B, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, dtype=vb.VECTOR_BF16 if is_bf else vb.VECTOR_F32,
                     cap_retain=cap, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret = t["lens"].data_ptr(), t["k_ret"].data_ptr(), t["v_ret"].data_ptr()
    cache.k_apx = t["k_apx"].data_ptr() if n_a else None
    cache.W = t["W"].data_ptr()
    shape = vb.Shape(n_q_heads=hq, n_kv_heads=hkv, head_dim=d, seq_len=max(cap + n_a, 64), window=1, pool_kernel=1,
                     dtype=cache.dtype)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, cap + n_a, n_a, B))
    scale = 1.0 / np.sqrt(d)
    ref = vo.decode_attn(dg.widen(q), dg.widen(k_ret), dg.widen(v_ret), lens, dg.widen(k_apx) if n_a else np.zeros((B, hkv, 0, d)),
                         dg.widen(W), scale)
    decode_check(cache, t["q"], scale, ws, ref)


def _route_cases():
    rng = np.random.default_rng(909)
    out = []
    for i in range(36):
        n = int(rng.choice([7, 63, 64, 65, 1000, 4095, 4096, 4100, 9000, 32767, 32768, 33000, 50000, 70001]))
        n_pool = int(rng.integers(0, n + 1))
        n_approx = int(rng.integers(0, n_pool + 1))
        kind = int(rng.integers(0, 5))
        out.append((i, n, n_pool, n_approx, kind))
    return out


@pytest.mark.parametrize("case", _route_cases(), ids=lambda c: f"{c[0]}-n{c[1]}-p{c[2]}-a{c[3]}-k{c[4]}")
def test_route_on_random_distributions(case):
    """Bit-exact routing on value distributions that stress the radix digits: few distinct values,
    values that differ only in the low mantissa bits, negative and infinite entries, denormals."""
    i, n, n_pool, n_approx, kind = case
    rng = np.random.default_rng(5000 + i)
    H = int(rng.integers(1, 4))
    if kind == 0:
        score, eps = rng.random((H, n)), rng.random((H, n))
    elif kind == 1:                                  # a handful of distinct values: ties everywhere
        score, eps = rng.integers(0, 3, (H, n)) * 0.5, rng.integers(0, 4, (H, n)) * 1.0
    elif kind == 2:                                  # differences in the last mantissa bits only
        score = 1.0 + rng.integers(0, 50, (H, n)) * 2.0 ** -23
        eps = 3.0 + rng.integers(0, 50, (H, n)) * 2.0 ** -22
    elif kind == 3:                                  # signs, infinities, zeros of both signs
        score = rng.standard_normal((H, n)) * 10.0 ** rng.integers(-30, 30, (H, n))
        score[:, :: 11] = np.inf
        score[:, 5:: 13] = -0.0
        eps = np.abs(rng.standard_normal((H, n))) * 10.0 ** rng.integers(-20, 20, (H, n))
        eps[:, 3:: 17] = np.inf
        eps[:, 1:: 19] = 0.0
    else:                                            # denormals and tiny values
        score = rng.random((H, n)) * 1e-41
        eps = rng.random((H, n)) * 1e-40
    score, eps = score.astype(np.float32), eps.astype(np.float32)
    shape = vb.Shape(n_q_heads=H, n_kv_heads=H, head_dim=64, seq_len=n, window=1, pool_kernel=1, dtype=0)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_pool, n_approx, 1))
    tier = torch.full((H, n), 77, dtype=torch.uint8, device="cuda:0")
    idx_r = torch.full((H, max(n_pool - n_approx, 1)), -1, dtype=torch.int32, device="cuda:0")
    idx_a = torch.full((H, max(n_approx, 1)), -1, dtype=torch.int32, device="cuda:0")
    vb.vector_route(H, n, pl.to_device(score), pl.to_device(eps), n_pool, n_approx, tier,
                    idx_r if n_pool - n_approx else None, idx_a if n_approx else None, ws)
    torch.cuda.synchronize()
    r_tier, r_ir, r_ia = vo.route(score, eps, n_pool, n_approx)
    assert np.array_equal(tier.cpu().numpy(), r_tier)
    assert np.array_equal(idx_r.cpu().numpy()[:, : n_pool - n_approx], r_ir)
    assert np.array_equal(idx_a.cpu().numpy()[:, :n_approx], r_ia)


@pytest.mark.parametrize("q_scale", [0.0, 30.0, 300.0])
def test_decode_with_flat_and_peaked_softmax(q_scale):
    """q = 0 gives the plain mean over live and approximated rows; a large q makes the softmax
    one-hot (running maxima jump, almost every weight underflows)."""
    rng = np.random.default_rng(int(q_scale) + 1)
    B, hkv, g, d, cap, n_a = 2, 2, 4, 128, 900, 700
    bf = lambda x: dg.f32_to_bf16_bits(np.asarray(x, np.float32))
    k_ret, v_ret = bf(rng.standard_normal((B, hkv, cap, d))), bf(rng.standard_normal((B, hkv, cap, d)))
    k_apx = bf(rng.standard_normal((B, hkv, n_a, d)))
    W = bf(rng.standard_normal((hkv, d, d)) / np.sqrt(d))
    q = bf(rng.standard_normal((B, hkv * g, d)) * q_scale)
    lens = np.array([cap, cap - 123], np.int32)
    t = [pl.to_device(x) for x in (k_ret, v_ret, k_apx, W, q, lens)]
    cache = vb.Cache(batch=B, n_q_heads=hkv * g, n_kv_heads=hkv, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=cap, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret, cache.k_apx, cache.W = (t[5].data_ptr(), t[0].data_ptr(), t[1].data_ptr(),
                                                                      t[2].data_ptr(), t[3].data_ptr())
    shape = vb.Shape(n_q_heads=hkv * g, n_kv_heads=hkv, head_dim=d, seq_len=cap + n_a, window=1, pool_kernel=1, dtype=1)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, cap + n_a, n_a, B))
    scale = 1.0 / np.sqrt(d)
    ref = vo.decode_attn(dg.widen(q), dg.widen(k_ret), dg.widen(v_ret), lens, dg.widen(k_apx), dg.widen(W), scale)
    for flags in (0, vb.VECTOR_DECODE_LITERAL):
        decode_check(cache, t[4], scale, ws, ref, f"flags {flags}", flags=flags)


@pytest.mark.parametrize("q_scale", [0.0, 6.0, 40.0])
def test_score_with_flat_and_peaked_attention(q_scale):
    """q = 0: every window row spreads its mass evenly over what it sees; large q: almost all of a
    row's mass sits on one key, row maxima are far apart and jump between tiles."""
    cfg = dg.scaled(dg.CONFIGS["cfg2"], seq_len=3000, n_kv_heads=2, n_q_heads=8, window=32)
    li = wl.make_layer(cfg, 1)
    q = dg.f32_to_bf16_bits((dg.widen(li.q_win) * q_scale).astype(np.float32))
    shape = pl.shape_of(cfg)
    n_r, n_a, n_p = cfg.counts()
    n, w = cfg.seq_len, cfg.window
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    score = torch.empty((cfg.n_kv_heads, n), device="cuda:0")
    eps = torch.empty((cfg.n_kv_heads, n), device="cuda:0")
    vb.vector_score_residual(shape, pl.to_device(q), pl.to_device(li.k), pl.to_device(li.v), pl.to_device(li.w_cal), score, eps, ws)
    torch.cuda.synchronize()
    ref = vo.score(dg.widen(q), dg.widen(li.k), w, cfg.pool_kernel)
    got = score.cpu().numpy()
    assert np.isfinite(got[:, : n - w]).all()
    _close(got[:, : n - w].astype(np.float64) * n, ref[:, : n - w].astype(np.float64) * n, f"n*score (q x {q_scale})")
