"""GPU parity of the post-RoPE entry points (Section 3.1, RoPE decoupling) against the oracle."""
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
THETA = 500000.0


def close(got, ref, what):
    err = np.abs(np.asarray(got, np.float64) - np.asarray(ref, np.float64))
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


CASES = {
    "bf16_d128": ("cfg2", dict(seq_len=2048, n_kv_heads=2, n_q_heads=8), False, 0),
    "bf16_d128_ragged_offset": ("cfg2", dict(seq_len=1777, n_kv_heads=2, n_q_heads=8, window=24), False, 31000),
    "bf16_d128_interleaved": ("cfg2", dict(seq_len=1100, n_kv_heads=1, n_q_heads=4), True, 7),
    "bf16_d64": ("cfg2", dict(seq_len=900, head_dim=64, n_kv_heads=2, n_q_heads=4, window=16), False, 0),
    "f32_d64": ("cfg1", dict(seq_len=1000, window=20, n_q_heads=6, n_kv_heads=2), False, 100),
    "f32_d64_interleaved": ("cfg1", dict(seq_len=640), True, 0),
}


@pytest.mark.parametrize("name", list(CASES))
def test_residual_and_score_on_rotated_keys(name):
    base, over, interleaved, offset = CASES[name]
    cfg = dg.scaled(dg.CONFIGS[base], **over)
    li = wl.make_layer(cfg, 0, rope_theta=THETA, rope_interleaved=interleaved, pos_offset=offset)
    inv_freq = li.extra["inv_freq"]
    H, n, w = cfg.n_kv_heads, cfg.seq_len, cfg.window
    n_r, n_a, n_p = cfg.counts()
    shape = pl.shape_of(cfg)
    dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    wide = {x: dg.widen(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    ref_eps = vo.residual(wide["k"], wide["v"], wide["w_cal"], pos=li.extra["pos"], inv_freq=inv_freq, interleaved=interleaved)
    ref_score = vo.score(wide["q_win"], wide["k"], w, cfg.pool_kernel)

    # positions implied by the row index plus an offset
    rope, keep = vb.make_rope(inv_freq, None, interleaved, offset)
    eps = torch.full((H, n), -1.0, device="cuda:0")
    vb.vector_residual_rope(shape, dev["k"], dev["v"], dev["w_cal"], rope, eps, ws)
    torch.cuda.synchronize()
    close(eps.cpu().numpy(), ref_eps, "eps (rope)")
    # without the un-rotation the residual is far off: the test would notice a path that skips it
    plain = torch.empty((H, n), device="cuda:0")
    vb.vector_residual(shape, dev["k"], dev["v"], dev["w_cal"], plain, ws)
    torch.cuda.synchronize()
    assert np.median(plain.cpu().numpy()) > 10 * np.median(ref_eps)

    # explicit positions, fused with the score
    pos_dev = pl.to_device(li.extra["pos"])
    rope2, keep2 = vb.make_rope(inv_freq, pos_dev, interleaved, 0)
    score = torch.full((H, n), -1.0, device="cuda:0")
    eps2 = torch.full((H, n), -1.0, device="cuda:0")
    vb.vector_score_residual_rope(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], rope2, score, eps2, ws)
    torch.cuda.synchronize()
    close(eps2.cpu().numpy(), ref_eps, "eps (rope, fused, explicit positions)")
    got = score.cpu().numpy()
    assert np.isposinf(got[:, n - w:]).all()
    close(got[:, : n - w].astype(np.float64) * n, ref_score[:, : n - w].astype(np.float64) * n, "n*score (rope call)")


@pytest.mark.parametrize("name", ["bf16_d128_ragged_offset", "bf16_d128_interleaved", "f32_d64"])
def test_one_call_compress_on_rotated_keys(name):
    """vector_compress_rope = vector_score_residual_rope + vector_route + vector_compact, bit for bit;
    the routing of its own floats is the oracle's and the packed rows are the cached (rotated) rows."""
    base, over, interleaved, offset = CASES[name]
    cfg = dg.scaled(dg.CONFIGS[base], **over)
    li = wl.make_layer(cfg, 0, rope_theta=THETA, rope_interleaved=interleaved, pos_offset=offset)
    H, n, w = cfg.n_kv_heads, cfg.seq_len, cfg.window
    n_r, n_a, n_p = cfg.counts()
    shape = pl.shape_of(cfg)
    dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    rope, keep = vb.make_rope(li.extra["inv_freq"], None, interleaved, offset)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    one = pl.alloc_outputs(shape, n_p, n_a, n_r + 2, tdt)
    ws1 = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a))
    vb.vector_compress_rope(shape, rope, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], n_p, n_a, one.score, one.eps, one.tier,
                            one.idx_retain, one.idx_approx, one.k_ret, one.v_ret, one.k_apx, n_r + 2, ws1)
    three = pl.alloc_outputs(shape, n_p, n_a, n_r + 2, tdt)
    ws3 = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    vb.vector_score_residual_rope(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], rope, three.score, three.eps, ws3)
    vb.vector_route(H, n, three.score, three.eps, n_p, n_a, three.tier, three.idx_retain, three.idx_approx, ws3)
    vb.vector_compact(shape, dev["k"], dev["v"], three.idx_retain, three.idx_approx, n_r, n_a, three.k_ret, three.v_ret, three.k_apx, n_r + 2)
    torch.cuda.synchronize()
    for f in ("score", "eps", "tier", "idx_retain", "idx_approx", "k_ret", "v_ret", "k_apx"):
        a, b = getattr(one, f), getattr(three, f)
        if a.dtype == torch.bfloat16:
            a, b = a.view(torch.int16), b.view(torch.int16)
        assert torch.equal(a, b), f
    wide = {x: dg.widen(getattr(li, x)) for x in ("k", "v", "w_cal")}
    close(one.eps.cpu().numpy(), vo.residual(wide["k"], wide["v"], wide["w_cal"], pos=li.extra["pos"], inv_freq=li.extra["inv_freq"],
                                             interleaved=interleaved), "eps (one call)")
    tier, idx_r, idx_a = vo.route(one.score.cpu().numpy(), one.eps.cpu().numpy(), n_p, n_a)
    assert np.array_equal(one.tier.cpu().numpy(), tier)
    assert np.array_equal(one.idx_retain.cpu().numpy(), idx_r) and np.array_equal(one.idx_approx.cpu().numpy(), idx_a)
    rk, rv, ra = vo.compact(li.k, li.v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(one.k_ret)[:, :n_r], rk) and np.array_equal(pl.to_host(one.v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(one.k_apx)[:, :n_a], ra)


@pytest.mark.parametrize("d,B,Hq,Hkv,n_r,n_a,interleaved", [
    (128, 2, 8, 2, 300, 200, False),
    (128, 1, 4, 4, 0, 65, True),
    (128, 3, 32, 8, 700, 900, False),
    (64, 2, 4, 2, 100, 77, False),
    (64, 1, 8, 1, 33, 40, True),
])
def test_decode_on_rotated_cache(d, B, Hq, Hkv, n_r, n_a, interleaved):
    rng = np.random.default_rng(d + n_a)
    inv_freq = dg.rotary_inv_freq(d, THETA)
    bf = lambda x: dg.f32_to_bf16_bits(np.asarray(x, np.float32))
    k_ret, v_ret = bf(rng.standard_normal((B, Hkv, max(n_r, 1), d))), bf(rng.standard_normal((B, Hkv, max(n_r, 1), d)))
    k_pre = rng.standard_normal((B, Hkv, n_a, d))
    pos = np.sort(rng.choice(32768, size=(B, Hkv, n_a)), axis=-1).astype(np.int32)
    k_apx = bf(dg.apply_rotary(k_pre, pos, inv_freq, interleaved))
    W = bf(rng.standard_normal((Hkv, d, d)) / np.sqrt(d))
    q = bf(rng.standard_normal((B, Hq, d)))
    t = [pl.to_device(x) for x in (k_ret, v_ret, k_apx, W, q, pos)]
    length = torch.full((B,), n_r, dtype=torch.int32, device="cuda:0")
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=max(n_r, 1), n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret, cache.k_apx, cache.W = (length.data_ptr(), t[0].data_ptr(), t[1].data_ptr(),
                                                                      t[2].data_ptr(), t[3].data_ptr())
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, seq_len=max(n_r + n_a, 64), window=1, pool_kernel=1, dtype=1)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_r + n_a, n_a, B))
    scale = 1.0 / np.sqrt(d)
    rope, keep = vb.make_rope(inv_freq, t[5], interleaved, 0)
    ref = vo.decode_attn(dg.widen(q), dg.widen(k_ret), dg.widen(v_ret), np.full(B, n_r), dg.widen(k_apx), dg.widen(W), scale,
                         pos_apx=pos, inv_freq=inv_freq, interleaved=interleaved)
    decode_check(cache, t[4], scale, ws, ref, "decode (rotary cache)", rope=rope)
    # the plain entry point on the same cache gives something else: the rotation matters here
    out2 = torch.empty((B, Hq, d), dtype=torch.bfloat16, device="cuda:0")
    vb.vector_decode_attn(cache, t[4], scale, out2, ws)
    torch.cuda.synchronize()
    assert np.abs(dg.widen(pl.to_host(out2)) - ref).max() > 10 * ATOL


@pytest.mark.parametrize("d,B,Hq,Hkv,n_r,n_a,interleaved", [
    (64, 2, 4, 2, 100, 77, False),
    (64, 1, 6, 1, 33, 140, True),
    (128, 2, 4, 2, 50, 65, False),
    (128, 1, 2, 2, 0, 40, True),
])
def test_decode_on_rotated_fp32_cache(d, B, Hq, Hkv, n_r, n_a, interleaved):
    """The fp32 (vector-ALU) decode kernel un-rotates approximated rows as well; a step with its
    append goes through the same kernel."""
    rng = np.random.default_rng(1000 + d + n_a)
    inv_freq = dg.rotary_inv_freq(d, THETA)
    f32 = lambda x: np.asarray(x, np.float32)
    cap = max(n_r, 1) + 2
    k_ret, v_ret = f32(rng.standard_normal((B, Hkv, cap, d))), f32(rng.standard_normal((B, Hkv, cap, d)))
    pos = np.sort(rng.choice(32768, size=(B, Hkv, n_a)), axis=-1).astype(np.int32)
    k_apx = f32(dg.apply_rotary(rng.standard_normal((B, Hkv, n_a, d)), pos, inv_freq, interleaved))
    W = f32(rng.standard_normal((Hkv, d, d)) / np.sqrt(d))
    q, k_new, v_new = f32(rng.standard_normal((B, Hq, d))), f32(rng.standard_normal((B, Hkv, d))), f32(rng.standard_normal((B, Hkv, d)))
    t = [pl.to_device(x) for x in (k_ret, v_ret, k_apx, W, q, pos, k_new, v_new)]
    length = torch.full((B,), n_r, dtype=torch.int32, device="cuda:0")
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, dtype=vb.VECTOR_F32, cap_retain=cap, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret, cache.k_apx, cache.W = (length.data_ptr(), t[0].data_ptr(), t[1].data_ptr(),
                                                                      t[2].data_ptr(), t[3].data_ptr())
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, seq_len=max(cap + n_a, 64), window=1, pool_kernel=1, dtype=0)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, cap + n_a, n_a, B))
    scale = 1.0 / np.sqrt(d)
    rope, keep = vb.make_rope(inv_freq, t[5], interleaved, 0)
    ref = vo.decode_attn(q, k_ret, v_ret, np.full(B, n_r), k_apx, W, scale, pos_apx=pos, inv_freq=inv_freq, interleaved=interleaved)
    out = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda:0")
    vb.vector_decode_attn_rope(cache, rope, t[4], scale, out, ws)
    torch.cuda.synchronize()
    close(out.cpu().numpy(), ref, "decode (rotary fp32 cache)")
    # the literal variant stays bf16-only and rotation-free
    with pytest.raises(vb.VectorError) as ei:
        vb.vector_decode_attn_rope(cache, rope, t[4], scale, out, ws, flags=vb.VECTOR_DECODE_LITERAL)
    assert ei.value.code == vb.VECTOR_ERR_DTYPE
    # one step with its append
    kk, vv = k_ret.copy(), v_ret.copy()
    kk[:, :, n_r], vv[:, :, n_r] = k_new, v_new
    ref = vo.decode_attn(q, kk, vv, np.full(B, n_r + 1), k_apx, W, scale, pos_apx=pos, inv_freq=inv_freq, interleaved=interleaved)
    vb.vector_decode_step_rope(cache, rope, t[4], t[6], t[7], scale, out, ws)
    torch.cuda.synchronize()
    close(out.cpu().numpy(), ref, "decode step (rotary fp32 cache)")
    assert length.cpu().numpy().tolist() == [n_r + 1] * B


def test_decode_step_on_rotated_cache():
    """vector_decode_step_rope: the new token's key is appended as cached (rotated), attends with
    the others, and only approximated rows are turned back."""
    d, B, Hq, Hkv, cap, n_a = 128, 2, 8, 2, 120, 90
    rng = np.random.default_rng(321)
    inv_freq = dg.rotary_inv_freq(d, THETA)
    bf = lambda x: dg.f32_to_bf16_bits(np.asarray(x, np.float32))
    k_ret, v_ret = bf(rng.standard_normal((B, Hkv, cap, d))), bf(rng.standard_normal((B, Hkv, cap, d)))
    pos = np.sort(rng.choice(32768, size=(B, Hkv, n_a)), axis=-1).astype(np.int32)
    k_apx = bf(dg.apply_rotary(rng.standard_normal((B, Hkv, n_a, d)), pos, inv_freq, False))
    W = bf(rng.standard_normal((Hkv, d, d)) / np.sqrt(d))
    q, k_new, v_new = bf(rng.standard_normal((B, Hq, d))), bf(rng.standard_normal((B, Hkv, d))), bf(rng.standard_normal((B, Hkv, d)))
    lens = np.array([cap - 1, 40], dtype=np.int32)
    kk, vv = k_ret.copy(), v_ret.copy()
    for b in range(B):
        kk[b, :, lens[b]] = k_new[b]
        vv[b, :, lens[b]] = v_new[b]
    scale = 1.0 / np.sqrt(d)
    ref = vo.decode_attn(dg.widen(q), dg.widen(kk), dg.widen(vv), lens + 1, dg.widen(k_apx), dg.widen(W), scale,
                         pos_apx=pos, inv_freq=inv_freq, interleaved=False)
    t = [pl.to_device(x) for x in (k_ret, v_ret, k_apx, W, q, pos, k_new, v_new)]
    length = pl.to_device(lens)
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=cap, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret, cache.k_apx, cache.W = (length.data_ptr(), t[0].data_ptr(), t[1].data_ptr(),
                                                                      t[2].data_ptr(), t[3].data_ptr())
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, seq_len=cap + n_a, window=1, pool_kernel=1, dtype=1)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, cap + n_a, n_a, B))
    rope, keep = vb.make_rope(inv_freq, t[5], False, 0)
    out = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda:0")
    vb.vector_decode_step_rope(cache, rope, t[4], t[6], t[7], scale, out, ws, flags=vb.VECTOR_DECODE_OUT_F32)
    torch.cuda.synchronize()
    close(out.cpu().numpy(), ref, "decode step (rotary cache)")
    assert length.cpu().numpy().tolist() == (lens + 1).tolist()
    assert np.array_equal(pl.to_host(t[0]), kk) and np.array_equal(pl.to_host(t[1]), vv)


def test_full_size_layer_and_decode_step():
    """The 32k-token layer and the batch-16 decode shape of the benchmark, read as post-RoPE caches."""
    cfg = dg.CONFIGS["cfg3"]
    li = wl.make_layer(cfg, 3, rope_theta=THETA)
    inv_freq = li.extra["inv_freq"]
    H, n, d = cfg.n_kv_heads, cfg.seq_len, cfg.head_dim
    n_r, n_a, n_p = cfg.counts()
    shape = pl.shape_of(cfg)
    dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    rope, keep = vb.make_rope(inv_freq, None, False, 0)
    score = torch.empty((H, n), device="cuda:0")
    eps = torch.empty((H, n), device="cuda:0")
    vb.vector_score_residual_rope(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], rope, score, eps, ws)
    torch.cuda.synchronize()
    ref_eps = vo.residual(dg.widen(li.k), dg.widen(li.v), dg.widen(li.w_cal), inv_freq=inv_freq)
    close(eps.cpu().numpy(), ref_eps, "eps (rope, 32k layer)")
    # decode: caches cut from this layer by the oracle's routing of the GPU's floats
    B, Hq = 4, cfg.n_q_heads
    _, idx_r, idx_a = vo.route(score.cpu().numpy(), eps.cpu().numpy(), n_p, n_a)
    rk, rv, ra = vo.compact(li.k, li.v, idx_r, idx_a)
    rng = np.random.default_rng(11)
    q = dg.f32_to_bf16_bits(rng.standard_normal((B, Hq, d)).astype(np.float32))
    k_ret, v_ret, k_apx = (np.broadcast_to(x, (B,) + x.shape).copy() for x in (rk, rv, ra))
    pos = np.broadcast_to(idx_a.astype(np.int32), (B,) + idx_a.shape).copy()
    t = [pl.to_device(x) for x in (k_ret, v_ret, k_apx, q, pos)]
    length = torch.full((B,), n_r, dtype=torch.int32, device="cuda:0")
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=n_r, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret, cache.k_apx, cache.W = (length.data_ptr(), t[0].data_ptr(), t[1].data_ptr(),
                                                                      t[2].data_ptr(), dev["w_cal"].data_ptr())
    wsd = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, B))
    scale = 1.0 / np.sqrt(d)
    rope_d, keep_d = vb.make_rope(inv_freq, t[4], False, 0)
    ref = vo.decode_attn(dg.widen(q), dg.widen(k_ret), dg.widen(v_ret), np.full(B, n_r), dg.widen(k_apx), dg.widen(li.w_cal), scale,
                         pos_apx=pos, inv_freq=inv_freq)
    decode_check(cache, t[3], scale, wsd, ref, "decode (rotary cache, full layer)", rope=rope_d)
