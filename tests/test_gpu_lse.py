"""The scorer with the window rows' log-sum-exp handed in (what a prefill attention kernel
returns), so that only one pass over the keys remains.  The log-sum-exp is an input: the test
forms it in float64 with the library routine and rounds it to float32; expected outputs are the
oracle's, which knows nothing of it."""
import numpy as np
import pytest
from scipy.special import logsumexp

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
from paper_2605_23258_amd import pipeline as pl
import workloads as wl

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-3, 2e-3

CASES = {
    "bf16_d128": ("cfg2", dict(seq_len=2048, n_kv_heads=2, n_q_heads=8)),
    "f32_d64_ragged": ("cfg1", dict(seq_len=1000, window=20, n_q_heads=6, n_kv_heads=2)),
    "bf16_d128_ragged_maxpool": ("cfg2", dict(seq_len=1777, n_kv_heads=2, n_q_heads=8, window=24, pool_kernel=5, pool_mode="max")),
    "bf16_G8_w64_groups": ("cfg3", dict(seq_len=1536, n_kv_heads=2, n_q_heads=16, layers=1)),
    "n_equals_w": ("cfg1", dict(seq_len=32, window=32)),
}


def window_lse(q_win, k, stride=None):
    """lse[hq, r] over the keys row r may see; optionally laid out with `stride` floats per head."""
    q, kk = dg.widen(q_win), dg.widen(k)
    Hq, w, d = q.shape
    H, n, _ = kk.shape
    G = Hq // H
    out = np.full((Hq, stride or w), 7.0e3, dtype=np.float32)        # poison where nothing may be read
    for hq in range(Hq):
        s = q[hq] @ kk[hq // G].T / np.sqrt(d)
        for r in range(w):
            out[hq, r] = logsumexp(s[r, : n - w + r + 1])
    return out


def close(got, ref, what):
    err = np.abs(np.asarray(got, dtype=np.float64) - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


@pytest.mark.parametrize("name", list(CASES))
def test_score_residual_with_lse(name):
    base, over = CASES[name]
    cfg = dg.scaled(dg.CONFIGS[base], **over)
    li = wl.make_layer(cfg, 0)
    shape = pl.shape_of(cfg)
    n, w, H = cfg.seq_len, cfg.window, cfg.n_kv_heads
    n_r, n_a, n_p = cfg.counts()
    dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    ref_score = vo.score(dg.widen(li.q_win), dg.widen(li.k), w, cfg.pool_kernel, cfg.pool_mode)
    ref_eps = vo.residual(dg.widen(li.k), dg.widen(li.v), dg.widen(li.w_cal))
    ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a))
    for stride in (0, w + 5):
        lse = pl.to_device(window_lse(li.q_win, li.k, stride or None))
        score = torch.full((H, n), -1.0, device="cuda:0")
        eps = torch.full((H, n), -1.0, device="cuda:0")
        vb.vector_score_residual_lse(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], lse, stride, score, eps, ws)
        torch.cuda.synchronize()
        g = score.cpu().numpy()
        assert np.isposinf(g[:, n - w:]).all()
        close(g[:, : n - w].astype(np.float64) * n, ref_score[:, : n - w].astype(np.float64) * n, f"n*score (stride {stride})")
        close(eps.cpu().numpy(), ref_eps, "eps")
    # the whole pass: the routing of its own floats is the oracle's, the packed rows are those rows
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    out = pl.alloc_outputs(shape, n_p, n_a, n_r + 3, tdt)
    lse = pl.to_device(window_lse(li.q_win, li.k))
    vb.vector_compress_lse(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], lse, 0, n_p, n_a, out.score, out.eps, out.tier,
                           out.idx_retain if n_r else None, out.idx_approx if n_a else None, out.k_ret, out.v_ret, out.k_apx,
                           n_r + 3, ws)
    torch.cuda.synchronize()
    g_score, g_eps = out.score.cpu().numpy(), out.eps.cpu().numpy()
    close(g_score[:, : n - w].astype(np.float64) * n, ref_score[:, : n - w].astype(np.float64) * n, "n*score (one call)")
    tier, idx_r, idx_a = vo.route(g_score, g_eps, n_p, n_a)
    assert np.array_equal(out.tier.cpu().numpy(), tier)
    assert np.array_equal(out.idx_retain.cpu().numpy(), idx_r) and np.array_equal(out.idx_approx.cpu().numpy(), idx_a)
    rk, rv, ra = vo.compact(li.k, li.v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(out.k_ret)[:, :n_r], rk) and np.array_equal(pl.to_host(out.v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(out.k_apx)[:, :n_a], ra)


def test_lse_arguments_are_checked():
    cfg = dg.scaled(dg.CONFIGS["cfg2"], seq_len=512, n_kv_heads=1, n_q_heads=4)
    li = wl.make_layer(cfg, 0)
    shape = pl.shape_of(cfg)
    dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    n_r, n_a, n_p = cfg.counts()
    ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a))
    score = torch.full((1, 512), -1.0, device="cuda:0")
    eps = torch.full((1, 512), -1.0, device="cuda:0")
    lse = pl.to_device(window_lse(li.q_win, li.k))
    for bad_lse, bad_stride in ((None, 0), (lse, cfg.window - 1), (lse, -4)):
        with pytest.raises(vb.VectorError) as ei:
            vb.vector_score_residual_lse(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], bad_lse, bad_stride, score, eps, ws)
        assert ei.value.code == vb.VECTOR_ERR_ARG
    torch.cuda.synchronize()
    assert (score == -1.0).all() and (eps == -1.0).all(), "an error must not launch anything"


def test_rotated_keys_and_lse_together_single_and_batch():
    """What a production prefill has: keys cached after RoPE and the window rows' log-sum-exp from its
    attention kernel.  vector_compress_ex with both: scores and residuals against the oracle, the
    routing of its own floats exact; vector_compress_batch_ex (unequal sequences around an equal
    run) bit for bit the single calls."""
    theta = 500000.0
    cfg = dg.scaled(dg.CONFIGS["cfg2"], n_kv_heads=2, n_q_heads=8, window=32)
    lens = [900, 640, 640, 1500, 333]
    offset = 17
    H, Hq, d, w = cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.window
    layers = [wl.make_layer(dg.scaled(cfg, seq_len=n), layer=b, rope_theta=theta, rope_interleaved=False, pos_offset=offset)
              for b, n in enumerate(lens)]
    inv_freq, W = layers[0].extra["inv_freq"], layers[0].w_cal
    counts = [vo.budget_counts_frac(n, cfg.f_retain, cfg.f_approx) for n in lens]
    n_pool, n_approx = [c[0] for c in counts], [c[1] for c in counts]
    n_ret = [p - a for p, a in zip(n_pool, n_approx)]
    rope, keep_r = vb.make_rope(inv_freq, None, False, offset)
    lse_all = pl.to_device(np.stack([window_lse(li.q_win, li.k) for li in layers]))            # [batch, Hq, w]
    W_dev = pl.to_device(W)
    singles = []
    for b, li in enumerate(layers):
        n, n_p, n_a, n_r = lens[b], n_pool[b], n_approx[b], n_ret[b]
        s1 = pl.shape_of(cfg, seq_len=n)
        one = pl.alloc_outputs(s1, n_p, n_a, n_r, torch.bfloat16)
        ws1 = pl.alloc_workspace(vb.vector_compress_workspace_bytes(s1, n_p, n_a))
        opt = vb.make_options(rope, lse_all[b], 0)
        vb.vector_compress_ex(s1, opt, pl.to_device(li.q_win), pl.to_device(li.k), pl.to_device(li.v), W_dev, n_p, n_a, one.score, one.eps,
                              one.tier, one.idx_retain, one.idx_approx, one.k_ret, one.v_ret, one.k_apx, n_r, ws1)
        torch.cuda.synchronize()
        g_score, g_eps = one.score.cpu().numpy(), one.eps.cpu().numpy()
        ref_score = vo.score(dg.widen(li.q_win), dg.widen(li.k), w, cfg.pool_kernel)
        ref_eps = vo.residual(dg.widen(li.k), dg.widen(li.v), dg.widen(W), pos=li.extra["pos"], inv_freq=inv_freq, interleaved=False)
        close(g_score[:, : n - w].astype(np.float64) * n, ref_score[:, : n - w].astype(np.float64) * n, f"sequence {b} n*score")
        close(g_eps, ref_eps, f"sequence {b} eps")
        tier, idx_r, idx_a = vo.route(g_score, g_eps, n_p, n_a)
        assert np.array_equal(one.tier.cpu().numpy(), tier)
        assert np.array_equal(one.idx_retain.cpu().numpy(), idx_r) and np.array_equal(one.idx_approx.cpu().numpy(), idx_a)
        singles.append(one)
    tok0 = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ret0 = np.concatenate([[0], np.cumsum(n_ret)]).astype(np.int64)
    apx0 = np.concatenate([[0], np.cumsum(n_approx)]).astype(np.int64)
    T, R, A = int(tok0[-1]), int(ret0[-1]), int(apx0[-1])
    shape = pl.shape_of(cfg, seq_len=1)
    batch, keep = vb.make_batch(lens, n_pool, n_approx, n_ret)
    ws = pl.alloc_workspace(vb.vector_compress_batch_workspace_bytes(shape, batch))
    out = dict(score=torch.full((H * T,), -1.0, device="cuda:0"), eps=torch.full((H * T,), -1.0, device="cuda:0"),
               tier=torch.full((H * T,), 9, dtype=torch.uint8, device="cuda:0"),
               ir=torch.full((H * R,), -1, dtype=torch.int32, device="cuda:0"), ia=torch.full((H * A,), -1, dtype=torch.int32, device="cuda:0"),
               kr=torch.zeros((H * R, d), dtype=torch.bfloat16, device="cuda:0"), vr=torch.zeros((H * R, d), dtype=torch.bfloat16, device="cuda:0"),
               ka=torch.zeros((H * A, d), dtype=torch.bfloat16, device="cuda:0"))
    opt = vb.make_options(rope, lse_all, 0)
    vb.vector_compress_batch_ex(shape, batch, opt, pl.to_device(np.stack([li.q_win for li in layers])),
                                pl.to_device(np.concatenate([li.k for li in layers], axis=1)),
                                pl.to_device(np.concatenate([li.v for li in layers], axis=1)), W_dev, out["score"], out["eps"], out["tier"],
                                out["ir"], out["ia"], out["kr"], out["vr"], out["ka"], ws)
    torch.cuda.synchronize()
    for b, one in enumerate(singles):
        n, n_a, n_r = lens[b], n_approx[b], n_ret[b]
        t0, r0, a0 = int(tok0[b]), int(ret0[b]), int(apx0[b])
        what = f"sequence {b}"
        assert torch.equal(out["score"][H * t0: H * (t0 + n)].view(H, n), one.score), what
        assert torch.equal(out["eps"][H * t0: H * (t0 + n)].view(H, n), one.eps), what
        assert torch.equal(out["tier"][H * t0: H * (t0 + n)].view(H, n), one.tier), what
        assert torch.equal(out["ir"][H * r0: H * (r0 + n_r)].view(H, n_r), one.idx_retain), what
        assert torch.equal(out["ia"][H * a0: H * (a0 + n_a)].view(H, n_a), one.idx_approx), what
        assert torch.equal(out["kr"][H * r0: H * (r0 + n_r)].view(torch.int16), one.k_ret.view(torch.int16).reshape(H * n_r, d)), what
        assert torch.equal(out["vr"][H * r0: H * (r0 + n_r)].view(torch.int16), one.v_ret.view(torch.int16).reshape(H * n_r, d)), what
    # no options at all is the plain call
    vb.vector_compress_batch_ex(shape, batch, None, pl.to_device(np.stack([li.q_win for li in layers])),
                                pl.to_device(np.concatenate([li.k for li in layers], axis=1)),
                                pl.to_device(np.concatenate([li.v for li in layers], axis=1)), W_dev, out["score"], out["eps"], out["tier"],
                                out["ir"], out["ia"], out["kr"], out["vr"], out["ka"], ws)
    torch.cuda.synchronize()
    del keep, keep_r
