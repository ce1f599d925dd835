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
