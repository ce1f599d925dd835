"""GPU parity of the distortion diagnostics (Section 4) against the oracle's report."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
import workloads as wl
from paper_2605_23258_amd import pipeline as pl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("base,over", [
    ("cfg2", dict(seq_len=4096, n_kv_heads=2, n_q_heads=8)),
    ("cfg2", dict(seq_len=1777, n_kv_heads=3, n_q_heads=6, head_dim=64, window=16)),
    ("cfg1", dict(seq_len=1000, n_kv_heads=2, n_q_heads=4, window=20)),
])
def test_report_matches_oracle(base, over):
    cfg = dg.scaled(dg.CONFIGS[base], **over)
    li = wl.make_layer(cfg, 0)
    H, n = cfg.n_kv_heads, cfg.seq_len
    n_r, n_a, n_p = cfg.counts()
    wide = {x: dg.widen(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    # weights: the un-pooled attention mass (sums to one per head); routing from the oracle
    w = vo.attention_mass(wide["q_win"], wide["k"]).astype(np.float32)
    score = vo.score(wide["q_win"], wide["k"], cfg.window, cfg.pool_kernel)
    eps = vo.residual(wide["k"], wide["v"], wide["w_cal"])
    tier, _, _ = vo.route(score, eps, n_p, n_a)
    ref = vo.distortion_report(w, tier, eps, wide["v"])
    shape = pl.shape_of(cfg)
    out = torch.zeros((H, len(vb.DISTORTION_FIELDS)), dtype=torch.float64, device="cuda:0")
    ws = pl.alloc_workspace(vb.vector_distortion_workspace_bytes(shape))
    vb.vector_distortion(shape, pl.to_device(w), pl.to_device(tier.astype(np.uint8)), pl.to_device(eps), pl.to_device(li.v), out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for i, name in enumerate(vb.DISTORTION_FIELDS):
        np.testing.assert_allclose(got[:, i], np.asarray(ref[name], np.float64), rtol=2e-5, atol=1e-9, err_msg=name)
    assert (got[:, 8] == n_a).all() and (got[:, 9] == n - n_p).all()
    # run to run the sums come out bit-identical
    out2 = torch.zeros_like(out)
    vb.vector_distortion(shape, pl.to_device(w), pl.to_device(tier.astype(np.uint8)), pl.to_device(eps), pl.to_device(li.v), out2, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("base,over,p_c", [
    ("cfg2", dict(seq_len=4096, n_kv_heads=2, n_q_heads=8), 0.85),
    ("cfg1", dict(seq_len=3000, n_kv_heads=2, n_q_heads=4, window=20), 0.75),
])
def test_three_way_routing_beats_binary_eviction_at_equal_footprint(base, over, p_c):
    """Section 4 (distortion measure, Proposition 1) and the approximation-ratio sweep of Section 5,
    through the library end to end: on planted data whose values are well predicted from the keys
    (noise far below the values' norm for the tokens that get approximated), moving budget from
    retained values to pool keys at a fixed footprint of 2 (1 - p_c) n rows lowers the
    importance-weighted loss.  p_a = 0 is binary eviction with the same memory."""
    cfg = dg.scaled(dg.CONFIGS[base], **over)
    li = wl.make_layer(cfg, 0)
    H, n = cfg.n_kv_heads, cfg.seq_len
    shape = pl.shape_of(cfg)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    wide = {x: dg.widen(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    weights = vo.attention_mass(wide["q_win"], wide["k"]).astype(np.float32)       # sums to one per head
    w_dev = pl.to_device(weights)
    o_score = vo.score(wide["q_win"], wide["k"], cfg.window, cfg.pool_kernel)
    o_eps = vo.residual(wide["k"], wide["v"], wide["w_cal"])
    dout = torch.zeros((H, len(vb.DISTORTION_FIELDS)), dtype=torch.float64, device="cuda:0")
    wsd = pl.alloc_workspace(vb.vector_distortion_workspace_bytes(shape))
    loss, loss_oracle, rows = {}, {}, {}
    for p_a in (0.0, 0.025, 0.05, 0.1):
        n_p, n_a = vb.vector_budget_counts(n, p_c, p_a)
        assert (n_p, n_a) == vo.budget_counts(n, p_c, p_a)
        n_r = n_p - n_a
        rows[p_a] = n_p + n_r                                  # key rows + value rows kept
        out = pl.alloc_outputs(shape, n_p, n_a, n_r, tdt)
        ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a))
        pl.compress_layer(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], n_p, n_a, out, ws, one_call=True)
        vb.vector_distortion(shape, w_dev, out.tier, out.eps, dev["v"], dout, wsd)
        torch.cuda.synchronize()
        loss[p_a] = dout.cpu().numpy()[:, 0].copy()
        o_tier, _, _ = vo.route(o_score, o_eps, n_p, n_a)
        loss_oracle[p_a] = vo.distortion_report(weights, o_tier, o_eps, wide["v"])["E"]
        # the library's loss is the oracle's: routing may differ only for tokens at a threshold
        np.testing.assert_allclose(loss[p_a], loss_oracle[p_a], rtol=1e-2, err_msg=f"p_a = {p_a}")
    for p_a in (0.025, 0.05, 0.1):
        assert abs(rows[p_a] - rows[0.0]) <= 2, "the sweep must hold the footprint fixed (up to count rounding)"
        assert (loss[p_a] < loss[0.0]).all(), f"p_a = {p_a}: {loss[p_a]} against binary eviction {loss[0.0]}"
        assert (loss_oracle[p_a] < loss_oracle[0.0]).all()
