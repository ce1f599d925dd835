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
