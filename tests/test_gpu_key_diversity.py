"""GPU parity of the query-agnostic key-diversity score, and its use as the importance score of the routing."""
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
    ("cfg2", dict(seq_len=8192, n_kv_heads=2, n_q_heads=8)),
    ("cfg2", dict(seq_len=5001, n_kv_heads=3, n_q_heads=3, head_dim=64)),
    ("cfg1", dict(seq_len=777, n_kv_heads=2, n_q_heads=2)),
    ("cfg1", dict(seq_len=3000, n_kv_heads=1, n_q_heads=1, head_dim=128)),
])
def test_score_and_routing_on_it(base, over):
    cfg = dg.scaled(dg.CONFIGS[base], **over)
    li = wl.make_layer(cfg, 0)
    # shift the keys so that they share a direction (as real keys do): cosines spread over (-1, 1)
    k = dg.widen(li.k) + 0.7
    k_store = dg.f32_to_bf16_bits(k.astype(np.float32)) if cfg.dtype == "bf16" else k.astype(np.float32)
    H, n = cfg.n_kv_heads, cfg.seq_len
    shape = pl.shape_of(cfg)
    n_r, n_a, n_p = cfg.counts()
    score = torch.full((H, n), 9.0, device="cuda:0")
    ws = pl.alloc_workspace(max(vb.vector_score_key_diversity_workspace_bytes(shape), vb.vector_workspace_bytes(shape, n_p, n_a, 1)))
    k_dev = pl.to_device(k_store)
    vb.vector_score_key_diversity(shape, k_dev, score, ws)
    torch.cuda.synchronize()
    ref = vo.score_key_diversity(dg.widen(k_store))
    got = score.cpu().numpy()
    err = np.abs(got.astype(np.float64) - ref)
    assert (err <= 1e-3 + 2e-3 * np.abs(ref)).all(), f"max err {err.max():.3e}"      # element by element
    # the routing takes this score like any other: bit-exact against the oracle on the same floats
    eps = vo.residual(dg.widen(k_store), dg.widen(li.v), dg.widen(li.w_cal))
    tier = torch.empty((H, n), dtype=torch.uint8, device="cuda:0")
    idx_r = torch.empty((H, max(n_r, 1)), dtype=torch.int32, device="cuda:0")
    idx_a = torch.empty((H, max(n_a, 1)), dtype=torch.int32, device="cuda:0")
    vb.vector_route(H, n, score, pl.to_device(eps), n_p, n_a, tier, idx_r, idx_a, ws)
    torch.cuda.synchronize()
    r_tier, r_ir, r_ia = vo.route(got, eps, n_p, n_a)
    assert np.array_equal(tier.cpu().numpy(), r_tier)
    assert np.array_equal(idx_r.cpu().numpy()[:, :n_r], r_ir) and np.array_equal(idx_a.cpu().numpy()[:, :n_a], r_ia)


def test_zero_keys_and_repeatability():
    H, n, d = 2, 4100, 128
    rng = np.random.default_rng(4)
    k = rng.standard_normal((H, n, d)).astype(np.float32) + 0.5
    k[0, 17] = 0.0                                       # no direction: scores 0, adds nothing to the anchor
    k_bits = dg.f32_to_bf16_bits(k)
    shape = vb.Shape(n_q_heads=H, n_kv_heads=H, head_dim=d, seq_len=n, window=1, pool_kernel=1, dtype=vb.VECTOR_BF16)
    ws = pl.alloc_workspace(vb.vector_score_key_diversity_workspace_bytes(shape))
    k_dev = pl.to_device(k_bits)
    a = torch.empty((H, n), device="cuda:0")
    b = torch.empty((H, n), device="cuda:0")
    vb.vector_score_key_diversity(shape, k_dev, a, ws)
    vb.vector_score_key_diversity(shape, k_dev, b, ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    assert a[0, 17].item() == 0.0
    # the oracle divides by the key norm, so the reference is written out here with the zero key left out
    got = a.cpu().numpy()
    unit = dg.widen(k_bits).astype(np.float64)
    nz = np.linalg.norm(unit, axis=-1, keepdims=True)
    unit = np.divide(unit, nz, out=np.zeros_like(unit), where=nz > 0)
    anchor = unit.sum(axis=1)
    anchor /= np.linalg.norm(anchor, axis=-1, keepdims=True)
    want = -(unit * anchor[:, None, :]).sum(-1)
    assert np.abs(got - want).max() < 2e-3
