"""Routing inside vector_compress when the scores of a head lie close together (flat attention
rows: every score within a few per cent of 1/n, or all equal).  The one-call path then cuts its
radix buckets over the range of the head's attention mass instead of over the keys' top bits; the
selection must stay exactly the oracle's on the same floats wherever the thresholds fall: among
equal scores, among the +inf window columns, among scores below the assumed range (a pooling
kernel longer than the prefix), with the whole sequence in the pool."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
from paper_2605_23258_amd import pipeline as pl

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-3, 2e-3

CASES = {
    # name: dtype, d, Hkv, G, n, w, pool kernel, pool mode, scale of q, n_pool, n_approx
    "flat_bf16_3chunks": ("bf16", 128, 2, 4, 6000, 32, 7, "avg", 0.02, 1800, 900),
    "flat_f32_d64": ("f32", 64, 2, 2, 5000, 16, 5, "avg", 0.05, 1500, 700),
    "uniform_rows_all_equal": ("bf16", 128, 1, 4, 4500, 32, 1, "avg", 0.0, 1000, 500),
    "uniform_rows_pooled": ("f32", 64, 1, 2, 3000, 8, 7, "avg", 0.0, 900, 100),
    "flat_maxpool": ("bf16", 128, 2, 4, 5000, 24, 9, "max", 0.03, 2000, 1000),
    "flat_20_chunks": ("bf16", 128, 1, 2, 40000, 16, 7, "avg", 0.05, 8000, 4000),
    "flat_131k_32_chunks": ("bf16", 128, 1, 2, 131072, 16, 7, "avg", 0.05, 13106, 6553),
    "pool_inside_the_window": ("bf16", 128, 2, 4, 3000, 32, 7, "avg", 0.02, 20, 10),
    "pool_is_everything": ("bf16", 64, 1, 4, 2500, 16, 3, "avg", 0.02, 2500, 1250),
    "pool_leaves_one_out": ("f32", 64, 1, 4, 2100, 16, 3, "avg", 0.02, 2099, 3),
    "kernel_longer_than_prefix": ("f32", 64, 2, 2, 200, 190, 101, "avg", 0.1, 195, 60),
    "kernel_longer_than_prefix_flat": ("bf16", 128, 1, 4, 300, 60, 1001, "avg", 0.0, 200, 100),
    "moderate_spread": ("bf16", 128, 2, 4, 7000, 32, 7, "avg", 0.3, 2100, 1400),
    # a flat bulk plus a few tokens every query attends to (and a few it avoids): they fall outside the buckets' range
    "flat_bulk_with_sinks": ("bf16", 128, 2, 4, 9000, 32, 7, "avg", 0.02, 2700, 1300),
    "sinks_are_the_pool": ("f32", 64, 1, 4, 5000, 16, 3, "avg", 0.02, 12, 5),
}
SINKS = {"flat_bulk_with_sinks": 6, "sinks_are_the_pool": 9}


def _store(x, dtype):
    x = x.astype(np.float32)
    return dg.f32_to_bf16_bits(x) if dtype == "bf16" else x


@pytest.mark.parametrize("name", list(CASES))
def test_compress_routes_close_scores_exactly(name):
    dtype, d, H, G, n, w, kern, mode, q_scale, n_p, n_a = CASES[name]
    rng = np.random.default_rng(sorted(CASES).index(name) + 400)
    q = rng.standard_normal((H * G, w, d)) * q_scale
    k = rng.standard_normal((H, n, d))
    if name in SINKS:                                    # logits of about +8 and -8 against every query row
        u = np.zeros(d)
        u[0] = 1.0
        q = q + u
        at = rng.choice(n - w, size=2 * SINKS[name], replace=False)
        k[:, at[: SINKS[name]]] = u * 8.0 * np.sqrt(d)
        k[:, at[SINKS[name]:]] = -u * 8.0 * np.sqrt(d)
    q, k = _store(q, dtype), _store(k, dtype)
    v = _store(rng.standard_normal((H, n, d)), dtype)
    W = _store(rng.standard_normal((H, d, d)) / np.sqrt(d), dtype)
    n_r = n_p - n_a
    shape = vb.Shape(n_q_heads=H * G, n_kv_heads=H, head_dim=d, seq_len=n, window=w, pool_kernel=kern,
                     pool_mode=vb.VECTOR_POOL_MAX if mode == "max" else vb.VECTOR_POOL_AVG,
                     dtype=vb.VECTOR_BF16 if dtype == "bf16" else vb.VECTOR_F32)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    out = pl.alloc_outputs(shape, n_p, n_a, n_r, tdt)
    out.tier.fill_(9)
    ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a))
    pl.compress_layer(shape, pl.to_device(q), pl.to_device(k), pl.to_device(v), pl.to_device(W), n_p, n_a, out, ws, one_call=True)
    torch.cuda.synchronize()
    g_score, g_eps = out.score.cpu().numpy(), out.eps.cpu().numpy()
    # the scores themselves
    ref = vo.score(dg.widen(q), dg.widen(k), w, kern, mode)
    assert np.isposinf(g_score[:, n - w:]).all()
    err = np.abs(g_score[:, : n - w].astype(np.float64) - ref[:, : n - w]) * n
    assert (err <= ATOL + RTOL * np.abs(ref[:, : n - w]) * n).all(), f"n*score: max err {err.max():.3e}"
    # the routing of exactly these floats
    tier, idx_r, idx_a = vo.route(g_score, g_eps, n_p, n_a)
    assert np.array_equal(out.tier.cpu().numpy(), tier), "tier"
    assert np.array_equal(out.idx_retain.cpu().numpy()[:, :n_r], idx_r), "idx_retain"
    assert np.array_equal(out.idx_approx.cpu().numpy()[:, :n_a], idx_a), "idx_approx"
    rk, rv, ra = vo.compact(k, v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(out.k_ret)[:, :n_r], rk) and np.array_equal(pl.to_host(out.v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(out.k_apx)[:, :n_a], ra)
    # and the same selection as the three separate calls (which bucket by the keys' top bits)
    out3 = pl.alloc_outputs(shape, n_p, n_a, n_r, tdt)
    ws3 = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    pl.compress_layer(shape, pl.to_device(q), pl.to_device(k), pl.to_device(v), pl.to_device(W), n_p, n_a, out3, ws3)
    torch.cuda.synchronize()
    assert torch.equal(out3.score, out.score) and torch.equal(out3.tier, out.tier)
    assert torch.equal(out3.idx_retain, out.idx_retain) and torch.equal(out3.idx_approx, out.idx_approx)
