"""The smallest sequences: one to a few tokens, the window covering one token or all of them.
Scores and residuals against the oracle, the routing of the GPU's own floats exact, the packed
rows byte for byte; both dtypes, both head dims, the one-call pass and the three calls."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
from paper_2605_23258_amd import pipeline as pl

pytestmark = pytest.mark.gpu

CASES = [
    # dtype, d, Hkv, G, n, w, pool kernel, n_pool, n_approx
    ("bf16", 128, 1, 4, 1, 1, 1, 1, 0),
    ("bf16", 128, 2, 2, 1, 1, 7, 1, 1),
    ("f32", 64, 1, 1, 1, 1, 3, 0, 0),
    ("f32", 64, 2, 2, 2, 1, 3, 2, 1),
    ("bf16", 64, 1, 4, 2, 2, 1, 1, 1),
    ("bf16", 128, 2, 4, 3, 1, 5, 2, 1),
    ("f32", 128, 1, 2, 5, 2, 7, 4, 2),
    ("bf16", 128, 1, 8, 5, 5, 3, 5, 5),
    ("bf16", 64, 3, 1, 17, 4, 9, 9, 3),
    ("f32", 64, 1, 4, 33, 32, 7, 20, 20),
]


@pytest.mark.parametrize("dtype,d,H,G,n,w,kern,n_p,n_a", CASES)
@pytest.mark.parametrize("one_call", [True, False], ids=["one_call", "three_calls"])
def test_tiny_sequence(dtype, d, H, G, n, w, kern, n_p, n_a, one_call):
    rng = np.random.default_rng(1000 * n + 10 * d + H + G + kern)
    store = (lambda x: dg.f32_to_bf16_bits(x.astype(np.float32))) if dtype == "bf16" else (lambda x: x.astype(np.float32))
    q = store(rng.standard_normal((H * G, w, d)))
    k = store(rng.standard_normal((H, n, d)))
    v = store(rng.standard_normal((H, n, d)))
    W = store(rng.standard_normal((H, d, d)) / np.sqrt(d))
    n_r = n_p - n_a
    shape = vb.Shape(n_q_heads=H * G, n_kv_heads=H, head_dim=d, seq_len=n, window=w, pool_kernel=kern,
                     dtype=vb.VECTOR_BF16 if dtype == "bf16" else vb.VECTOR_F32)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    out = pl.alloc_outputs(shape, n_p, n_a, n_r + 1, tdt)
    out.tier.fill_(9)
    ws = pl.alloc_workspace(max(vb.vector_compress_workspace_bytes(shape, n_p, n_a), vb.vector_workspace_bytes(shape, n_p, n_a, 1)))
    pl.compress_layer(shape, pl.to_device(q), pl.to_device(k), pl.to_device(v), pl.to_device(W), n_p, n_a, out, ws, one_call=one_call)
    torch.cuda.synchronize()
    g_score, g_eps = out.score.cpu().numpy(), out.eps.cpu().numpy()
    ref_score = vo.score(dg.widen(q), dg.widen(k), w, kern)
    ref_eps = vo.residual(dg.widen(k), dg.widen(v), dg.widen(W))
    assert np.isposinf(g_score[:, n - w:]).all()
    err = np.abs(g_score[:, : n - w].astype(np.float64) - ref_score[:, : n - w]) * n
    assert (err <= 1e-3 + 2e-3 * np.abs(ref_score[:, : n - w]) * n).all()
    err = np.abs(g_eps.astype(np.float64) - ref_eps)
    assert (err <= 1e-3 + 2e-3 * np.abs(ref_eps)).all(), f"eps: max err {err.max():.3e}"
    tier, idx_r, idx_a = vo.route(g_score, g_eps, n_p, n_a)
    assert np.array_equal(out.tier.cpu().numpy(), tier)
    if n_r:
        assert np.array_equal(out.idx_retain.cpu().numpy()[:, :n_r], idx_r)
    if n_a:
        assert np.array_equal(out.idx_approx.cpu().numpy()[:, :n_a], idx_a)
    rk, rv, ra = vo.compact(k, v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(out.k_ret)[:, :n_r], rk) and np.array_equal(pl.to_host(out.v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(out.k_apx)[:, :n_a], ra)
    assert not pl.to_host(out.k_ret)[:, n_r:].any(), "the spare row stays untouched"
