"""The longest sequence the routing accepts (2^20 tokens): 32 chunks of 32768 tokens, whose digit
tables count up to the limit of their 16-bit entries, and bucket lists too long to be put
together in LDS.  Routing alone against the oracle's two sorts, then the whole one-call pass."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
from paper_2605_23258_amd import pipeline as pl

pytestmark = pytest.mark.gpu

N_MAX = 1 << 20


def _route(score, eps, n_pool, n_approx):
    H, n = score.shape
    shape = vb.Shape(n_q_heads=H, n_kv_heads=H, head_dim=64, seq_len=n, window=1, pool_kernel=1, dtype=0)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_pool, n_approx, 1))
    tier = torch.full((H, n), 77, dtype=torch.uint8, device="cuda:0")
    idx_r = torch.full((H, n_pool - n_approx), -1, dtype=torch.int32, device="cuda:0")
    idx_a = torch.full((H, n_approx), -1, dtype=torch.int32, device="cuda:0")
    vb.vector_route(H, n, pl.to_device(score), pl.to_device(eps), n_pool, n_approx, tier, idx_r, idx_a, ws)
    torch.cuda.synchronize()
    return tier.cpu().numpy(), idx_r.cpu().numpy(), idx_a.cpu().numpy()


@pytest.mark.parametrize("kind", ["lognormal", "few_distinct_values", "one_chunk_holds_the_pool"])
def test_route_at_the_longest_sequence(kind):
    rng = np.random.default_rng({"lognormal": 1, "few_distinct_values": 2, "one_chunk_holds_the_pool": 3}[kind])
    H, n = 2, N_MAX
    if kind == "lognormal":
        score = np.exp(rng.standard_normal((H, n))).astype(np.float32) / n
        eps = np.exp(0.3 * rng.standard_normal((H, n))).astype(np.float32)
    elif kind == "few_distinct_values":                      # heavy ties in both selections
        score = rng.integers(0, 9, size=(H, n)).astype(np.float32) * 0.125
        eps = rng.integers(0, 5, size=(H, n)).astype(np.float32)
    else:                                                    # every pool member in one 32768-token chunk: its table entries reach 32768
        score = rng.random((H, n)).astype(np.float32) * 0.5
        score[:, 5 * 32768: 6 * 32768] += 1.0
        eps = rng.random((H, n)).astype(np.float32)
    n_pool, n_approx = (32768, 12000) if kind == "one_chunk_holds_the_pool" else (100000, 40000)
    got = _route(score, eps, n_pool, n_approx)
    ref = vo.route(score, eps, n_pool, n_approx)
    for g, r, what in zip(got, ref, ("tier", "idx_retain", "idx_approx")):
        assert np.array_equal(g, r), f"{kind}: {what}"


def test_one_token_more_is_refused():
    H, n = 1, N_MAX + 1
    z = torch.zeros((H, n), device="cuda:0")
    tier = torch.full((H, n), 9, dtype=torch.uint8, device="cuda:0")
    idx = torch.zeros((H, 8), dtype=torch.int32, device="cuda:0")
    ws = pl.alloc_workspace(1 << 26)
    with pytest.raises(vb.VectorError) as ei:
        vb.vector_route(H, n, z, z, 8, 4, tier, idx, idx, ws)
    assert ei.value.code == vb.VECTOR_ERR_SHAPE
    torch.cuda.synchronize()
    assert (tier == 9).all()


def test_compress_at_the_longest_sequence():
    """bf16, d = 64, one KV head with two query heads, window 16: scores and residuals within
    tolerance, the routing of the GPU's own floats exact, the packed rows byte for byte."""
    rng = np.random.default_rng(12)
    n, d, w, G = N_MAX, 64, 16, 2
    n_p, n_a = 60000, 25000
    n_r = n_p - n_a
    q = dg.f32_to_bf16_bits((rng.standard_normal((G, w, d)) * 1.5).astype(np.float32))
    k = dg.f32_to_bf16_bits(rng.standard_normal((1, n, d)).astype(np.float32))
    W = (rng.standard_normal((1, d, d)) / np.sqrt(d)).astype(np.float32)
    noise = np.exp(rng.uniform(np.log(1e-3), 0.0, size=(1, n, 1))).astype(np.float32)
    v = dg.f32_to_bf16_bits((dg.bf16_bits_to_f32(k) @ W + noise * rng.standard_normal((1, n, d)).astype(np.float32)).astype(np.float32))
    Wb = dg.f32_to_bf16_bits(W)
    shape = vb.Shape(n_q_heads=G, n_kv_heads=1, head_dim=d, seq_len=n, window=w, pool_kernel=7, dtype=vb.VECTOR_BF16)
    out = pl.alloc_outputs(shape, n_p, n_a, n_r, torch.bfloat16)
    ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a))
    pl.compress_layer(shape, pl.to_device(q), pl.to_device(k), pl.to_device(v), pl.to_device(Wb), n_p, n_a, out, ws, one_call=True)
    torch.cuda.synchronize()
    g_score, g_eps = out.score.cpu().numpy(), out.eps.cpu().numpy()
    ref_score = vo.score(dg.widen(q), dg.widen(k), w, 7)
    ref_eps = vo.residual(dg.widen(k), dg.widen(v), dg.widen(Wb))
    assert np.isposinf(g_score[:, n - w:]).all()
    err = np.abs(g_score[:, : n - w].astype(np.float64) - ref_score[:, : n - w]) * n
    assert (err <= 1e-3 + 2e-3 * np.abs(ref_score[:, : n - w]) * n).all(), f"n*score: max err {err.max():.3e}"
    err = np.abs(g_eps.astype(np.float64) - ref_eps)
    assert (err <= 1e-3 + 2e-3 * np.abs(ref_eps)).all(), f"eps: max err {err.max():.3e}"
    tier, idx_r, idx_a = vo.route(g_score, g_eps, n_p, n_a)
    assert np.array_equal(out.tier.cpu().numpy(), tier)
    assert np.array_equal(out.idx_retain.cpu().numpy(), idx_r) and np.array_equal(out.idx_approx.cpu().numpy(), idx_a)
    rk, rv, ra = vo.compact(k, v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(out.k_ret)[:, :n_r], rk) and np.array_equal(pl.to_host(out.v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(out.k_apx)[:, :n_a], ra)
