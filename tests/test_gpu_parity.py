"""GPU parity: every entry point of the C ABI against the CPU oracle on the same
seeded inputs.  Integer and byte outputs must be bit-exact; floats within
|g - o| <= 1e-3 + 2e-3 |o| (scores are compared after scaling by n, since a
score is O(1/n) and the absolute term would otherwise be vacuous)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
import workloads as wl
from paper_2605_23258_amd import pipeline as pl
from parity_util import band_check as _band_check, decode_check

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-3, 2e-3


def close(got, ref, what):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


def score_close(got, ref, n, window):
    got, ref = np.asarray(got), np.asarray(ref)
    assert np.isposinf(got[:, n - window:]).all(), "window columns must be +inf"
    assert np.isfinite(got[:, : n - window]).all()
    close(got[:, : n - window].astype(np.float64) * n, ref[:, : n - window].astype(np.float64) * n, "n*score")


CASES = {
    # name: (base config, overrides) -- several tiles, ragged tails, both dtypes and head dims
    "f32_d64_n1024": ("cfg1", {}),
    "f32_d64_ragged": ("cfg1", dict(seq_len=1000, window=20, n_q_heads=6, n_kv_heads=2)),
    "bf16_d128_n2048": ("cfg2", dict(seq_len=2048, n_kv_heads=2, n_q_heads=8)),
    "bf16_d128_ragged": ("cfg2", dict(seq_len=1777, n_kv_heads=2, n_q_heads=8, window=24, pool_kernel=5)),
    "bf16_d128_w64": ("cfg3", dict(seq_len=1536, n_kv_heads=1, n_q_heads=4, layers=1)),
    "bf16_d64": ("cfg2", dict(seq_len=900, head_dim=64, n_kv_heads=2, n_q_heads=4, window=16)),
    # 256 query rows per KV head (two row blocks per wave in the first pass): an odd length whose last
    # chunk and last 128-token step are partial, rows padded from 240 to 256, d = 64, and eight and two
    # KV heads (the grid of both passes is dealt out over the XCDs by head)
    "bf16_d128_w64_ragged": ("cfg3", dict(seq_len=1733, n_kv_heads=2, n_q_heads=8, layers=1)),
    "bf16_d128_w60_padded_rows": ("cfg3", dict(seq_len=1100, n_kv_heads=1, n_q_heads=4, window=60, layers=1)),
    "bf16_d64_w64": ("cfg3", dict(seq_len=1400, head_dim=64, n_kv_heads=1, n_q_heads=4, layers=1)),
    "bf16_d128_w64_eight_heads": ("cfg3", dict(seq_len=700, n_kv_heads=8, n_q_heads=32, layers=1)),
    # four KV heads (two XCDs per head, the chunks of a head split between them) and sixteen (two heads per XCD)
    "bf16_d128_four_heads": ("cfg2", dict(seq_len=2040, n_kv_heads=4, n_q_heads=16)),    # 8 and 4 chunks: even, as the split needs
    "bf16_d128_sixteen_heads": ("cfg2", dict(seq_len=1300, n_kv_heads=16, n_q_heads=32, window=48)),
    "f32_d128": ("cfg1", dict(seq_len=700, head_dim=128, n_kv_heads=1, n_q_heads=2, window=8, pool_kernel=3)),
    "tiny_n_equals_w": ("cfg1", dict(seq_len=32, window=32)),
    "short": ("cfg2", dict(seq_len=70, n_kv_heads=1, n_q_heads=4, window=5, pool_kernel=1)),
    # maximum pooling: the vector path (kernel <= 9), the general loop (kernel 13), an unaligned length
    "bf16_maxpool7": ("cfg2", dict(seq_len=2048, n_kv_heads=2, n_q_heads=8, pool_mode="max")),
    "bf16_maxpool5_ragged": ("cfg2", dict(seq_len=1777, n_kv_heads=2, n_q_heads=8, window=24, pool_kernel=5, pool_mode="max")),
    # more query rows per KV head than the kernels hold at once: the query heads go in groups
    # (two groups of 4 heads; 4 + 2 heads; 3 + 1 heads of fp32 rows; 6 + 1 heads at d = 64)
    "bf16_G8_w64_groups": ("cfg3", dict(seq_len=1536, n_kv_heads=2, n_q_heads=16, layers=1)),
    "bf16_G6_w64_groups": ("cfg3", dict(seq_len=1300, n_kv_heads=1, n_q_heads=6, layers=1)),
    "f32_d128_G4_w48_groups": ("cfg1", dict(seq_len=700, head_dim=128, n_kv_heads=1, n_q_heads=4, window=48, pool_kernel=3)),
    "bf16_d64_G7_w60_groups": ("cfg2", dict(seq_len=900, head_dim=64, n_kv_heads=2, n_q_heads=14, window=60, pool_mode="max")),
    "f32_maxpool13": ("cfg1", dict(seq_len=1000, window=20, n_q_heads=6, n_kv_heads=2, pool_kernel=13, pool_mode="max")),
}


def _inputs(name):
    base, over = CASES[name]
    cfg = dg.scaled(dg.CONFIGS[base], **over)
    li = wl.make_layer(cfg, 0)
    dev = {k: pl.to_device(getattr(li, k)) for k in ("q_win", "k", "v", "w_cal")}
    wide = {k: dg.widen(getattr(li, k)) for k in ("q_win", "k", "v", "w_cal")}
    return cfg, li, dev, wide


@pytest.mark.parametrize("name", list(CASES))
def test_score_and_residual(name):
    cfg, li, dev, wide = _inputs(name)
    shape = pl.shape_of(cfg)
    n_r, n_a, n_p = cfg.counts()
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    H, n = cfg.n_kv_heads, cfg.seq_len
    score = torch.full((H, n), -1.0, device="cuda:0")
    eps = torch.full((H, n), -1.0, device="cuda:0")
    vb.vector_score(shape, dev["q_win"], dev["k"], score, ws)
    vb.vector_residual(shape, dev["k"], dev["v"], dev["w_cal"], eps, ws)
    torch.cuda.synchronize()
    ref_score = vo.score(wide["q_win"], wide["k"], cfg.window, cfg.pool_kernel, cfg.pool_mode)
    ref_eps = vo.residual(wide["k"], wide["v"], wide["w_cal"])
    score_close(score.cpu().numpy(), ref_score, n, cfg.window)
    close(eps.cpu().numpy(), ref_eps, "eps")
    # the fused entry point gives the same two outputs
    score2 = torch.full((H, n), -1.0, device="cuda:0")
    eps2 = torch.full((H, n), -1.0, device="cuda:0")
    vb.vector_score_residual(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], score2, eps2, ws)
    torch.cuda.synchronize()
    score_close(score2.cpu().numpy(), ref_score, n, cfg.window)
    close(eps2.cpu().numpy(), ref_eps, "eps (fused)")


@pytest.mark.parametrize("name", ["bf16_d128_ragged", "bf16_d64"])
def test_residual_probe_matches_oracle(name):
    """The contraction probe repeats each tile's arithmetic on resident operands; its eps output
    is still the residual, whatever the repeat count."""
    cfg, li, dev, wide = _inputs(name)
    shape = pl.shape_of(cfg)
    ref_eps = vo.residual(wide["k"], wide["v"], wide["w_cal"])
    for repeat in (1, 3):
        eps = torch.full((cfg.n_kv_heads, cfg.seq_len), -1.0, device="cuda:0")
        vb.vector_probe_residual_mfma(shape, dev["k"], dev["v"], dev["w_cal"], eps, repeat)
        torch.cuda.synchronize()
        close(eps.cpu().numpy(), ref_eps, f"eps (probe, repeat {repeat})")


def _route_gpu(score, eps, n_pool, n_approx):
    H, n = score.shape
    shape = vb.Shape(n_q_heads=H, n_kv_heads=H, head_dim=64, seq_len=n, window=1, pool_kernel=1, dtype=0)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_pool, n_approx, 1))
    tier = torch.full((H, n), 77, dtype=torch.uint8, device="cuda:0")
    idx_r = torch.full((H, max(n_pool - n_approx, 1)), -1, dtype=torch.int32, device="cuda:0")
    idx_a = torch.full((H, max(n_approx, 1)), -1, dtype=torch.int32, device="cuda:0")
    vb.vector_route(H, n, pl.to_device(score), pl.to_device(eps), n_pool, n_approx, tier,
                    idx_r if n_pool - n_approx else None, idx_a if n_approx else None, ws)
    torch.cuda.synchronize()
    return tier.cpu().numpy(), idx_r.cpu().numpy()[:, : n_pool - n_approx], idx_a.cpu().numpy()[:, :n_approx]


def _assert_route_equal(score, eps, n_pool, n_approx):
    got = _route_gpu(score, eps, n_pool, n_approx)
    ref = vo.route(score, eps, n_pool, n_approx)
    for g, r, what in zip(got, ref, ("tier", "idx_retain", "idx_approx")):
        assert np.array_equal(g, r), f"{what} differs (n={score.shape[1]}, n_pool={n_pool}, n_approx={n_approx})"


@pytest.mark.parametrize("n,n_pool,n_approx", [
    (1, 1, 1), (1, 0, 0), (5, 5, 0), (64, 10, 10), (1000, 300, 150), (4096, 1228, 614), (4097, 4097, 2000),
    (5000, 0, 0), (12345, 2469, 1234), (40000, 8000, 4000),
    # beyond 32768 tokens per head the selection by score runs chip-wide in chunks of 8192
    (32769, 100, 50), (65536, 65536, 30000), (70000, 40000, 20000), (100000, 1, 1), (49152, 0, 0), (90001, 9000, 0)])
def test_route_bit_exact_random(n, n_pool, n_approx):
    rng = np.random.default_rng(n * 7 + n_pool)
    score = rng.random((3, n)).astype(np.float32)
    score[:, max(0, n - 16):] = np.inf
    eps = (rng.random((3, n)) ** 4).astype(np.float32)
    _assert_route_equal(score, eps, n_pool, n_approx)


def test_route_bit_exact_heavy_ties_and_signed_zero():
    rng = np.random.default_rng(5)
    n = 6000
    score = rng.integers(0, 5, size=(4, n)).astype(np.float32) * 0.25
    eps = rng.integers(0, 3, size=(4, n)).astype(np.float32)
    score[0, ::7] = -0.0
    eps[1, ::5] = -0.0
    score[2] = 1.0                      # all equal: lowest indices win
    eps[3] = 0.0
    for n_pool, n_approx in ((1500, 700), (n, n // 2), (1, 1), (2999, 0)):
        _assert_route_equal(score, eps, n_pool, n_approx)


def test_route_long_sequence_with_heavy_ties():
    """Ties across chunk boundaries of the chip-wide path: the lowest token indices win."""
    rng = np.random.default_rng(9)
    n = 50000
    score = rng.integers(0, 4, size=(3, n)).astype(np.float32) * 0.5
    eps = rng.integers(0, 3, size=(3, n)).astype(np.float32)
    score[1] = 2.0                      # all equal
    score[2, ::3] = -0.0
    for n_pool, n_approx in ((20000, 9000), (n, 100), (8193, 8193), (1, 0)):
        _assert_route_equal(score, eps, n_pool, n_approx)


def test_route_many_candidates_one_ulp_apart():
    """More keys share the threshold's bucket than the kernel keeps in LDS, and they are not all
    equal (two neighbouring floats, for the scores and for the residuals): the select has to go
    back to memory for every level.  With one value only, the plateau shortcut takes over."""
    rng = np.random.default_rng(21)
    n = 60000
    one, nxt = np.float32(1.0), np.nextafter(np.float32(1.0), np.float32(2.0))
    score = np.where(rng.random((3, n)) < 0.5, one, nxt).astype(np.float32)
    eps = np.where(rng.random((3, n)) < 0.3, one, nxt).astype(np.float32)
    score[2] = one                                        # a plateau
    score[:, ::9973] = 50.0                               # a few tokens far above
    for n_pool, n_approx in ((20000, 9000), (45000, 44000), (7, 3)):
        _assert_route_equal(score, eps, n_pool, n_approx)


def test_route_is_deterministic():
    rng = np.random.default_rng(6)
    score = rng.integers(0, 50, size=(8, 20000)).astype(np.float32)
    eps = rng.integers(0, 50, size=(8, 20000)).astype(np.float32)
    first = _route_gpu(score, eps, 5000, 2500)
    for _ in range(5):
        again = _route_gpu(score, eps, 5000, 2500)
        assert all(np.array_equal(a, b) for a, b in zip(first, again))


@pytest.mark.parametrize("name", ["f32_d64_ragged", "bf16_d128_ragged", "bf16_d64", "f32_d128"])
def test_compact_bit_exact(name):
    cfg, li, dev, wide = _inputs(name)
    shape = pl.shape_of(cfg)
    n_r, n_a, n_p = cfg.counts()
    rng = np.random.default_rng(3)
    H, n, d = cfg.n_kv_heads, cfg.seq_len, cfg.head_dim
    tier, idx_r, idx_a = vo.route(rng.random((H, n)).astype(np.float32), rng.random((H, n)).astype(np.float32), n_p, n_a)
    cap = n_r + 9
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    k_ret = torch.zeros((H, cap, d), dtype=tdt, device="cuda:0")
    v_ret = torch.zeros((H, cap, d), dtype=tdt, device="cuda:0")
    k_apx = torch.zeros((H, n_a, d), dtype=tdt, device="cuda:0")
    vb.vector_compact(shape, dev["k"], dev["v"], pl.to_device(idx_r), pl.to_device(idx_a), n_r, n_a,
                      k_ret, v_ret, k_apx, cap)
    torch.cuda.synchronize()
    rk, rv, ra = vo.compact(li.k, li.v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(k_ret)[:, :n_r], rk)
    assert np.array_equal(pl.to_host(v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(k_apx), ra)
    assert not pl.to_host(k_ret)[:, n_r:].any(), "rows beyond n_retain must stay untouched"


DECODE_CASES = [
    # dtype, d, B, Hq, Hkv, n_r, n_a, cap
    ("bf16", 128, 3, 8, 2, 300, 200, 320),
    ("bf16", 128, 2, 4, 4, 33, 0, 40),
    ("bf16", 128, 2, 8, 1, 0, 65, 4),
    ("f32", 64, 2, 4, 1, 100, 77, 128),
    ("bf16", 64, 1, 4, 2, 1, 1, 1),
    ("f32", 128, 1, 2, 2, 50, 31, 50),
    ("bf16", 128, 1, 32, 8, 1500, 1400, 1600),
    # sixteen, twelve and ten query heads per KV head
    ("bf16", 128, 2, 32, 2, 700, 300, 710),
    ("bf16", 64, 1, 24, 2, 90, 333, 100),
    ("f32", 64, 2, 10, 1, 120, 77, 128),
    ("f32", 128, 1, 16, 1, 65, 40, 70),
]


@pytest.mark.parametrize("dtype,d,B,Hq,Hkv,n_r,n_a,cap", DECODE_CASES)
def test_decode_attn(dtype, d, B, Hq, Hkv, n_r, n_a, cap):
    rng = np.random.default_rng(d + B + n_r)
    def store(x):
        x = x.astype(np.float32)
        return dg.f32_to_bf16_bits(x) if dtype == "bf16" else x
    q = store(rng.standard_normal((B, Hq, d)))
    k_ret = store(rng.standard_normal((B, Hkv, cap, d)))
    v_ret = store(rng.standard_normal((B, Hkv, cap, d)))
    k_apx = store(rng.standard_normal((B, Hkv, max(n_a, 1), d)))[:, :, :n_a]
    W = store(rng.standard_normal((Hkv, d, d)) / np.sqrt(d))
    length = np.full(B, n_r, dtype=np.int32)
    if B > 1:
        length[1] = max(0, n_r - 7)            # ragged batch
    # poison rows beyond the live length: they must never be read into the result
    for b in range(B):
        k_ret[b, :, length[b]:] = store(np.full((1,), 1e30))[0]
        v_ret[b, :, length[b]:] = store(np.full((1,), -1e30))[0]
    scale = 1.0 / np.sqrt(d)
    ref = vo.decode_attn(dg.widen(q), dg.widen(k_ret), dg.widen(v_ret), length, dg.widen(k_apx), dg.widen(W), scale)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                     dtype=vb.VECTOR_BF16 if dtype == "bf16" else vb.VECTOR_F32, cap_retain=cap, n_approx=n_a)
    t = dict(len=pl.to_device(length), k_ret=pl.to_device(k_ret), v_ret=pl.to_device(v_ret),
             k_apx=pl.to_device(np.ascontiguousarray(k_apx)) if n_a else None, W=pl.to_device(W), q=pl.to_device(q))
    cache.len_retain, cache.k_ret, cache.v_ret = t["len"].data_ptr(), t["k_ret"].data_ptr(), t["v_ret"].data_ptr()
    cache.k_apx = t["k_apx"].data_ptr() if n_a else None
    cache.W = t["W"].data_ptr()
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, seq_len=max(cap, 1), window=1, pool_kernel=1, dtype=cache.dtype)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, max(cap, 1), 0, B) + (1 << 20))
    out = torch.full((B, Hq, d), 7.0, dtype=tdt, device="cuda:0")
    got = decode_check(cache, t["q"], scale, ws, ref, "decode out")
    if B > 1 and length[1] == 0 and n_a == 0:
        assert not got[1].any()
    if dtype == "bf16":
        # the literal variant (every approximated value rebuilt as k W before it is weighted) is
        # the same sum in another order
        decode_check(cache, t["q"], scale, ws, ref, "decode out (literal)", flags=vb.VECTOR_DECODE_LITERAL)
    else:
        with pytest.raises(vb.VectorError) as ei:
            vb.vector_decode_attn(cache, t["q"], scale, out, ws, flags=vb.VECTOR_DECODE_LITERAL)
        assert ei.value.code == vb.VECTOR_ERR_DTYPE


@pytest.mark.parametrize("name", ["f32_d64_n1024", "bf16_d128_n2048", "bf16_d128_ragged", "bf16_G8_w64_groups", "bf16_d128_w64_ragged",
                                  "bf16_d128_w64_eight_heads", "bf16_d128_four_heads", "bf16_d128_sixteen_heads"])
def test_end_to_end_compress(name):
    cfg, li, dev, wide = _inputs(name)
    shape = pl.shape_of(cfg)
    n_r, n_a, n_p = cfg.counts()
    n = cfg.seq_len
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    out = pl.alloc_outputs(shape, n_p, n_a, n_r + 4, tdt)
    pl.compress_layer(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], n_p, n_a, out, ws)
    torch.cuda.synchronize()
    g_score, g_eps = out.score.cpu().numpy(), out.eps.cpu().numpy()
    # the GPU's routing of its own floats equals the oracle's routing of those same floats
    tier, idx_r, idx_a = vo.route(g_score, g_eps, n_p, n_a)
    assert np.array_equal(out.tier.cpu().numpy(), tier)
    assert np.array_equal(out.idx_retain.cpu().numpy(), idx_r)
    assert np.array_equal(out.idx_approx.cpu().numpy(), idx_a)
    rk, rv, ra = vo.compact(li.k, li.v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(out.k_ret)[:, :n_r], rk)
    assert np.array_equal(pl.to_host(out.v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(out.k_apx)[:, :n_a], ra)
    # against the oracle end to end: differences only inside the tolerance band of the thresholds
    o_score = vo.score(wide["q_win"], wide["k"], cfg.window, cfg.pool_kernel)
    o_eps = vo.residual(wide["k"], wide["v"], wide["w_cal"])
    o_tier, _, _ = vo.route(o_score, o_eps, n_p, n_a)
    flips = _band_check(o_score, o_eps, n_p, n_a, tier, o_tier, n, name)
    assert flips <= 0.002 * tier.size
