"""GPU tests of what the C header promises beyond the packed default layout: strided
K/V views, one W shared by all heads, and error returns that leave outputs untouched."""
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


def close(got, ref, what):
    err = np.abs(np.asarray(got, np.float64) - np.asarray(ref, np.float64))
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


def _layer(**over):
    cfg = dg.scaled(dg.CONFIGS["cfg2"], **over)
    return cfg, wl.make_layer(cfg, 0)


def test_token_major_interleaved_kv_layout():
    """K and V live in one [n, Hkv, 2, d] buffer (token-major, K and V of a head adjacent):
    every entry point that takes strides reads the same logical tensors as the packed layout."""
    cfg, li = _layer(seq_len=1500, n_kv_heads=2, n_q_heads=8, window=16)
    H, n, d = cfg.n_kv_heads, cfg.seq_len, cfg.head_dim
    n_r, n_a, n_p = cfg.counts()
    fused = np.zeros((n, H, 2, d), np.uint16)
    fused[:, :, 0] = np.transpose(li.k, (1, 0, 2))
    fused[:, :, 1] = np.transpose(li.v, (1, 0, 2))
    buf = pl.to_device(fused)
    k_view, v_view = buf[:, :, 0], buf[:, :, 1]                 # views only: pointers into buf
    shape = pl.shape_of(cfg)
    shape.k_stride_head = shape.v_stride_head = 2 * d
    shape.k_stride_tok = shape.v_stride_tok = H * 2 * d
    q, W = pl.to_device(li.q_win), pl.to_device(li.w_cal)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    score = torch.empty((H, n), device="cuda:0")
    eps = torch.empty((H, n), device="cuda:0")
    vb.vector_score_residual(shape, q, k_view, v_view, W, score, eps, ws)
    torch.cuda.synchronize()
    wide = {x: dg.widen(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    ref_s = vo.score(wide["q_win"], wide["k"], cfg.window, cfg.pool_kernel)
    ref_e = vo.residual(wide["k"], wide["v"], wide["w_cal"])
    w = cfg.window
    close(score.cpu().numpy()[:, : n - w].astype(np.float64) * n, ref_s[:, : n - w].astype(np.float64) * n, "n*score (strided)")
    close(eps.cpu().numpy(), ref_e, "eps (strided)")
    # separate entry points on the same views
    score1 = torch.empty((H, n), device="cuda:0")
    eps1 = torch.empty((H, n), device="cuda:0")
    vb.vector_score(shape, q, k_view, score1, ws)
    vb.vector_residual(shape, k_view, v_view, W, eps1, ws)
    torch.cuda.synchronize()
    close(score1.cpu().numpy()[:, : n - w].astype(np.float64) * n, ref_s[:, : n - w].astype(np.float64) * n, "n*score (strided, own call)")
    close(eps1.cpu().numpy(), ref_e, "eps (strided, own call)")
    # compaction gathers from the strided source, bit for bit
    tier, idx_r, idx_a = vo.route(score.cpu().numpy(), eps.cpu().numpy(), n_p, n_a)
    cap = n_r + 3
    k_ret = torch.zeros((H, cap, d), dtype=torch.bfloat16, device="cuda:0")
    v_ret = torch.zeros_like(k_ret)
    k_apx = torch.zeros((H, n_a, d), dtype=torch.bfloat16, device="cuda:0")
    vb.vector_compact(shape, k_view, v_view, pl.to_device(idx_r.astype(np.int32)), pl.to_device(idx_a.astype(np.int32)),
                      n_r, n_a, k_ret, v_ret, k_apx, cap)
    torch.cuda.synchronize()
    rk, rv, ra = vo.compact(li.k, li.v, idx_r, idx_a)
    assert np.array_equal(pl.to_host(k_ret)[:, :n_r], rk) and np.array_equal(pl.to_host(v_ret)[:, :n_r], rv)
    assert np.array_equal(pl.to_host(k_apx), ra)
    assert not pl.to_host(k_ret)[:, n_r:].any() and not pl.to_host(v_ret)[:, n_r:].any(), "rows past n_retain are the caller's"


def test_one_map_shared_by_all_heads():
    cfg, li = _layer(seq_len=640, n_kv_heads=4, n_q_heads=8, window=8)
    H, n, d = cfg.n_kv_heads, cfg.seq_len, cfg.head_dim
    W1 = li.w_cal[2:3]                                           # one [d, d] map
    shape = pl.shape_of(cfg)
    shape.w_shared = 1
    eps = torch.empty((H, n), device="cuda:0")
    vb.vector_residual(shape, pl.to_device(li.k), pl.to_device(li.v), pl.to_device(W1), eps)
    torch.cuda.synchronize()
    Wb = np.broadcast_to(dg.widen(W1), (H, d, d))
    close(eps.cpu().numpy(), vo.residual(dg.widen(li.k), dg.widen(li.v), Wb), "eps (shared W)")
    # decode with the shared map
    B, Hq, n_r, n_a = 2, cfg.n_q_heads, 40, 50
    rng = np.random.default_rng(3)
    k_ret = dg.f32_to_bf16_bits(rng.standard_normal((B, H, n_r, d)).astype(np.float32))
    v_ret = dg.f32_to_bf16_bits(rng.standard_normal((B, H, n_r, d)).astype(np.float32))
    k_apx = dg.f32_to_bf16_bits(rng.standard_normal((B, H, n_a, d)).astype(np.float32))
    q = dg.f32_to_bf16_bits(rng.standard_normal((B, Hq, d)).astype(np.float32))
    t = [pl.to_device(x) for x in (k_ret, v_ret, k_apx, W1, q)]
    length = torch.full((B,), n_r, dtype=torch.int32, device="cuda:0")
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=n_r, n_approx=n_a,
                     w_shared=1)
    cache.len_retain, cache.k_ret, cache.v_ret, cache.k_apx, cache.W = (length.data_ptr(), t[0].data_ptr(), t[1].data_ptr(),
                                                                      t[2].data_ptr(), t[3].data_ptr())
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(pl.shape_of(cfg), n_r + n_a, n_a, B))
    scale = 1.0 / np.sqrt(d)
    ref = vo.decode_attn(dg.widen(q), dg.widen(k_ret), dg.widen(v_ret), np.full(B, n_r), dg.widen(k_apx), Wb, scale)
    decode_check(cache, t[4], scale, ws, ref, "decode (shared W)")


def test_errors_are_reported_before_any_launch():
    cfg, li = _layer(seq_len=256, n_kv_heads=1, n_q_heads=4, window=8)
    H, n = cfg.n_kv_heads, cfg.seq_len
    n_r, n_a, n_p = cfg.counts()
    dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    shape = pl.shape_of(cfg)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    sentinel = 123.0
    score = torch.full((H, n), sentinel, device="cuda:0")
    eps = torch.full((H, n), sentinel, device="cuda:0")

    def code_of(fn):
        with pytest.raises(vb.VectorError) as ei:
            fn()
        return ei.value.code

    def with_shape(**kw):
        s = pl.shape_of(cfg)
        for k, v in kw.items():
            setattr(s, k, v)
        return s

    run = lambda s, w=ws: vb.vector_score_residual(s, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], score, eps, w)
    assert code_of(lambda: run(with_shape(head_dim=96))) == vb.VECTOR_ERR_SHAPE
    assert code_of(lambda: run(with_shape(dtype=7))) == vb.VECTOR_ERR_DTYPE
    assert code_of(lambda: run(with_shape(window=n + 1))) == vb.VECTOR_ERR_SHAPE
    assert code_of(lambda: run(with_shape(pool_kernel=4))) == vb.VECTOR_ERR_SHAPE
    assert code_of(lambda: run(with_shape(pool_mode=2))) == vb.VECTOR_ERR_SHAPE
    assert code_of(lambda: run(with_shape(n_q_heads=3, n_kv_heads=2))) == vb.VECTOR_ERR_SHAPE
    assert code_of(lambda: run(with_shape(k_stride_tok=cfg.head_dim - 8))) == vb.VECTOR_ERR_SHAPE
    assert code_of(lambda: run(shape, ws[:256])) == vb.VECTOR_ERR_WORKSPACE        # too small
    assert code_of(lambda: run(shape, ws[8:])) == vb.VECTOR_ERR_WORKSPACE          # misaligned
    assert code_of(lambda: vb.vector_score_residual(shape, dev["q_win"], None, dev["v"], dev["w_cal"], score, eps, ws)) == vb.VECTOR_ERR_ARG
    assert code_of(lambda: vb.vector_score_residual(shape, dev["q_win"], dev["k"].view(torch.int16).flatten()[1:], dev["v"],
                                                    dev["w_cal"], score, eps, ws)) == vb.VECTOR_ERR_ARG   # 2-byte offset
    tier = torch.full((H, n), 77, dtype=torch.uint8, device="cuda:0")
    idx_r = torch.full((H, n), -5, dtype=torch.int32, device="cuda:0")
    idx_a = torch.full((H, n), -5, dtype=torch.int32, device="cuda:0")
    assert code_of(lambda: vb.vector_route(H, n, score, eps, n + 1, 0, tier, idx_r, idx_a, ws)) == vb.VECTOR_ERR_ARG
    assert code_of(lambda: vb.vector_route(H, n, score, eps, 10, 11, tier, idx_r, idx_a, ws)) == vb.VECTOR_ERR_ARG
    torch.cuda.synchronize()
    assert (score == sentinel).all() and (eps == sentinel).all(), "a failing call must not write"
    assert (tier == 77).all() and (idx_r == -5).all() and (idx_a == -5).all()


@pytest.mark.parametrize("base,over", [
    ("cfg2", dict(seq_len=2048, n_kv_heads=2, n_q_heads=8)),
    ("cfg2", dict(seq_len=1777, n_kv_heads=2, n_q_heads=8, window=24, pool_kernel=5)),
    ("cfg2", dict(seq_len=4096, n_kv_heads=1, n_q_heads=4, pool_kernel=1)),
    ("cfg2", dict(seq_len=3000, n_kv_heads=1, n_q_heads=4, pool_kernel=13)),
    ("cfg1", dict(seq_len=1000, window=20, n_q_heads=6, n_kv_heads=2)),
    ("cfg2", dict(seq_len=40000, n_kv_heads=1, n_q_heads=2, window=16)),           # several chunks per head
    ("cfg2", dict(seq_len=2500, n_kv_heads=2, n_q_heads=8, f_approx=0.0)),          # nothing approximated
    ("cfg2", dict(seq_len=2500, n_kv_heads=2, n_q_heads=8, f_retain=0.0)),          # nothing retained
    ("cfg1", dict(seq_len=3000, head_dim=128, n_kv_heads=1, n_q_heads=2, window=8)),   # fp32 rows of 512 bytes
    ("cfg2", dict(seq_len=4500, n_kv_heads=2, n_q_heads=4, pool_mode="max")),
])
def test_one_call_pass_equals_the_three_calls(base, over):
    cfg = dg.scaled(dg.CONFIGS[base], **over)
    li = wl.make_layer(cfg, 0)
    shape = pl.shape_of(cfg)
    n_r, n_a, n_p = cfg.counts()
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
    a = pl.alloc_outputs(shape, n_p, n_a, n_r + 1, tdt)
    b = pl.alloc_outputs(shape, n_p, n_a, n_r + 1, tdt)
    ws_a = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
    ws_b = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a))
    pl.compress_layer(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], n_p, n_a, a, ws_a)
    pl.compress_layer(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], n_p, n_a, b, ws_b, one_call=True)
    torch.cuda.synchronize()
    for name in ("score", "eps", "tier", "idx_retain", "idx_approx", "k_ret", "v_ret", "k_apx"):
        x, y = getattr(a, name), getattr(b, name)
        if x.dtype == torch.bfloat16:
            x, y = x.view(torch.int16), y.view(torch.int16)
        assert torch.equal(x, y), name


def test_query_row_limit():
    """The query rows of a KV head are staged in LDS.  288 rows go in one group; 320 rows go as
    groups of query heads; a single head's window that does not fit is refused."""
    def run(cfg):
        li = wl.make_layer(cfg, 0)
        shape = pl.shape_of(cfg)
        n_r, n_a, n_p = cfg.counts()
        dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
        ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1))
        score = torch.empty((1, cfg.seq_len), device="cuda:0")
        eps = torch.empty((1, cfg.seq_len), device="cuda:0")
        vb.vector_score_residual(shape, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], score, eps, ws)
        torch.cuda.synchronize()
        return li, score.cpu().numpy(), eps.cpu().numpy()
    for window in (72, 80):                                                                      # 288 and 320 rows
        cfg = dg.scaled(dg.CONFIGS["cfg2"], seq_len=600, n_kv_heads=1, n_q_heads=4, window=window)
        li, score, eps = run(cfg)
        ref = vo.score(dg.widen(li.q_win), dg.widen(li.k), window, cfg.pool_kernel)
        m = 600 - window
        close(score[:, :m].astype(np.float64) * 600, ref[:, :m].astype(np.float64) * 600, f"n*score ({4 * window} rows)")
        close(eps, vo.residual(dg.widen(li.k), dg.widen(li.v), dg.widen(li.w_cal)), f"eps ({4 * window} rows)")
    too_wide = dg.scaled(dg.CONFIGS["cfg2"], seq_len=600, n_kv_heads=1, n_q_heads=1, window=300)  # one head, 300 rows
    with pytest.raises(vb.VectorError) as ei:
        run(too_wide)
    assert ei.value.code == vb.VECTOR_ERR_SHAPE


def test_layers_stacked_along_the_head_axis():
    """Every step is independent per KV head: four layers stacked as 8 heads give, head for head,
    exactly what the four separate calls give."""
    cfg = dg.scaled(dg.CONFIGS["cfg2"], seq_len=2048, n_kv_heads=2, n_q_heads=8)
    lis = [wl.make_layer(cfg, l) for l in range(4)]
    n_r, n_a, n_p = cfg.counts()
    shape1 = pl.shape_of(cfg)
    singles = []
    for li in lis:
        dev = {x: pl.to_device(getattr(li, x)) for x in ("q_win", "k", "v", "w_cal")}
        out = pl.alloc_outputs(shape1, n_p, n_a, n_r, torch.bfloat16)
        ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape1, n_p, n_a, 1))
        pl.compress_layer(shape1, dev["q_win"], dev["k"], dev["v"], dev["w_cal"], n_p, n_a, out, ws)
        singles.append(out)
    big = dg.scaled(cfg, n_kv_heads=8, n_q_heads=32)
    shape4 = pl.shape_of(big)
    stack = {x: pl.to_device(np.concatenate([getattr(li, x) for li in lis], axis=0)) for x in ("q_win", "k", "v", "w_cal")}
    out4 = pl.alloc_outputs(shape4, n_p, n_a, n_r, torch.bfloat16)
    ws4 = pl.alloc_workspace(vb.vector_workspace_bytes(shape4, n_p, n_a, 1))
    pl.compress_layer(shape4, stack["q_win"], stack["k"], stack["v"], stack["w_cal"], n_p, n_a, out4, ws4)
    torch.cuda.synchronize()
    for name in ("score", "eps", "tier", "idx_retain", "idx_approx", "k_ret", "v_ret", "k_apx"):
        got = getattr(out4, name)
        want = torch.cat([getattr(o, name) for o in singles], dim=0)
        if got.dtype == torch.bfloat16:
            got, want = got.view(torch.int16), want.view(torch.int16)
        assert torch.equal(got, want), name


def test_read_stream_probe_reads_what_it_reports():
    """The read-only streaming probe reads whole rounds of 64 KiB per workgroup and nothing beyond
    the buffer, leaves its sink alone, and refuses buffers it cannot cut that way."""
    import ctypes as C
    src = torch.ones(96 * 1024 * 1024 + 4096, dtype=torch.uint8, device="cuda:0")     # one and a half rounds
    sink = torch.zeros(1024, dtype=torch.float32, device="cuda:0")
    assert vb.vector_probe_read_stream(src, sink) == 64 * 1024 * 1024
    assert vb.vector_probe_read_stream(src[: 64 * 1024 * 1024], sink) == 64 * 1024 * 1024
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0
    n = C.c_int64()
    L = vb.lib()
    too_small = src[: 32 * 1024 * 1024]
    assert L.vector_probe_read_stream(too_small.data_ptr(), too_small.numel(), sink.data_ptr(), C.byref(n), None) == -1
    assert L.vector_probe_read_stream(src.data_ptr() + 4, src.numel() - 4, sink.data_ptr(), C.byref(n), None) == -1
    assert L.vector_probe_read_stream(None, src.numel(), sink.data_ptr(), C.byref(n), None) == -1
