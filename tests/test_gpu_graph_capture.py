"""The entry points enqueue kernels only (no allocation, no host wait, no memset), so a caller can
record them into a HIP graph.  A captured compression pass and a captured decode step (whose live
length lives on the device and advances inside the step) are replayed several times, with eager
work and synchronisations between the replays, and every replay is held against the eager result."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
from paper_2605_23258_amd import pipeline as pl
import workloads as wl

pytestmark = pytest.mark.gpu


def test_compression_pass_replays_bit_for_bit():
    cfg = dg.scaled(dg.CONFIGS["cfg2"], seq_len=3000, n_kv_heads=2, n_q_heads=8, window=24)
    n_r, n_a, n_p = cfg.counts()
    shape = pl.shape_of(cfg)
    layers = [wl.make_layer(cfg, i) for i in range(2)]
    # static input buffers: a replay reads whatever they hold at that time
    buf = {x: pl.to_device(getattr(layers[0], x)) for x in ("q_win", "k", "v", "w_cal")}
    ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a))
    out = pl.alloc_outputs(shape, n_p, n_a, n_r, torch.bfloat16)
    eager = []
    for li in layers:
        for x in buf:
            buf[x].copy_(pl.to_device(getattr(li, x)))
        ref = pl.alloc_outputs(shape, n_p, n_a, n_r, torch.bfloat16)
        pl.compress_layer(shape, buf["q_win"], buf["k"], buf["v"], buf["w_cal"], n_p, n_a, ref, ws, one_call=True)
        torch.cuda.synchronize()
        eager.append(ref)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream, as torch asks for
        pl.compress_layer(shape, buf["q_win"], buf["k"], buf["v"], buf["w_cal"], n_p, n_a, out, ws, stream=side, one_call=True)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pl.compress_layer(shape, buf["q_win"], buf["k"], buf["v"], buf["w_cal"], n_p, n_a, out, ws,
                          stream=torch.cuda.current_stream(), one_call=True)
    for rep in range(4):
        li, ref = layers[rep % 2], eager[rep % 2]
        for x in buf:
            buf[x].copy_(pl.to_device(getattr(li, x)))
        out.tier.fill_(7)                               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in ("score", "eps", "tier", "idx_retain", "idx_approx", "k_ret", "v_ret", "k_apx"):
            assert torch.equal(getattr(out, name), getattr(ref, name)), f"replay {rep}: {name}"


def test_decode_step_replays_and_advances_its_length():
    d, Hq, H, B, cap, n_a = 128, 8, 2, 3, 200, 90
    g = torch.Generator(device="cuda:0").manual_seed(5)
    rnd = lambda *s: torch.randn(*s, generator=g, device="cuda:0").bfloat16()
    k_ret, v_ret, k_apx, W = rnd(B, H, cap, d), rnd(B, H, cap, d), rnd(B, H, n_a, d), (rnd(H, d, d).float() / d ** 0.5).bfloat16()
    steps = 5
    qs, ks, vs = rnd(steps, B, Hq, d), rnd(steps, B, H, d), rnd(steps, B, H, d)
    start = torch.tensor([100, 0, 190], dtype=torch.int32, device="cuda:0")
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=H, head_dim=d, seq_len=cap, window=1, pool_kernel=1, dtype=vb.VECTOR_BF16)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, cap, 0, B) + (1 << 20))
    scale = 1.0 / float(np.sqrt(d))

    def make_cache(k, v, length):
        c = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=cap, n_approx=n_a)
        c.len_retain, c.k_ret, c.v_ret, c.k_apx, c.W = length.data_ptr(), k.data_ptr(), v.data_ptr(), k_apx.data_ptr(), W.data_ptr()
        return c

    # eager run of the five steps
    ke, ve, le = k_ret.clone(), v_ret.clone(), start.clone()
    ce = make_cache(ke, ve, le)
    eager = torch.empty(steps, B, Hq, d, dtype=torch.float32, device="cuda:0")
    for s in range(steps):
        vb.vector_decode_step(ce, qs[s], ks[s], vs[s], scale, eager[s], ws, flags=vb.VECTOR_DECODE_OUT_F32)
    torch.cuda.synchronize()
    # one captured step on static buffers, replayed five times
    kg, vg, lg = k_ret.clone(), v_ret.clone(), start.clone()
    cg = make_cache(kg, vg, lg)
    q_in, k_in, v_in = qs[0].clone(), ks[0].clone(), vs[0].clone()
    o = torch.empty(B, Hq, d, dtype=torch.float32, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on throw-away state
        kw, vw, lw = k_ret.clone(), v_ret.clone(), start.clone()
        vb.vector_decode_step(make_cache(kw, vw, lw), q_in, k_in, v_in, scale, o, ws, flags=vb.VECTOR_DECODE_OUT_F32, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        vb.vector_decode_step(cg, q_in, k_in, v_in, scale, o, ws, flags=vb.VECTOR_DECODE_OUT_F32, stream=torch.cuda.current_stream())
    assert torch.equal(lg, start), "capture must not run the step"
    for s in range(steps):
        q_in.copy_(qs[s]); k_in.copy_(ks[s]); v_in.copy_(vs[s])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, eager[s]), f"replayed step {s}"
    assert torch.equal(lg, le) and torch.equal(kg, ke) and torch.equal(vg, ve)
