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


def test_batch_of_unequal_sequences_replays_bit_for_bit():
    """The batch call ships its per-sequence parameter tables as arguments of copy launches, so a
    captured call keeps them: replays with other inputs in the same buffers give what the eager
    call gives."""
    cfg = dg.scaled(dg.CONFIGS["cfg2"], n_kv_heads=2, n_q_heads=8, window=32)
    lens = [900, 2500, 333, 1200]
    H, d = cfg.n_kv_heads, cfg.head_dim
    counts = [vb.vector_budget_counts_frac(n, cfg.f_retain, cfg.f_approx) for n in lens]
    n_pool, n_approx = [c[0] for c in counts], [c[1] for c in counts]
    n_ret = [p - a for p, a in zip(n_pool, n_approx)]
    shape = pl.shape_of(cfg, seq_len=1)
    batch, keep = vb.make_batch(lens, n_pool, n_approx, n_ret)
    ws = pl.alloc_workspace(vb.vector_compress_batch_workspace_bytes(shape, batch))
    T, R, A = sum(lens), sum(n_ret), sum(n_approx)

    def draw(seed):
        layers = [wl.make_layer(dg.scaled(cfg, seq_len=n), layer=seed * 10 + b) for b, n in enumerate(lens)]
        return dict(q=pl.to_device(np.stack([li.q_win for li in layers])), k=pl.to_device(np.concatenate([li.k for li in layers], axis=1)),
                    v=pl.to_device(np.concatenate([li.v for li in layers], axis=1)), W=pl.to_device(layers[0].w_cal))

    def outputs():
        return dict(score=torch.full((H * T,), -1.0, device="cuda:0"), eps=torch.full((H * T,), -1.0, device="cuda:0"),
                    tier=torch.full((H * T,), 9, dtype=torch.uint8, device="cuda:0"),
                    ir=torch.full((H * R,), -1, dtype=torch.int32, device="cuda:0"), ia=torch.full((H * A,), -1, dtype=torch.int32, device="cuda:0"),
                    kr=torch.zeros((H * R, d), dtype=torch.bfloat16, device="cuda:0"), vr=torch.zeros((H * R, d), dtype=torch.bfloat16, device="cuda:0"),
                    ka=torch.zeros((H * A, d), dtype=torch.bfloat16, device="cuda:0"))

    def call(buf, o, stream=None):
        vb.vector_compress_batch(shape, batch, buf["q"], buf["k"], buf["v"], buf["W"], o["score"], o["eps"], o["tier"], o["ir"], o["ia"],
                                 o["kr"], o["vr"], o["ka"], ws, stream)

    inputs = [draw(0), draw(1)]
    buf = {x: t.clone() for x, t in inputs[0].items()}
    eager = []
    for inp in inputs:
        for x in buf:
            buf[x].copy_(inp[x])
        ref = outputs()
        call(buf, ref)
        torch.cuda.synchronize()
        eager.append(ref)
    out = outputs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(buf, out, side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(buf, out, torch.cuda.current_stream())
    for rep in range(4):
        inp, ref = inputs[rep % 2], eager[rep % 2]
        for x in buf:
            buf[x].copy_(inp[x])
        out["tier"].fill_(7)
        ws.zero_()                                      # the tables are rewritten by the replay itself
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in out:
            a, b = out[name], ref[name]
            if a.dtype == torch.bfloat16:
                a, b = a.view(torch.int16), b.view(torch.int16)
            assert torch.equal(a, b), f"replay {rep}: {name}"
    del keep
