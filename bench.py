#!/usr/bin/env python3
"""Benchmark of the VECTOR hot path on one MI355X.

One step = one full prefill compression pass of the 32-layer, 32k-token workload
(score + residual, routing, compaction, layer by layer), inputs resident in HBM.
The decode-attention leg (batch 16 over compressed 32k caches, 256 steps) is timed
in the same run and reported in the same JSON line, as is the CPU oracle on a
bounded sample of the compression workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as wl   # noqa: E402  (harness: input draws + the offline least-squares calibration)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def blas_single_thread():
    """Input generation runs one layer per worker thread: keep BLAS from oversubscribing the cores."""
    try:
        from threadpoolctl import threadpool_limits
        return threadpool_limits(limits=1)
    except Exception:
        import contextlib
        return contextlib.nullcontext()


def compress_bytes_per_token_head(cfg) -> dict:
    """Algorithmic HBM bytes per token-head of each kernel of the compression pass
    (bf16, d=128): what a kernel has to read and write once, not what it re-reads."""
    esz = 2 if cfg.dtype == "bf16" else 4
    row = cfg.head_dim * esz
    n_r, n_a, n_p = cfg.counts()
    f_p, f_r = n_p / cfg.seq_len, n_r / cfg.seq_len
    return {
        "score_stats": row,                       # read K
        "mass_residual": 2 * row + 8,             # read K (again) and V, write mass and eps
        "pool_scores": 8,                         # read mass, write score
        "route": 8 + 1 + 8 * f_p,                 # read score, eps; write tier and index lists
        "gather_rows": 2 * row * (f_p + f_r),     # read and write pool K rows and retained V rows
        # the whole pass, counting K and V once: the second streaming read of K that the
        # two-pass softmax makes is not algorithmic
        "pass": 2 * row + 8 + 8 + 1 + 8 * f_p + 2 * row * (f_p + f_r),
    }


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only)")
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-layers", type=int, default=6)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (reference kernel for scaling HBM counters)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the entry points beyond the benchmark workload (post-RoPE variants, calibration, diagnostics)")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams the layers are spread over (layers are independent)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2605_23258_amd import binding as vb
    from paper_2605_23258_amd import datagen as dg
    from paper_2605_23258_amd import pipeline as pl

    vb.lib()                                   # fail loudly if the HIP library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = dg.CONFIGS["cfg3"]
    if args.layers:
        cfg = dg.scaled(cfg, layers=args.layers)
    n_r, n_a, n_p = cfg.counts()
    shape = pl.shape_of(cfg)
    H, n, d = cfg.n_kv_heads, cfg.seq_len, cfg.head_dim
    workers = min(16, os.cpu_count() or 1)

    # ---- inputs: every layer has its own draws; all of them resident in HBM ----
    t0 = time.time()
    def gen(layer):
        li = wl.make_layer(cfg, layer)
        return {k: getattr(li, k) for k in ("q_win", "k", "v", "w_cal")}
    with blas_single_thread(), ThreadPoolExecutor(workers) as ex:
        host_layers = list(ex.map(gen, range(cfg.layers)))
    layers = [{k: pl.to_device(v, dev) for k, v in hl.items()} for hl in host_layers]
    log(f"generated {cfg.layers} layers of K/V [{H},{n},{d}] {cfg.dtype} in {time.time() - t0:.1f}s")
    # Layers are independent, so consecutive layers go to different streams (each with its own
    # workspace): the routing kernel of one layer, which occupies 8 CUs, and the launch ramps
    # of the streaming kernels overlap with the next layer's work.
    n_streams = max(1, args.streams)
    streams = [torch.cuda.Stream(device=dev) for _ in range(n_streams)]
    wss = [pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1), dev) for _ in range(n_streams)]
    outs = [pl.alloc_outputs(shape, n_p, n_a, n_r, torch.bfloat16, dev) for _ in range(cfg.layers)]
    torch.cuda.synchronize()

    def step():
        for i, (L, o) in enumerate(zip(layers, outs)):
            pl.compress_layer(shape, L["q_win"], L["k"], L["v"], L["w_cal"], n_p, n_a, o, wss[i % n_streams],
                              stream=streams[i % n_streams])

    if args.copy_calibration:                  # known traffic: 256 MiB read, 256 MiB written per copy
        src = torch.empty(128 * 1024 * 1024, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = cfg.layers * n * args.steps / elapsed
    log(f"compression pass: {ms_per_step:.3f} ms/step, {tokens_per_s / 1e6:.2f} M KV tokens/s")

    # ---- per-kernel durations over the same steps, HIP events on the launch stream.  The
    # layers run on one stream here: a duration measured while another layer's kernels share
    # the chip says little about the kernel itself ----
    def step_one_stream():
        for L, o in zip(layers, outs):
            pl.compress_layer(shape, L["q_win"], L["k"], L["v"], L["w_cal"], n_p, n_a, o, wss[0], stream=streams[0])
    vb.vector_timing_enable(True)
    for _ in range(args.steps):
        step_one_stream()
    torch.cuda.synchronize()
    timing = vb.vector_timing_read()
    vb.vector_timing_enable(False)
    bpt = compress_bytes_per_token_head(cfg)
    kernels = {}
    for name, (ms, cnt) in timing.items():
        if cnt:
            avg_us = ms / cnt * 1e3
            kernels[name] = {"avg_us": round(avg_us, 2), "launches": cnt}
            if name in bpt:
                kernels[name]["alg_GBs"] = round(bpt[name] * H * n / (avg_us * 1e-6) / 1e9, 1)
    # The roofline kernel is the longest of the kernels that occupy the whole chip.  The routing
    # kernel is listed with the others, but it runs on 8 workgroups (one per KV head) next to the
    # following layer's streaming kernels and moves 13 bytes per token: no bandwidth bound applies.
    chip_wide = [k for k in ("score_stats", "mass_residual", "gather_rows", "pool_scores") if k in kernels]
    dominant = max(chip_wide, key=lambda k: kernels[k]["avg_us"])
    dom_bytes = bpt[dominant] * H * n
    dom_gbs = dom_bytes / (kernels[dominant]["avg_us"] * 1e-6) / 1e9
    sum_us = sum(v["avg_us"] for v in kernels.values())
    pass_bytes = bpt["pass"] * H * n
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if os.path.exists(tpath):                  # rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy
        for line in open(tpath):
            parts = line.split()
            if len(parts) == 2 and parts[0] == dominant:
                traffic = int(parts[1])
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                "bytes_per_launch": int(dom_bytes), "avg_us": kernels[dominant]["avg_us"],
                "pass_alg_bytes_per_layer": int(pass_bytes),
                "pass_frac_of_hbm_peak": round(pass_bytes * cfg.layers / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    # MFMA work of the pass (both softmax passes and the residual contraction)
    G = cfg.group
    flops_layer = H * n * (2 * 2 * G * cfg.window * d + 2 * d * d)
    mfma_tflops = flops_layer * cfg.layers / (ms_per_step * 1e-3) / 1e12
    log(f"kernels: {json.dumps(kernels)} (sum {sum_us:.1f} us per layer)")

    # The reconstruction contraction with memory out of the picture: the residual kernel re-runs
    # each tile's arithmetic `repeat` times on operands it already holds; the time added per
    # extra repeat is one pass of the contraction code at the rate the matrix cores sustain.
    def probe_ms(repeat, launches=10):
        x = layers[0]
        o = outs[0]
        vb.vector_probe_residual_mfma(shape, x["k"], x["v"], x["w_cal"], o.eps, repeat)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(launches):
            vb.vector_probe_residual_mfma(shape, x["k"], x["v"], x["w_cal"], o.eps, repeat)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / launches * 1e3
    r_hi = 17
    t_lo, t_hi = probe_ms(1), probe_ms(r_hi)
    res_flops = H * n * 2 * d * d
    iso_tflops = res_flops / ((t_hi - t_lo) / (r_hi - 1) * 1e-3) / 1e12
    log(f"residual contraction probe: repeat 1 {t_lo * 1e3:.1f} us, repeat {r_hi} {t_hi * 1e3:.1f} us -> {iso_tflops:.0f} TFLOP/s isolated")

    # ---- decode attention over compressed caches ----
    decode = None
    if not args.no_decode:
        decode = run_decode(args, vb, dg, pl, torch, np, dev, workers)

    # ---- CPU oracle on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import vector_oracle as vo
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            blas_threads = 1
        ns = min(args.cpu_sample_layers, cfg.layers)
        t0 = time.perf_counter()
        for hl in host_layers[:ns]:
            wide = {k: dg.widen(v) for k, v in hl.items()}
            s = vo.score(wide["q_win"], wide["k"], cfg.window, cfg.pool_kernel)
            e = vo.residual(wide["k"], wide["v"], wide["w_cal"])
            _, ir, ia = vo.route(s, e, n_p, n_a)
            vo.compact(hl["k"], hl["v"], ir, ia)
        dt = time.perf_counter() - t0
        cpu = {"value": round(ns * n / dt, 1), "unit": "KV tokens/s", "cores": int(blas_threads), "kind": "oracle",
               "sample": f"{ns} of {cfg.layers} layers of the same workload, {dt:.1f}s (numpy fp64; BLAS threads as listed, Python loops single-threaded)"}
        log(f"cpu oracle: {cpu}")

    extras = None
    if args.extras:
        extras = run_extras(vb, dg, pl, torch, np, dev, cfg, shape, layers[0], outs[0], wss[0], n_p, n_a)
        extras.update(run_stacked(vb, pl, torch, dev, cfg, layers, n_p, n_a, n_r))

    line = {
        "metric": "KV tokens compressed/sec (prefill pass)", "value": round(tokens_per_s, 1), "unit": "KV tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg3: {cfg.layers}-layer compression pass, n={n}, Hq/Hkv={cfg.n_q_heads}/{H}, d={d}, "
                               f"window={cfg.window}, pool={cfg.pool_kernel}, retain/approx={n_r}/{n_a} per head",
                   "seed": dg.MASTER_SEED, "streams": n_streams},
        "roofline": roofline,
        "kernels": kernels,
        "mfma": {"achieved_TFLOPs": round(mfma_tflops, 1), "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
                 "frac": round(mfma_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                 "residual_contraction_isolated_TFLOPs": round(iso_tflops, 1),
                 "residual_contraction_isolated_frac": round(iso_tflops / MFMA_BF16_PEAK_TFLOPS, 4)},
        "decode": decode,
        "cpu_baseline": cpu,
    }
    if extras is not None:
        line["extras"] = extras
    print(json.dumps(line), flush=True)


def run_stacked(vb, pl, torch, dev, cfg, layers, n_p, n_a, n_r):
    """The same 32 layers as one call per entry point: every step of the path is independent per KV
    head, so layers stacked along the head axis ([layers * Hkv, n, d]) are just more heads.  Not the
    benchmark's configuration (which compresses layer by layer); it shows what the kernels sustain
    once their launch ramps are amortised."""
    L, H, Hq = len(layers), cfg.n_kv_heads, cfg.n_q_heads
    stack = {k: torch.cat([x[k] for x in layers], dim=0).contiguous() for k in ("q_win", "k", "v", "w_cal")}
    shape = vb.Shape(n_q_heads=Hq * L, n_kv_heads=H * L, head_dim=cfg.head_dim, seq_len=cfg.seq_len, window=cfg.window,
                     pool_kernel=cfg.pool_kernel, dtype=vb.VECTOR_BF16)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, 1), dev)
    out = pl.alloc_outputs(shape, n_p, n_a, n_r, torch.bfloat16, dev)
    run = lambda: pl.compress_layer(shape, stack["q_win"], stack["k"], stack["v"], stack["w_cal"], n_p, n_a, out, ws)
    run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / 5
    vb.vector_timing_enable(True)
    run()
    torch.cuda.synchronize()
    t = vb.vector_timing_read()
    vb.vector_timing_enable(False)
    res = {"stacked_layers_ms_per_pass": round(dt * 1e3, 3), "stacked_layers_KV_tokens_per_s": round(L * cfg.seq_len / dt, 1),
           "stacked_layers_kernel_us_per_layer": {k: round(ms / L * 1e3, 2) for k, (ms, c) in t.items() if c}}
    log(f"stacked: {res}")
    return res


def run_extras(vb, dg, pl, torch, np, dev, cfg, shape, layer, out, ws, n_p, n_a):
    """Entry points outside the benchmark workload, timed as back-to-back launches on one stream
    (wall clock per call, synchronised at both ends)."""
    H, n, d = cfg.n_kv_heads, cfg.seq_len, cfg.head_dim

    def per_call_us(fn, calls=20):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(calls):
            fn()
        torch.cuda.synchronize()
        return round((time.perf_counter() - t0) / calls * 1e6, 1)

    res = {}
    inv_freq = dg.rotary_inv_freq(d, 500000.0)
    rope, keep = vb.make_rope(inv_freq, None, False, 0)
    # the cfg-3 layer read as a post-RoPE cache (same bytes; the un-rotation does the same work on any keys)
    res["score_residual_rope_us_per_layer"] = per_call_us(
        lambda: vb.vector_score_residual_rope(shape, layer["q_win"], layer["k"], layer["v"], layer["w_cal"], rope, out.score, out.eps, ws))
    res["score_residual_us_per_layer"] = per_call_us(
        lambda: vb.vector_score_residual(shape, layer["q_win"], layer["k"], layer["v"], layer["w_cal"], out.score, out.eps, ws))
    # decode over a cfg-5 shaped cache of random rows, with and without the un-rotation
    c5 = dg.CONFIGS["cfg5"]
    n_r5, n_a5, n_p5 = c5.counts()
    B = c5.batch
    g = torch.Generator(device=dev).manual_seed(7)
    rnd = lambda *sh: torch.randn(*sh, generator=g, device=dev, dtype=torch.float32).bfloat16()
    k_ret, v_ret, k_apx = rnd(B, H, n_r5, d), rnd(B, H, n_r5, d), rnd(B, H, n_a5, d)
    q = rnd(B, c5.n_q_heads, d)
    pos = torch.sort(torch.randint(0, c5.seq_len, (B, H, n_a5), generator=g, device=dev, dtype=torch.int32), dim=-1).values.contiguous()
    length = torch.full((B,), n_r5, dtype=torch.int32, device=dev)
    cache = vb.Cache(batch=B, n_q_heads=c5.n_q_heads, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=n_r5, n_approx=n_a5)
    cache.len_retain, cache.k_ret, cache.v_ret = length.data_ptr(), k_ret.data_ptr(), v_ret.data_ptr()
    cache.k_apx, cache.W = k_apx.data_ptr(), layer["w_cal"].data_ptr()
    ws5 = pl.alloc_workspace(vb.vector_workspace_bytes(pl.shape_of(c5), n_p5, n_a5, B), dev)
    o5 = torch.empty((B, c5.n_q_heads, d), dtype=torch.bfloat16, device=dev)
    rope5, keep5 = vb.make_rope(inv_freq, pos, False, 0)
    scale = 1.0 / float(np.sqrt(d))
    res["decode_attn_rope_us_per_step"] = per_call_us(lambda: vb.vector_decode_attn_rope(cache, rope5, q, scale, o5, ws5), 50)
    res["decode_attn_us_per_step"] = per_call_us(lambda: vb.vector_decode_attn(cache, q, scale, o5, ws5), 50)
    res["decode_attn_literal_us_per_step"] = per_call_us(
        lambda: vb.vector_decode_attn(cache, q, scale, o5, ws5, flags=vb.VECTOR_DECODE_LITERAL), 50)
    # calibration on 262144 tokens per head (random keys, values linear in them plus noise)
    m = 262144
    kc = rnd(H, m, d)
    vc = (kc.float() @ (torch.randn(H, d, d, generator=g, device=dev) / d ** 0.5) + 0.1 * torch.randn(H, m, d, generator=g, device=dev)).bfloat16()
    cshape = vb.Shape(n_q_heads=H, n_kv_heads=H, head_dim=d, seq_len=m, window=1, pool_kernel=1, dtype=vb.VECTOR_BF16)
    wsc = pl.alloc_workspace(vb.vector_calibrate_workspace_bytes(cshape), dev)
    Wc = torch.empty((H, d, d), dtype=torch.bfloat16, device=dev)
    us = per_call_us(lambda: vb.vector_calibrate(cshape, kc, vc, Wc, wsc), 5)
    res["calibrate_262144_tokens_us"] = us
    res["calibrate_gram_flops"] = int(H * 2 * 2 * m * d * d)
    del kc, vc
    # the query-agnostic scorer on the same keys
    wsk = pl.alloc_workspace(vb.vector_score_key_diversity_workspace_bytes(shape), dev)
    sk = torch.empty((H, n), device=dev)
    res["score_key_diversity_us_per_layer"] = per_call_us(lambda: vb.vector_score_key_diversity(shape, layer["k"], sk, wsk))
    # diagnostics on the layer's own routing
    dout = torch.empty((H, len(vb.DISTORTION_FIELDS)), dtype=torch.float64, device=dev)
    wsd = pl.alloc_workspace(vb.vector_distortion_workspace_bytes(shape), dev)
    wts = torch.softmax(torch.randn(H, n, generator=g, device=dev), dim=-1)
    res["distortion_us_per_layer"] = per_call_us(lambda: vb.vector_distortion(shape, wts, out.tier, out.eps, layer["v"], dout, wsd))
    log(f"extras: {res}")
    return res


def run_decode(args, vb, dg, pl, torch, np, dev, workers):
    """Batch-16 decode over caches produced by the compression pass (routing fixed at prefill)."""
    cfg = dg.CONFIGS["cfg5"]
    n_r, n_a, n_p = cfg.counts()
    B, H, Hq, d, n = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.seq_len
    steps = args.decode_steps
    cap = n_r + steps
    shape = pl.shape_of(cfg)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_p, n_a, B), dev)
    k_ret = torch.zeros((B, H, cap, d), dtype=torch.bfloat16, device=dev)
    v_ret = torch.zeros((B, H, cap, d), dtype=torch.bfloat16, device=dev)
    k_apx = torch.zeros((B, H, n_a, d), dtype=torch.bfloat16, device=dev)
    t0 = time.time()
    with blas_single_thread(), ThreadPoolExecutor(workers) as ex:
        seqs = list(ex.map(lambda b: wl.make_layer(cfg, 0, sub=b), range(B)))
    # the first sequence's map is used for every sequence: W belongs to the layer, not the sequence
    W = pl.to_device(seqs[0].w_cal, dev)
    scratch = pl.alloc_outputs(shape, n_p, n_a, 1, torch.bfloat16, dev)
    for b, li in enumerate(seqs):
        q_win, k, v = (pl.to_device(getattr(li, x), dev) for x in ("q_win", "k", "v"))
        vb.vector_score_residual(shape, q_win, k, v, W, scratch.score, scratch.eps, ws)
        vb.vector_route(H, n, scratch.score, scratch.eps, n_p, n_a, scratch.tier, scratch.idx_retain, scratch.idx_approx, ws)
        vb.vector_compact(shape, k, v, scratch.idx_retain, scratch.idx_approx, n_r, n_a, k_ret[b], v_ret[b], k_apx[b], cap)
    torch.cuda.synchronize()
    log(f"decode: built {B} compressed caches ({n_r} retained + {n_a} approximated of {n}) in {time.time() - t0:.1f}s")
    qs, ks, vs = [], [], []
    for s in range(steps):
        q, k, v = dg.make_decode_step(cfg, s)
        qs.append(q); ks.append(k); vs.append(v)
    qs = pl.to_device(np.stack(qs), dev)            # [steps, B, Hq, d]
    ks = pl.to_device(np.stack(ks), dev)            # [steps, B, H, d]
    vs = pl.to_device(np.stack(vs), dev)
    length = torch.full((B,), n_r, dtype=torch.int32, device=dev)
    out = torch.empty((steps, B, Hq, d), dtype=torch.bfloat16, device=dev)
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=cap, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret = length.data_ptr(), k_ret.data_ptr(), v_ret.data_ptr()
    cache.k_apx, cache.W = k_apx.data_ptr(), W.data_ptr()
    scale = 1.0 / float(np.sqrt(d))

    def loop(timed: bool):
        length.fill_(n_r)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            # the new token's exact key and value join the retained segment, then it attends
            k_ret[:, :, n_r + s] = ks[s]
            v_ret[:, :, n_r + s] = vs[s]
            length.add_(1)
            vb.vector_decode_attn(cache, qs[s], scale, out[s], ws)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    loop(False)                                     # warm-up
    wall = loop(True)
    # attention alone, back to back: every appended row is in place after the loops above, so
    # step s only needs its own live length (read from a precomputed table, no extra kernel)
    lengths = (torch.arange(steps, dtype=torch.int32, device=dev) + (n_r + 1))[:, None].expand(steps, B).contiguous()
    q_l, out_l, len_l = list(qs.unbind(0)), list(out.unbind(0)), [lengths[s].data_ptr() for s in range(steps)]

    def attn_only():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            cache.len_retain = len_l[s]
            vb.vector_decode_attn(cache, q_l[s], scale, out_l[s], ws)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    attn_only()
    attn_us = min(attn_only() for _ in range(3)) / steps * 1e6
    vb.vector_timing_enable(True)
    attn_only()
    timing = vb.vector_timing_read()
    vb.vector_timing_enable(False)
    row = d * 2
    mean_appended = (steps + 1) / 2.0
    bytes_step = B * H * (n_p + n_r + 2 * mean_appended) * row + 2 * B * Hq * row
    gbs = bytes_step / (attn_us * 1e-6) / 1e9
    res = {"workload": f"cfg5: batch {B}, {Hq}/{H} heads, d={d}, {n_r} retained + {n_a} approximated per head of {n}, {steps} steps",
           "attn_us_per_step": round(attn_us, 2), "alg_bytes_per_step": int(bytes_step), "achieved_GBs": round(gbs, 1),
           "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
           "step_us_with_append": round(wall / steps * 1e6, 2),
           "kernels": {k: round(timing[k][0] / max(timing[k][1], 1) * 1e3, 2) for k in ("decode_split", "decode_combine")}}
    log(f"decode: {res}")
    return res


if __name__ == "__main__":
    main()
