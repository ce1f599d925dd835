#!/usr/bin/env python3
"""Benchmark of the VECTOR hot path on one MI355X.

One step = one full prefill compression pass of the 32-layer, 32k-token workload
(score + residual, routing, compaction), strictly layer by layer on one stream, inputs
resident in HBM.  The same JSON line carries: per-kernel durations (HIP events on the launch
stream), the roofline of the longest kernel and of the two streaming kernels together, the
matrix-core figures of the contractions as they run, the single-layer 8k and 128k workloads,
the decode-attention leg (batch 16 over compressed 32k caches, 256 steps), peaks measured
in the same run (device copy, register-only MFMA loop), and the CPU oracle on a bounded sample
of the compression workload (single-threaded and on all threads).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
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


def blas_threads(n):
    try:
        from threadpoolctl import threadpool_limits
        return threadpool_limits(limits=n)
    except Exception:
        import contextlib
        return contextlib.nullcontext()


def compress_bytes_per_token_head(cfg) -> dict:
    """Algorithmic HBM bytes per token-head of each kernel of the compression pass: what has to be
    read and written once.  K is counted once across the two softmax passes (in the first); the
    second streaming read of K that the two-pass softmax makes is not algorithmic and shows up
    under `executed`."""
    esz = 2 if cfg.dtype == "bf16" else 4
    row = cfg.head_dim * esz
    n_r, n_a, n_p = cfg.counts()
    f_p, f_r = n_p / cfg.seq_len, n_r / cfg.seq_len
    alg = {
        "score_stats": row,                       # read K
        "mass_residual": row + 8,                 # read V, write mass and eps (K again: not algorithmic)
        "pool_scores": 8,                         # read mass, write score
        "route": 8 + 1 + 8 * f_p,                 # read score, eps; write tier and index lists
        "gather_rows": 2 * row * (f_p + f_r),     # read and write pool K rows and retained V rows
    }
    alg["pass"] = sum(alg.values())
    alg["score_residual_pair"] = alg["score_stats"] + alg["mass_residual"]
    executed = dict(alg)
    executed["mass_residual"] = 2 * row + 8
    executed["pass"] = alg["pass"] + row
    return {"algorithmic": alg, "executed": executed}


def profile_value(fname: str, key: str):
    """A figure from a committed rocprofv3 summary under profiles/ (two columns: name, value)."""
    path = os.path.join(ROOT, "profiles", fname)
    if os.path.exists(path):
        for line in open(path):
            parts = line.split()
            if len(parts) >= 2 and parts[0] == key:
                try:
                    return float(parts[1])
                except ValueError:
                    return None
    return None


def timed(fn, torch, iters):
    """Wall-clock seconds per call of fn, device idle before and after."""
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / iters


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only)")
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the single-layer 8k / 128k workloads and the measured peaks")
    ap.add_argument("--cpu-sample-layers", type=int, default=24)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (reference kernel for scaling HBM counters)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the entry points beyond the benchmark workload (post-RoPE variants, calibration, diagnostics)")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams the layers of the timed region are spread over (1 = layer by layer, the workload as stated)")
    ap.add_argument("--overlap-streams", type=int, default=3,
                    help="also report the pass with the layers spread over this many streams (0 = skip)")
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
    with blas_threads(1), ThreadPoolExecutor(workers) as ex:
        host_layers = list(ex.map(gen, range(cfg.layers)))
    layers = [{k: pl.to_device(v, dev) for k, v in hl.items()} for hl in host_layers]
    log(f"generated {cfg.layers} layers of K/V [{H},{n},{d}] {cfg.dtype} in {time.time() - t0:.1f}s")
    max_streams = max(1, args.streams, args.overlap_streams)
    streams = [torch.cuda.Stream(device=dev) for _ in range(max_streams)]
    ws_bytes = vb.vector_compress_workspace_bytes(shape, n_p, n_a)
    wss = [pl.alloc_workspace(ws_bytes, dev) for _ in range(max_streams)]
    outs = [pl.alloc_outputs(shape, n_p, n_a, n_r, torch.bfloat16, dev) for _ in range(cfg.layers)]
    torch.cuda.synchronize()

    def make_step(n_streams):
        def step():
            for i, (L, o) in enumerate(zip(layers, outs)):
                pl.compress_layer(shape, L["q_win"], L["k"], L["v"], L["w_cal"], n_p, n_a, o, wss[i % n_streams],
                                  stream=streams[i % n_streams], one_call=True)
        return step

    if args.copy_calibration:                  # known traffic: 256 MiB read, 256 MiB written per copy
        src = torch.empty(128 * 1024 * 1024, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    step = make_step(max(1, args.streams))
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
    log(f"compression pass ({max(1, args.streams)} stream): {ms_per_step:.3f} ms/step, {tokens_per_s / 1e6:.2f} M KV tokens/s")

    overlap = None
    if args.overlap_streams > 1:               # named extra: consecutive layers' passes allowed to overlap
        ostep = make_step(args.overlap_streams)
        dt = timed(ostep, torch, max(3, args.steps // 2))
        overlap = {"streams": args.overlap_streams, "ms_per_step": round(dt * 1e3, 4),
                   "KV_tokens_per_s": round(cfg.layers * n / dt, 1),
                   "note": "layers round-robin over several streams; not the headline: the workload runs layer by layer"}
        log(f"overlapped: {overlap}")

    # ---- per-kernel durations over the same steps, HIP events on the launch stream ----
    vb.vector_timing_enable(True)
    one = make_step(1)
    for _ in range(args.steps):
        one()
    torch.cuda.synchronize()
    timing = vb.vector_timing_read()
    vb.vector_timing_enable(False)
    bpt = compress_bytes_per_token_head(cfg)
    alg, executed = bpt["algorithmic"], bpt["executed"]
    units = H * n
    kernels = {}
    for name, (ms, cnt) in timing.items():
        if cnt:
            avg_us = ms / cnt * 1e3
            kernels[name] = {"avg_us": round(avg_us, 2), "launches": cnt}
            if name in alg:
                kernels[name]["alg_GBs"] = round(alg[name] * units / (avg_us * 1e-6) / 1e9, 1)
    sum_us = sum(v["avg_us"] for v in kernels.values())
    # The roofline kernel is the longest kernel of the pass, whichever it is.
    dominant = max(kernels, key=lambda k: kernels[k]["avg_us"])
    dom_bytes = alg[dominant] * units
    dom_gbs = dom_bytes / (kernels[dominant]["avg_us"] * 1e-6) / 1e9
    pass_bytes = alg["pass"] * units
    pair_us = kernels.get("score_stats", {}).get("avg_us", 0.0) + kernels.get("mass_residual", {}).get("avg_us", 0.0)
    pair_bytes = alg["score_residual_pair"] * units
    traffic = profile_value("hbm_traffic.txt", dominant)
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
                "traffic": int(traffic) if traffic else None,
                "traffic_source": "profiles/hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE of a committed profile run, not measured in this run",
                "bytes_per_launch": int(dom_bytes), "executed_bytes_per_launch": int(executed[dominant] * units),
                "avg_us": kernels[dominant]["avg_us"],
                "accounting": "algorithmic bytes, K counted once across the two softmax passes",
                "score_residual_pair": {"kernels": ["score_stats", "mass_residual"], "bytes_per_layer": int(pair_bytes),
                                        "us_per_layer": round(pair_us, 2),
                                        "achieved": round(pair_bytes / (pair_us * 1e-6) / 1e9, 1) if pair_us else None,
                                        "frac": round(pair_bytes / (pair_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4) if pair_us else None},
                "pass_alg_bytes_per_layer": int(pass_bytes),
                "pass_frac_of_hbm_peak": round(pass_bytes * cfg.layers / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    log(f"kernels: {json.dumps(kernels)} (sum {sum_us:.1f} us per layer)")

    # ---- matrix cores: the contractions as they run inside the two streaming kernels ----
    G = cfg.group
    flops_exec = units * (2 * 2 * G * cfg.window * d + 2 * d * d)      # both softmax passes and the residual
    flops_alg = units * (2 * G * cfg.window * d + 2 * d * d)           # one Q K^T and K W
    mfma_run = flops_exec / (pair_us * 1e-6) / 1e12 if pair_us else None
    intensity = flops_alg / pass_bytes                                  # flop per algorithmic byte of the pass
    attainable = min(MFMA_BF16_PEAK_TFLOPS, intensity * HBM_PEAK_GBS / 1e3)

    # The reconstruction contraction with memory out of the picture: the residual kernel re-runs
    # each tile's arithmetic `repeat` times on operands it already holds; the time added per
    # extra repeat is one pass of the contraction code at the rate the matrix cores sustain.
    def probe_ms(repeat, launches=10):
        x, o = layers[0], outs[0]
        return timed(lambda: vb.vector_probe_residual_mfma(shape, x["k"], x["v"], x["w_cal"], o.eps, repeat), torch, launches) * 1e3
    r_hi = 17
    t_lo, t_hi = probe_ms(1), probe_ms(r_hi)
    iso_tflops = units * 2 * d * d / ((t_hi - t_lo) / (r_hi - 1) * 1e-3) / 1e12
    log(f"residual contraction probe: repeat 1 {t_lo * 1e3:.1f} us, repeat {r_hi} {t_hi * 1e3:.1f} us -> {iso_tflops:.0f} TFLOP/s isolated")
    mfma = {"contraction_kernels_TFLOPs": round(mfma_run, 1) if mfma_run else None, "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
            "frac": round(mfma_run / MFMA_BF16_PEAK_TFLOPS, 4) if mfma_run else None,
            "what": "executed flops of score_stats + mass_residual (both Q K^T passes and K W) over their summed durations",
            "whole_pass_TFLOPs": round(flops_exec * cfg.layers / (ms_per_step * 1e-3) / 1e12, 1),
            "intensity_flop_per_alg_byte": round(intensity, 1),
            "attainable_TFLOPs": round(attainable, 1),
            "attainable_what": "min(bf16 peak, algorithmic flops per algorithmic byte of the pass x 8 TB/s)",
            "frac_of_attainable": round(flops_alg / (pair_us * 1e-6) / 1e12 / attainable, 4) if pair_us else None,
            "matrix_pipe_busy_pct": {"score_stats": profile_value("sq_busy.txt", "score_stats_mfma_busy_pct"),
                                     "mass_residual": profile_value("sq_busy.txt", "mass_residual_mfma_busy_pct"),
                                     "source": "profiles/sq_busy.txt: rocprofv3 --pmc SQ counters of a committed profile run"},
            "residual_contraction_isolated_TFLOPs": round(iso_tflops, 1),
            "residual_contraction_isolated_frac": round(iso_tflops / MFMA_BF16_PEAK_TFLOPS, 4)}

    sweep = None
    if not args.no_sweep:
        sweep = run_sweep(args, vb, dg, pl, torch, np, dev, workers)
        if sweep.get("measured_peaks", {}).get("mfma_loop_TFLOPs") and mfma_run:
            mfma["frac_of_measured_mfma_loop"] = round(mfma_run / sweep["measured_peaks"]["mfma_loop_TFLOPs"], 4)
        cp = sweep.get("measured_peaks", {}).get("device_copy_GBs")
        if cp:
            roofline["frac_of_measured_copy"] = round(dom_gbs / cp, 4)
            roofline["score_residual_pair"]["frac_of_measured_copy"] = round(roofline["score_residual_pair"]["achieved"] / cp, 4)
            roofline["pass_frac_of_measured_copy"] = round(pass_bytes * cfg.layers / (ms_per_step * 1e-3) / 1e9 / cp, 4)
        rd = sweep.get("measured_peaks", {}).get("device_read_GBs")
        if rd:
            roofline["frac_of_measured_read"] = round(dom_gbs / rd, 4)
            roofline["pass_frac_of_measured_read"] = round(pass_bytes * cfg.layers / (ms_per_step * 1e-3) / 1e9 / rd, 4)

    # ---- decode attention over compressed caches ----
    decode = None
    if not args.no_decode:
        decode = run_decode(args, vb, dg, pl, torch, np, dev, workers)

    # ---- CPU oracle on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        cpu = run_cpu_baseline(args, cfg, host_layers, dg, n_p, n_a)

    extras = None
    if args.extras:
        extras = run_extras(vb, dg, pl, torch, np, dev, cfg, shape, layers[0], outs[0], wss[0], n_p, n_a)
        extras.update(run_stacked(vb, pl, torch, dev, cfg, layers, n_p, n_a, n_r))

    line = {
        "metric": "KV tokens compressed/sec (prefill pass)", "value": round(tokens_per_s, 1), "unit": "KV tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg3: {cfg.layers}-layer compression pass, layer by layer, n={n}, Hq/Hkv={cfg.n_q_heads}/{H}, d={d}, "
                               f"window={cfg.window}, pool={cfg.pool_kernel}, retain/approx={n_r}/{n_a} per head",
                   "seed": dg.MASTER_SEED, "streams": max(1, args.streams)},
        "roofline": roofline,
        "kernels": kernels,
        "mfma": mfma,
        "overlapped": overlap,
        "workloads": sweep,
        "decode": decode,
        "cpu_baseline": cpu,
    }
    if extras is not None:
        line["extras"] = extras
    print(json.dumps(line), flush=True)


def run_cpu_baseline(args, cfg, host_layers, dg, n_p, n_a):
    """The oracle as it stands on the host cores: all BLAS threads on most layers, one thread on a few."""
    from oracle import vector_oracle as vo
    try:
        from threadpoolctl import threadpool_info
        n_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        n_threads = 1
    n = cfg.seq_len

    def run(layers_):
        t0 = time.perf_counter()
        for hl in layers_:
            wide = {k: dg.widen(v) for k, v in hl.items()}
            s = vo.score(wide["q_win"], wide["k"], cfg.window, cfg.pool_kernel)
            e = vo.residual(wide["k"], wide["v"], wide["w_cal"])
            _, ir, ia = vo.route(s, e, n_p, n_a)
            vo.compact(hl["k"], hl["v"], ir, ia)
        return time.perf_counter() - t0
    ns = min(args.cpu_sample_layers, cfg.layers)
    dt_all = run(host_layers[:ns])
    n1 = min(8, cfg.layers)
    with blas_threads(1):
        dt_one = run(host_layers[:n1])
    cpu = {"value": round(ns * n / dt_all, 1), "unit": "KV tokens/s", "cores": int(n_threads), "kind": "oracle",
           "sample": f"{ns} of {cfg.layers} layers of the same workload, {dt_all:.1f}s (numpy fp64; BLAS on {n_threads} threads, Python loops single-threaded)",
           "single_thread": {"value": round(n1 * n / dt_one, 1), "unit": "KV tokens/s", "cores": 1,
                             "sample": f"{n1} layers, {dt_one:.1f}s"},
           "host_cpus": os.cpu_count()}
    log(f"cpu oracle: {cpu}")
    return cpu


def run_sweep(args, vb, dg, pl, torch, np, dev, workers):
    """The single-layer workloads (8k tokens, 128k tokens) and two peaks measured in this run."""
    res = {}
    for name, n_sets, iters in (("cfg2", 12, 240), ("cfg4", 1, 20)):
        cfg = dg.CONFIGS[name]
        n_r, n_a, n_p = cfg.counts()
        shape = pl.shape_of(cfg)
        with blas_threads(1), ThreadPoolExecutor(workers) as ex:
            sets = list(ex.map(lambda i: wl.make_layer(cfg, i), range(n_sets)))
        devs = [{k: pl.to_device(getattr(li, k), dev) for k in ("q_win", "k", "v", "w_cal")} for li in sets]
        ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a), dev)
        out = pl.alloc_outputs(shape, n_p, n_a, n_r, torch.bfloat16, dev)
        state = {"i": 0}

        def one():                             # rotate over distinct inputs so that nothing stays cached between calls
            x = devs[state["i"] % n_sets]
            state["i"] += 1
            pl.compress_layer(shape, x["q_win"], x["k"], x["v"], x["w_cal"], n_p, n_a, out, ws, one_call=True)
        for _ in range(n_sets):
            one()
        dt = timed(one, torch, iters)
        vb.vector_timing_enable(True)
        for _ in range(max(n_sets, 4)):
            one()
        torch.cuda.synchronize()
        t = vb.vector_timing_read()
        vb.vector_timing_enable(False)
        alg = compress_bytes_per_token_head(cfg)["algorithmic"]
        pass_bytes = alg["pass"] * cfg.n_kv_heads * cfg.seq_len
        input_mb = n_sets * 2 * cfg.n_kv_heads * cfg.seq_len * cfg.head_dim * 2 / 1e6
        res[name] = {"workload": f"{name}: 1 layer, n={cfg.seq_len}, window={cfg.window}, retain/approx={n_r}/{n_a} per head",
                     "us_per_layer": round(dt * 1e6, 2), "KV_tokens_per_s": round(cfg.seq_len / dt, 1),
                     "pass_alg_bytes": int(pass_bytes), "pass_frac_of_hbm_peak": round(pass_bytes / dt / 1e9 / HBM_PEAK_GBS, 4),
                     "distinct_input_sets": n_sets, "distinct_input_MB": round(input_mb, 1),
                     "note": "inputs rotate over sets larger than the 256 MB Infinity Cache" if n_sets > 1 else "one input set, larger than the 256 MB Infinity Cache",
                     "kernels_us": {k: round(ms / c * 1e3, 2) for k, (ms, c) in t.items() if c}}
        log(f"{name}: {res[name]}")
        del devs, sets, out, ws
        torch.cuda.empty_cache()
    # measured peaks: a plain device-to-device copy (256 MiB read + 256 MiB written), a register-only MFMA loop
    src = torch.empty(128 * 1024 * 1024, dtype=torch.bfloat16, device=dev).normal_()
    dst = torch.empty_like(src)
    dt = timed(lambda: dst.copy_(src), torch, 20)
    copy_gbs = 2 * src.numel() * 2 / dt / 1e9
    del src, dst
    # a buffer that is only read, four times the Infinity Cache
    big = torch.empty(512 * 1024 * 1024, dtype=torch.bfloat16, device=dev).normal_()
    rsink = torch.zeros(1024, dtype=torch.float32, device=dev)
    nread = vb.vector_probe_read_stream(big, rsink)
    dt = timed(lambda: vb.vector_probe_read_stream(big, rsink), torch, 10)
    read_gbs = nread / dt / 1e9
    del big, rsink
    sink = torch.empty(262144, dtype=torch.float32, device=dev)
    iters = 20000
    flops = vb.vector_probe_mfma_loop(sink, iters)
    dt = timed(lambda: vb.vector_probe_mfma_loop(sink, iters), torch, 5)
    res["measured_peaks"] = {"device_copy_GBs": round(copy_gbs, 1), "device_copy_frac_of_hbm_peak": round(copy_gbs / HBM_PEAK_GBS, 4),
                             "device_read_GBs": round(read_gbs, 1), "device_read_frac_of_hbm_peak": round(read_gbs / HBM_PEAK_GBS, 4),
                             "mfma_loop_TFLOPs": round(flops / dt / 1e12, 1),
                             "mfma_loop_frac_of_bf16_peak": round(flops / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                             "what": "256 MiB device-to-device copy (bytes read + written); 1 GiB read-only stream (vector_probe_read_stream); 32x32x16 bf16 MFMA loop on register operands, 16 waves per CU"}
    log(f"measured peaks: {res['measured_peaks']}")
    return res


def run_stacked(vb, pl, torch, dev, cfg, layers, n_p, n_a, n_r):
    """The same 32 layers as one call per entry point: every step of the path is independent per KV
    head, so layers stacked along the head axis ([layers * Hkv, n, d]) are just more heads.  Not the
    benchmark's configuration (which compresses layer by layer); it shows what the kernels sustain
    once their launch ramps are amortised."""
    L, H, Hq = len(layers), cfg.n_kv_heads, cfg.n_q_heads
    stack = {k: torch.cat([x[k] for x in layers], dim=0).contiguous() for k in ("q_win", "k", "v", "w_cal")}
    shape = vb.Shape(n_q_heads=Hq * L, n_kv_heads=H * L, head_dim=cfg.head_dim, seq_len=cfg.seq_len, window=cfg.window,
                     pool_kernel=cfg.pool_kernel, dtype=vb.VECTOR_BF16)
    ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a), dev)
    out = pl.alloc_outputs(shape, n_p, n_a, n_r, torch.bfloat16, dev)
    run = lambda: pl.compress_layer(shape, stack["q_win"], stack["k"], stack["v"], stack["w_cal"], n_p, n_a, out, ws, one_call=True)
    dt = timed(run, torch, 5)
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
        return round(timed(fn, torch, calls) * 1e6, 1)

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
    # the same retained rows read through a block table (blocks of 64 rows in shuffled order)
    blk = 64
    bps = (n_r5 + blk - 1) // blk
    table = torch.randperm(B * H * bps, generator=torch.Generator().manual_seed(3)).to(torch.int32).to(dev)
    k_pool, v_pool = rnd(B * H * bps, blk, d), rnd(B * H * bps, blk, d)
    paged = vb.Cache(batch=B, n_q_heads=c5.n_q_heads, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=n_r5, n_approx=n_a5)
    paged.len_retain, paged.k_ret, paged.v_ret = length.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr()
    paged.k_apx, paged.W = k_apx.data_ptr(), layer["w_cal"].data_ptr()
    paged.ret_block_table, paged.ret_block_rows, paged.ret_blocks_per_seq = table.data_ptr(), blk, bps
    res["decode_attn_paged_us_per_step"] = per_call_us(lambda: vb.vector_decode_attn(paged, q, scale, o5, ws5), 50)
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
    # a batch of equal prompts (8 x 8192 tokens, cfg-2 shape): one call with the heads of the run stacked
    # against one vector_compress call per sequence
    c2 = dg.CONFIGS["cfg2"]
    Bq, n2 = 8, c2.seq_len
    npool2, napx2 = vb.vector_budget_counts_frac(n2, c2.f_retain, c2.f_approx)
    nr2 = npool2 - napx2
    shape2 = pl.shape_of(c2)
    kb, vbt = rnd(H, Bq * n2, d), rnd(H, Bq * n2, d)                    # ragged layout: [Hkv, T, d]
    qb = rnd(Bq, c2.n_q_heads, c2.window, d)
    batch, keep_b = vb.make_batch([n2] * Bq, [npool2] * Bq, [napx2] * Bq, [nr2] * Bq)
    wsb = pl.alloc_workspace(vb.vector_compress_batch_workspace_bytes(shape2, batch), dev)
    ob = dict(score=torch.empty(Bq * H * n2, device=dev), eps=torch.empty(Bq * H * n2, device=dev),
              tier=torch.empty(Bq * H * n2, dtype=torch.uint8, device=dev),
              ir=torch.empty(Bq * H * nr2, dtype=torch.int32, device=dev), ia=torch.empty(Bq * H * napx2, dtype=torch.int32, device=dev),
              kr=torch.empty(Bq * H * nr2, d, dtype=torch.bfloat16, device=dev), vr=torch.empty(Bq * H * nr2, d, dtype=torch.bfloat16, device=dev),
              ka=torch.empty(Bq * H * napx2, d, dtype=torch.bfloat16, device=dev))
    res["compress_batch_8x8192_us"] = per_call_us(
        lambda: vb.vector_compress_batch(shape2, batch, qb, kb, vbt, layer["w_cal"], ob["score"], ob["eps"], ob["tier"], ob["ir"], ob["ia"],
                                         ob["kr"], ob["vr"], ob["ka"], wsb), 10)
    one_b, keep_1 = vb.make_batch([n2], [npool2], [napx2], [nr2])
    # the same sequences one call each: sequence b alone is a batch of one with its own strides
    shape2s = pl.shape_of(c2)
    shape2s.k_stride_head = shape2s.v_stride_head = Bq * n2 * d
    shape2s.k_stride_tok = shape2s.v_stride_tok = d

    def per_sequence():
        for b in range(Bq):
            vb.vector_compress(shape2s, qb[b], kb[:, b * n2:], vbt[:, b * n2:], layer["w_cal"], npool2, napx2,
                               ob["score"][b * H * n2:], ob["eps"][b * H * n2:], ob["tier"][b * H * n2:], ob["ir"][b * H * nr2:],
                               ob["ia"][b * H * napx2:], ob["kr"][b * H * nr2:], ob["vr"][b * H * nr2:], ob["ka"][b * H * napx2:], nr2, wsb)
    res["compress_8x8192_one_call_each_us"] = per_call_us(per_sequence, 10)
    # eight prompts of different lengths in the same buffers (one set of launches over their
    # parameter tables), against one vector_compress call per prompt
    lens = [8192, 3000, 6100, 4096, 7000, 2048, 5000, 7500]
    cnt = [vb.vector_budget_counts_frac(m, c2.f_retain, c2.f_approx) for m in lens]
    np_u, na_u = [c[0] for c in cnt], [c[1] for c in cnt]
    nr_u = [p_ - a_ for p_, a_ in zip(np_u, na_u)]
    ubatch, keep_u = vb.make_batch(lens, np_u, na_u, nr_u)
    wsu = pl.alloc_workspace(vb.vector_compress_batch_workspace_bytes(shape2, ubatch), dev)
    res["compress_batch_8_unequal_us"] = per_call_us(
        lambda: vb.vector_compress_batch(shape2, ubatch, qb, kb, vbt, layer["w_cal"], ob["score"], ob["eps"], ob["tier"], ob["ir"], ob["ia"],
                                         ob["kr"], ob["vr"], ob["ka"], wsu), 10)
    t0s = np.concatenate([[0], np.cumsum(lens)])
    r0s = np.concatenate([[0], np.cumsum(nr_u)])
    a0s = np.concatenate([[0], np.cumsum(na_u)])
    shape_u = pl.shape_of(c2)
    shape_u.k_stride_head = shape_u.v_stride_head = Bq * n2 * d
    shape_u.k_stride_tok = shape_u.v_stride_tok = d

    def per_unequal_sequence():
        for b in range(len(lens)):
            shape_u.seq_len = lens[b]
            t0, r0, a0 = int(t0s[b]), int(r0s[b]), int(a0s[b])
            vb.vector_compress(shape_u, qb[b], kb[:, t0:], vbt[:, t0:], layer["w_cal"], np_u[b], na_u[b],
                               ob["score"][H * t0:], ob["eps"][H * t0:], ob["tier"][H * t0:], ob["ir"][H * r0:],
                               ob["ia"][H * a0:], ob["kr"][H * r0:], ob["vr"][H * r0:], ob["ka"][H * a0:], nr_u[b], wsb)
    res["compress_8_unequal_one_call_each_us"] = per_call_us(per_unequal_sequence, 10)
    res["compress_8_unequal_tokens"] = int(sum(lens))
    del kb, vbt, ob, keep_1, one_b, keep_u, ubatch, wsu
    # The same layer shape with attention rows that are nearly uniform (queries scaled to 0.02, every
    # score within a few per cent of 1/n) plus eight sink and eight anti-sink keys: the selection's
    # radix buckets then have to follow the bulk of the scores, not the keys' leading bits.
    gq = torch.Generator(device=dev).manual_seed(11)
    q_flat = torch.randn(cfg.n_q_heads, cfg.window, d, generator=gq, device=dev) * 0.02
    q_flat[:, :, 0] += 1.0
    k_flat = torch.randn(H, n, d, generator=gq, device=dev)
    at = torch.randperm(n - cfg.window, generator=gq, device=dev)[:16]
    k_flat[:, at] = 0
    k_flat[:, at[:8], 0] = 8.0 * d ** 0.5
    k_flat[:, at[8:], 0] = -8.0 * d ** 0.5
    q_flat, k_flat = q_flat.bfloat16(), k_flat.bfloat16()
    wsc = pl.alloc_workspace(vb.vector_compress_workspace_bytes(shape, n_p, n_a), dev)
    res["compress_flat_heads_us_per_layer"] = per_call_us(
        lambda: pl.compress_layer(shape, q_flat, k_flat, layer["v"], layer["w_cal"], n_p, n_a, out, wsc, one_call=True))
    # the same pass when the prefill's attention kernel hands over the window rows' log-sum-exp
    # (an input here: formed with torch in fp32), so that the first pass over the keys is not run
    G = cfg.n_q_heads // H
    w = cfg.window
    logits = torch.einsum("hgrd,hnd->hgrn", layer["q_win"].float().view(H, G, w, d), layer["k"].float()) / float(np.sqrt(d))
    cols = torch.arange(n, device=dev).view(1, 1, 1, n)
    rows = (n - w + torch.arange(w, device=dev)).view(1, 1, w, 1)
    lse = torch.logsumexp(logits.masked_fill(cols > rows, float("-inf")), dim=-1).reshape(cfg.n_q_heads, w).contiguous()
    del logits
    res["compress_with_lse_us_per_layer"] = per_call_us(
        lambda: vb.vector_compress_lse(shape, layer["q_win"], layer["k"], layer["v"], layer["w_cal"], lse, 0, n_p, n_a, out.score,
                                       out.eps, out.tier, out.idx_retain, out.idx_approx, out.k_ret, out.v_ret, out.k_apx,
                                       out.k_ret.shape[1], wsc))
    res["compress_us_per_layer"] = per_call_us(
        lambda: pl.compress_layer(shape, layer["q_win"], layer["k"], layer["v"], layer["w_cal"], n_p, n_a, out, wsc, one_call=True))
    # the layer read as a post-RoPE cache, without and with that log-sum-exp: what a production prefill calls
    for key, opt in (("compress_rope_us_per_layer", vb.make_options(rope, None, 0)),
                     ("compress_rope_with_lse_us_per_layer", vb.make_options(rope, lse, 0))):
        res[key] = per_call_us(
            lambda: vb.vector_compress_ex(shape, opt, layer["q_win"], layer["k"], layer["v"], layer["w_cal"], n_p, n_a, out.score, out.eps,
                                          out.tier, out.idx_retain, out.idx_approx, out.k_ret, out.v_ret, out.k_apx, out.k_ret.shape[1],
                                          wsc))
    del q_flat, k_flat, wsc, lse
    # Section 5's approximation-ratio sweep re-expressed on the distortion measure of Section 4: at a
    # fixed compression ratio (fixed footprint of 2 (1 - p_c) n rows) budget moves from retained
    # values to pool keys; p_a = 0 is binary eviction with the same memory.  Weights: the layer's
    # un-pooled attention mass from the scorer itself (window columns, which are always kept, weigh 0).
    p_c = 1.0 - cfg.f_retain - cfg.f_approx / 2.0
    mshape = pl.shape_of(cfg)
    mshape.pool_kernel = 1
    mass = torch.empty((H, n), device=dev)
    vb.vector_score(mshape, layer["q_win"], layer["k"], mass, ws)
    mass = torch.where(torch.isinf(mass), torch.zeros_like(mass), mass)
    wsr = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n, n, 1), dev)
    tier = torch.empty((H, n), dtype=torch.uint8, device=dev)
    idx_r = torch.empty((H, n), dtype=torch.int32, device=dev)
    idx_a = torch.empty((H, n), dtype=torch.int32, device=dev)
    sweep = []
    for i in range(0, 9):
        p_a = round((1.0 - p_c) * i / 8.0, 6)                  # 0 .. 1 - p_c: nothing retained at the end
        npool, napx = vb.vector_budget_counts(n, p_c, p_a)
        vb.vector_route(H, n, out.score, out.eps, npool, napx, tier, idx_r if npool > napx else None,
                        idx_a if napx else None, wsr)
        vb.vector_distortion(shape, mass, tier, out.eps, layer["v"], dout, wsd)
        torch.cuda.synchronize()
        rep = dout.cpu().numpy()
        sweep.append({"p_a": p_a, "n_pool": npool, "n_approx": napx, "rows_kept": 2 * npool - napx,
                      "E_mean_over_heads": float(rep[:, 0].mean()), "w_evict": float(rep[:, 1].mean()),
                      "r2_approx": float(rep[:, 4].mean()), "prop1_threshold": float(rep[:, 7].mean())})
    res["pa_sweep"] = {"p_c": round(p_c, 6), "weights": "un-pooled attention mass of the layer (GPU scorer, pool 1)",
                       "points": sweep, "binary_eviction_E": sweep[0]["E_mean_over_heads"],
                       "best_p_a": min(sweep, key=lambda r: r["E_mean_over_heads"])["p_a"]}
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
    ws = pl.alloc_workspace(max(vb.vector_workspace_bytes(shape, n_p, n_a, B), vb.vector_compress_workspace_bytes(shape, n_p, n_a)), dev)
    k_ret = torch.zeros((B, H, cap, d), dtype=torch.bfloat16, device=dev)
    v_ret = torch.zeros((B, H, cap, d), dtype=torch.bfloat16, device=dev)
    k_apx = torch.zeros((B, H, n_a, d), dtype=torch.bfloat16, device=dev)
    t0 = time.time()
    with blas_threads(1), ThreadPoolExecutor(workers) as ex:
        seqs = list(ex.map(lambda b: wl.make_layer(cfg, 0, sub=b), range(B)))
    # the first sequence's map is used for every sequence: W belongs to the layer, not the sequence
    W = pl.to_device(seqs[0].w_cal, dev)
    scratch = pl.alloc_outputs(shape, n_p, n_a, 1, torch.bfloat16, dev)
    for b, li in enumerate(seqs):
        q_win, k, v = (pl.to_device(getattr(li, x), dev) for x in ("q_win", "k", "v"))
        vb.vector_compress(shape, q_win, k, v, W, n_p, n_a, scratch.score, scratch.eps, scratch.tier, scratch.idx_retain,
                           scratch.idx_approx, k_ret[b], v_ret[b], k_apx[b], cap, ws)
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

    k_l, v_l = list(ks.unbind(0)), list(vs.unbind(0))

    def loop():
        length.fill_(n_r)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            # the new token's exact key and value join the retained segment and it attends, in one call
            vb.vector_decode_step(cache, qs[s], k_l[s], v_l[s], scale, out[s], ws)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    loop()                                          # warm-up
    wall = statistics.median([loop() for _ in range(3)])
    # attention alone, back to back: every appended row is in place after the loops above, so
    # step s only needs its own live length (read from a precomputed table, no extra kernel)
    lengths = (torch.arange(steps, dtype=torch.int32, device=dev) + (n_r + 1))[:, None].expand(steps, B).contiguous()
    q_l, out_l, len_l = list(qs.unbind(0)), list(out.unbind(0)), [lengths[s].data_ptr() for s in range(steps)]

    def attn_only(c=cache):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            c.len_retain = len_l[s]
            vb.vector_decode_attn(c, q_l[s], scale, out_l[s], ws)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    attn_only()
    runs = [attn_only() for _ in range(5)]
    attn_us = statistics.median(runs) / steps * 1e6
    vb.vector_timing_enable(True)
    attn_only()
    timing = vb.vector_timing_read()
    vb.vector_timing_enable(False)
    row = d * 2
    mean_appended = (steps + 1) / 2.0
    bytes_step = B * H * (n_p + n_r + 2 * mean_appended) * row + 2 * B * Hq * row
    gbs = bytes_step / (attn_us * 1e-6) / 1e9
    # Reference point at equal footprint: plain binary eviction keeps (n_pool + n_retain) / 2 full
    # key-value pairs per head in the same bytes; the same kernel with nothing approximated.
    n_eq = (n_p + n_r) // 2
    g = torch.Generator(device=dev).manual_seed(11)
    k_eq = torch.randn((B, H, n_eq, d), generator=g, device=dev, dtype=torch.float32).bfloat16()
    v_eq = torch.randn((B, H, n_eq, d), generator=g, device=dev, dtype=torch.float32).bfloat16()
    cache_eq = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=n_eq, n_approx=0)
    len_eq = torch.full((B,), n_eq, dtype=torch.int32, device=dev)
    cache_eq.len_retain, cache_eq.k_ret, cache_eq.v_ret = len_eq.data_ptr(), k_eq.data_ptr(), v_eq.data_ptr()
    cache_eq.k_apx, cache_eq.W = None, W.data_ptr()

    def eq_loop():
        for s in range(steps):
            vb.vector_decode_attn(cache_eq, q_l[s], scale, out_l[s], ws)
    eq_us = statistics.median([timed(eq_loop, torch, 1) for _ in range(3)]) / steps * 1e6
    res = {"workload": f"cfg5: batch {B}, {Hq}/{H} heads, d={d}, {n_r} retained + {n_a} approximated per head of {n}, {steps} steps",
           "attn_us_per_step": round(attn_us, 2), "attn_us_per_step_runs": [round(r / steps * 1e6, 2) for r in runs],
           "alg_bytes_per_step": int(bytes_step), "achieved_GBs": round(gbs, 1),
           "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
           "step_us_with_append": round(wall / steps * 1e6, 2),
           "binary_eviction_equal_footprint": {"full_pairs_per_head": n_eq, "attn_us_per_step": round(eq_us, 2) if eq_us else None,
                                               "note": f"VECTOR attends over {n_p} tokens per head in the bytes of {n_eq} full pairs"},
           "kernels": {k: round(timing[k][0] / max(timing[k][1], 1) * 1e3, 2) for k in ("decode_split", "decode_combine")}}
    log(f"decode: {res}")
    return res


if __name__ == "__main__":
    main()
