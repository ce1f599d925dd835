"""GPU parity for batches of sequences of unequal length: vector_compress_batch (ragged token axis,
per-sequence counts and capacities) and decode attention over the per-sequence blocks it writes.

Section 3.2 applies to every sequence on its own, so the oracle is called once per sequence and the
batch must reproduce each result: floats within |g - o| <= 1e-3 + 2e-3 |o|, routing and packed rows
bit for bit on the floats the GPU produced, tier differences against the end-to-end oracle only
inside the tolerance band of a threshold."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
from paper_2605_23258_amd import pipeline as pl
import workloads as wl
from parity_util import band_check, close, decode_check

pytestmark = pytest.mark.gpu

BATCHES = {
    # name: (base config, overrides, sequence lengths, spare rows of each retained block)
    "bf16_four_lengths": ("cfg2", dict(n_kv_heads=2, n_q_heads=8, window=32), (700, 2048, 1531, 32), (5, 0, 9, 2)),
    "f32_three_lengths": ("cfg1", dict(n_kv_heads=2, n_q_heads=4, window=20), (1000, 333, 1024), (0, 3, 1)),
    "bf16_one_sequence": ("cfg2", dict(n_kv_heads=1, n_q_heads=4, window=24, pool_kernel=5), (1777,), (4,)),
    "bf16_max_pool": ("cfg2", dict(n_kv_heads=2, n_q_heads=4, window=16, pool_mode="max"), (640, 900), (0, 0)),
    # runs of equal sequences are launched with their heads stacked; a change of capacity alone ends a run
    "bf16_equal_runs": ("cfg2", dict(n_kv_heads=2, n_q_heads=8, window=32), (1024, 1024, 1024, 700, 700, 2048, 2048), (3, 3, 3, 0, 0, 1, 2)),
    "f32_equal_pair": ("cfg1", dict(n_kv_heads=2, n_q_heads=4, window=20), (1000, 1000), (2, 2)),
    # sequences of different lengths go through one set of launches, each with its own parameter block:
    # twenty lengths from one tile to several chunks; equal runs between unequal neighbours; more
    # sequences than one such group takes
    "bf16_twenty_lengths": ("cfg2", dict(n_kv_heads=2, n_q_heads=8, window=32),
                            (40, 5000, 333, 2048, 6100, 64, 1500, 4097, 900, 32, 2500, 777, 4096, 128, 3000, 1025, 450, 5500, 70, 2000),
                            (1, 0, 2, 0, 3, 0, 1, 0, 2, 0, 1, 0, 2, 0, 1, 0, 2, 0, 1, 0)),
    "bf16_runs_between_unequal": ("cfg2", dict(n_kv_heads=2, n_q_heads=8, window=32), (500, 900, 900, 700, 1200, 1200, 1200, 300, 333),
                                  (0, 1, 1, 0, 2, 2, 2, 0, 5)),
    # counts at their limits inside one ragged part: the whole sequence kept, a pool with no retained
    # token, nothing kept at all (that sequence is routed on its own), no approximated token
    "bf16_counts_at_the_limits": ("cfg2", dict(n_kv_heads=2, n_q_heads=8, window=32), (600, 900, 700, 1200, 450), (0, 2, 1, 0, 3),
                                  ((600, 200), (100, 100), (0, 0), (300, 0), (32, 7))),
    "f32_d128_unequal": ("cfg1", dict(head_dim=128, n_kv_heads=1, n_q_heads=2, window=8, pool_kernel=3), (500, 777, 300), (0, 1, 0)),
    "bf16_d64_unequal": ("cfg2", dict(head_dim=64, n_kv_heads=2, n_q_heads=4, window=16), (900, 450, 1300, 2200), (0, 0, 2, 1)),
    "f32_tiny_lengths": ("cfg1", dict(n_kv_heads=1, n_q_heads=2, window=1, pool_kernel=3), (1, 2, 5, 1, 9, 3), (0, 1, 0, 2, 0, 0),
                         ((1, 0), (2, 1), (3, 1), (1, 1), (4, 2), (2, 0))),
    "f32_seventy_short": ("cfg1", dict(n_kv_heads=1, n_q_heads=4, window=20), tuple(64 + 5 * i for i in range(70)), tuple(i % 3 for i in range(70))),
}


class RaggedBatch:
    """Seeded sequences of one layer, concatenated along the token axis, and their per-sequence sizes."""

    def __init__(self, name):
        base, over, lens, spare = BATCHES[name][:4]
        given = BATCHES[name][4] if len(BATCHES[name]) > 4 else None
        self.cfg = dg.scaled(dg.CONFIGS[base], **over)
        self.lens = list(lens)
        self.layers = [wl.make_layer(dg.scaled(self.cfg, seq_len=n), layer=b) for b, n in enumerate(lens)]
        self.W = self.layers[0].w_cal                     # one calibrated map for all sequences
        counts = given or [vo.budget_counts_frac(n, self.cfg.f_retain, self.cfg.f_approx) for n in lens]
        self.n_pool = [c[0] for c in counts]
        self.n_approx = [c[1] for c in counts]
        self.n_retain = [p - a for p, a in zip(self.n_pool, self.n_approx)]
        self.cap = [r + s for r, s in zip(self.n_retain, spare)]
        self.k = np.concatenate([li.k for li in self.layers], axis=1)
        self.v = np.concatenate([li.v for li in self.layers], axis=1)
        self.q_win = np.stack([li.q_win for li in self.layers])
        self.tok0 = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        self.ret0 = np.concatenate([[0], np.cumsum(self.n_retain)]).astype(np.int64)
        self.apx0 = np.concatenate([[0], np.cumsum(self.n_approx)]).astype(np.int64)
        self.cap0 = np.concatenate([[0], np.cumsum(self.cap)]).astype(np.int64)


def _run_batch(rb):
    cfg = rb.cfg
    H, d = cfg.n_kv_heads, cfg.head_dim
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    shape = pl.shape_of(cfg, seq_len=1)                    # seq_len is ignored by the batch call
    batch, keep = vb.make_batch(rb.lens, rb.n_pool, rb.n_approx, rb.cap)
    ws = pl.alloc_workspace(vb.vector_compress_batch_workspace_bytes(shape, batch))
    T, R, A, Cp = int(rb.tok0[-1]), int(rb.ret0[-1]), int(rb.apx0[-1]), int(rb.cap0[-1])
    dev = dict(q=pl.to_device(rb.q_win), k=pl.to_device(rb.k), v=pl.to_device(rb.v), W=pl.to_device(rb.W))
    out = dict(
        score=torch.full((H * T,), -1.0, device="cuda:0"), eps=torch.full((H * T,), -1.0, device="cuda:0"),
        tier=torch.full((H * T,), 9, dtype=torch.uint8, device="cuda:0"),
        idx_r=torch.full((max(H * R, 1),), -1, dtype=torch.int32, device="cuda:0"),
        idx_a=torch.full((max(H * A, 1),), -1, dtype=torch.int32, device="cuda:0"),
        k_ret=torch.zeros((max(H * Cp, 1), d), dtype=tdt, device="cuda:0"),
        v_ret=torch.zeros((max(H * Cp, 1), d), dtype=tdt, device="cuda:0"),
        k_apx=torch.zeros((max(H * A, 1), d), dtype=tdt, device="cuda:0"))
    vb.vector_compress_batch(shape, batch, dev["q"], dev["k"], dev["v"], dev["W"], out["score"], out["eps"], out["tier"],
                             out["idx_r"], out["idx_a"], out["k_ret"], out["v_ret"], out["k_apx"], ws)
    torch.cuda.synchronize()
    del keep
    return shape, dev, out


def _blocks(rb, out, b):
    """Sequence b's blocks of the batch outputs, as host arrays shaped like the one-sequence outputs."""
    H, d, n = rb.cfg.n_kv_heads, rb.cfg.head_dim, rb.lens[b]
    t0, r0, a0, c0 = (int(x[b]) for x in (rb.tok0, rb.ret0, rb.apx0, rb.cap0))
    n_r, n_a, cap = rb.n_retain[b], rb.n_approx[b], rb.cap[b]
    host = lambda t: pl.to_host(t)
    return dict(
        score=out["score"][H * t0: H * (t0 + n)].cpu().numpy().reshape(H, n),
        eps=out["eps"][H * t0: H * (t0 + n)].cpu().numpy().reshape(H, n),
        tier=out["tier"][H * t0: H * (t0 + n)].cpu().numpy().reshape(H, n),
        idx_r=out["idx_r"][H * r0: H * (r0 + n_r)].cpu().numpy().reshape(H, n_r),
        idx_a=out["idx_a"][H * a0: H * (a0 + n_a)].cpu().numpy().reshape(H, n_a),
        k_ret=host(out["k_ret"][H * c0: H * (c0 + cap)]).reshape(H, cap, d),
        v_ret=host(out["v_ret"][H * c0: H * (c0 + cap)]).reshape(H, cap, d),
        k_apx=host(out["k_apx"][H * a0: H * (a0 + n_a)]).reshape(H, n_a, d))


@pytest.mark.parametrize("name", list(BATCHES))
def test_compress_batch_against_the_oracle_sequence_by_sequence(name):
    rb = RaggedBatch(name)
    cfg = rb.cfg
    shape, dev, out = _run_batch(rb)
    w_wide = dg.widen(rb.W)
    for b, li in enumerate(rb.layers):
        n, n_p, n_a, n_r = rb.lens[b], rb.n_pool[b], rb.n_approx[b], rb.n_retain[b]
        got = _blocks(rb, out, b)
        what = f"{name} sequence {b} (n={n})"
        o_score = vo.score(dg.widen(li.q_win), dg.widen(li.k), cfg.window, cfg.pool_kernel, cfg.pool_mode)
        o_eps = vo.residual(dg.widen(li.k), dg.widen(li.v), w_wide)
        assert np.isposinf(got["score"][:, n - cfg.window:]).all(), what
        close(got["score"][:, : n - cfg.window].astype(np.float64) * n, o_score[:, : n - cfg.window].astype(np.float64) * n,
              what + " n*score")
        close(got["eps"], o_eps, what + " eps")
        # integer and byte work: exact on the floats the GPU produced
        tier, idx_r, idx_a = vo.route(got["score"], got["eps"], n_p, n_a)
        assert np.array_equal(got["tier"], tier), what
        assert np.array_equal(got["idx_r"], idx_r) and np.array_equal(got["idx_a"], idx_a), what
        rk, rv, ra = vo.compact(li.k, li.v, idx_r, idx_a)
        assert np.array_equal(got["k_ret"][:, :n_r], rk) and np.array_equal(got["v_ret"][:, :n_r], rv), what
        assert np.array_equal(got["k_apx"], ra), what
        assert not got["k_ret"][:, n_r:].any() and not got["v_ret"][:, n_r:].any(), what + ": spare rows were written"
        # end to end: tiers differ from the oracle's only inside the tolerance band of a threshold
        o_tier, _, _ = vo.route(o_score, o_eps, n_p, n_a)
        flips = band_check(o_score, o_eps, n_p, n_a, tier, o_tier, n, what)
        assert flips <= max(2, 0.004 * tier.size), what


@pytest.mark.parametrize("name", ["bf16_four_lengths", "bf16_equal_runs", "bf16_twenty_lengths", "bf16_runs_between_unequal", "bf16_counts_at_the_limits"])
def test_compress_batch_equals_one_call_per_sequence(name):
    """Bit for bit what vector_compress gives for each sequence alone, also where sequences share
    their launches (equal ones with their heads stacked, unequal ones over parameter tables)."""
    rb = RaggedBatch(name)
    cfg = rb.cfg
    H, d = cfg.n_kv_heads, cfg.head_dim
    shape, dev, out = _run_batch(rb)
    for b, li in enumerate(rb.layers):
        n, n_p, n_a, n_r, cap = rb.lens[b], rb.n_pool[b], rb.n_approx[b], rb.n_retain[b], rb.cap[b]
        s1 = pl.shape_of(cfg, seq_len=n)
        one = pl.alloc_outputs(s1, n_p, n_a, cap, torch.bfloat16)
        ws = pl.alloc_workspace(vb.vector_compress_workspace_bytes(s1, n_p, n_a))
        pl.compress_layer(s1, pl.to_device(li.q_win), pl.to_device(li.k), pl.to_device(li.v), dev["W"], n_p, n_a, one, ws,
                          cap_retain=cap, one_call=True)
        torch.cuda.synchronize()
        got = _blocks(rb, out, b)
        assert np.array_equal(got["score"], one.score.cpu().numpy())
        assert np.array_equal(got["eps"], one.eps.cpu().numpy())
        assert np.array_equal(got["tier"], one.tier.cpu().numpy())
        assert np.array_equal(got["idx_r"], one.idx_retain.cpu().numpy())
        assert np.array_equal(got["idx_a"], one.idx_approx.cpu().numpy())
        assert np.array_equal(got["k_ret"][:, :n_r], pl.to_host(one.k_ret)[:, :n_r])
        assert np.array_equal(got["v_ret"][:, :n_r], pl.to_host(one.v_ret)[:, :n_r])
        assert np.array_equal(got["k_apx"], pl.to_host(one.k_apx)[:, :n_a])


def test_compress_batch_rejects_bad_sizes_before_any_launch():
    rb = RaggedBatch("bf16_max_pool")
    cfg = rb.cfg
    shape = pl.shape_of(cfg, seq_len=1)
    H, d = cfg.n_kv_heads, cfg.head_dim
    dev = dict(q=pl.to_device(rb.q_win), k=pl.to_device(rb.k), v=pl.to_device(rb.v), W=pl.to_device(rb.W))
    T = int(rb.tok0[-1])
    score = torch.full((H * T,), -1.0, device="cuda:0")
    eps = torch.full((H * T,), -1.0, device="cuda:0")
    tier = torch.full((H * T,), 9, dtype=torch.uint8, device="cuda:0")
    idx = torch.zeros((H * T,), dtype=torch.int32, device="cuda:0")
    rows = torch.zeros((H * T, d), dtype=torch.bfloat16, device="cuda:0")
    good, keep = vb.make_batch(rb.lens, rb.n_pool, rb.n_approx, rb.cap)
    ws = pl.alloc_workspace(vb.vector_compress_batch_workspace_bytes(shape, good))

    def code(lens, n_pool, n_approx, cap, w=ws):
        bt, keep2 = vb.make_batch(lens, n_pool, n_approx, cap)
        with pytest.raises(vb.VectorError) as ei:
            vb.vector_compress_batch(shape, bt, dev["q"], dev["k"], dev["v"], dev["W"], score, eps, tier, idx, idx, rows, rows,
                                     rows, w)
        return ei.value.code

    # the second sequence is wrong in each case: nothing of the first may have been written
    assert code([640, 8], rb.n_pool, rb.n_approx, rb.cap) == vb.VECTOR_ERR_SHAPE          # shorter than the window
    assert code(rb.lens, [rb.n_pool[0], 901], rb.n_approx, rb.cap) == vb.VECTOR_ERR_ARG     # pool beyond the sequence
    assert code(rb.lens, rb.n_pool, rb.n_approx, [rb.cap[0], rb.n_retain[1] - 1]) == vb.VECTOR_ERR_ARG
    assert code(rb.lens, rb.n_pool, rb.n_approx, rb.cap, ws[:256]) == vb.VECTOR_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (score == -1.0).all() and (tier == 9).all()
    assert vb.vector_compress_batch_workspace_bytes(shape, vb.make_batch([640, 8], rb.n_pool, rb.n_approx, rb.cap)[0]) == 0


@pytest.mark.parametrize("name,flags", [("bf16_four_lengths", 0), ("bf16_four_lengths", vb.VECTOR_DECODE_LITERAL),
                                        ("f32_three_lengths", 0)])
def test_decode_over_per_sequence_blocks(name, flags):
    """Decode attention straight over the blocks vector_compress_batch wrote (each sequence with its
    own capacities), a few appended rows included, against the oracle sequence by sequence."""
    rb = RaggedBatch(name)
    cfg = rb.cfg
    H, Hq, d, B = cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, len(rb.lens)
    is_bf = cfg.dtype == "bf16"
    shape, dev, out = _run_batch(rb)
    rng = np.random.default_rng(1234)
    store = (lambda a: dg.f32_to_bf16_bits(a.astype(np.float32))) if is_bf else (lambda a: a.astype(np.float32))
    # append rows (exact key and value) to the sequences that have spare capacity
    k_ret, v_ret = pl.to_host(out["k_ret"]).copy(), pl.to_host(out["v_ret"]).copy()
    live = []
    for b in range(B):
        extra = min(rb.cap[b] - rb.n_retain[b], 3)
        live.append(rb.n_retain[b] + extra)
        for h in range(H):
            row0 = H * int(rb.cap0[b]) + h * rb.cap[b] + rb.n_retain[b]
            k_ret[row0: row0 + extra] = store(rng.standard_normal((extra, d)))
            v_ret[row0: row0 + extra] = store(rng.standard_normal((extra, d)))
    q = store(rng.standard_normal((B, Hq, d)))
    scale = 1.0 / np.sqrt(d)
    # the oracle, one sequence at a time, on host copies of the blocks
    ref = np.zeros((B, Hq, d))
    k_apx = pl.to_host(out["k_apx"])
    for b in range(B):
        c0, a0, cap, n_a = H * int(rb.cap0[b]), H * int(rb.apx0[b]), rb.cap[b], rb.n_approx[b]
        kr = dg.widen(k_ret[c0: c0 + H * cap].reshape(1, H, cap, d))
        vr = dg.widen(v_ret[c0: c0 + H * cap].reshape(1, H, cap, d))
        ka = dg.widen(k_apx[a0: a0 + H * n_a].reshape(1, H, n_a, d))
        ref[b] = vo.decode_attn(dg.widen(q[b: b + 1]), kr, vr, np.array([live[b]]), ka, dg.widen(rb.W), scale)[0]
    t = dict(k_ret=pl.to_device(k_ret), v_ret=pl.to_device(v_ret), q=pl.to_device(q),
             len=torch.tensor(live, dtype=torch.int32, device="cuda:0"),
             cap=torch.tensor(rb.cap, dtype=torch.int32, device="cuda:0"),
             n_a=torch.tensor(rb.n_approx, dtype=torch.int32, device="cuda:0"),
             ret0=torch.tensor([H * int(x) for x in rb.cap0[:-1]], dtype=torch.int64, device="cuda:0"),
             apx0=torch.tensor([H * int(x) for x in rb.apx0[:-1]], dtype=torch.int64, device="cuda:0"))
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16 if is_bf else vb.VECTOR_F32,
                     cap_retain=max(rb.cap), n_approx=max(rb.n_approx))
    cache.len_retain, cache.k_ret, cache.v_ret = t["len"].data_ptr(), t["k_ret"].data_ptr(), t["v_ret"].data_ptr()
    cache.k_apx, cache.W = out["k_apx"].data_ptr(), dev["W"].data_ptr()
    cache.cap_retain_seq, cache.n_approx_seq = t["cap"].data_ptr(), t["n_a"].data_ptr()
    cache.ret_row_start, cache.apx_row_start = t["ret0"].data_ptr(), t["apx0"].data_ptr()
    dshape = vb.Shape(n_q_heads=Hq, n_kv_heads=H, head_dim=d, seq_len=max(max(rb.cap), 64), window=1, pool_kernel=1,
                      dtype=cache.dtype)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(dshape, max(rb.cap), 0, B) + (1 << 20))
    decode_check(cache, t["q"], scale, ws, ref, f"{name} decode", flags=flags)
    # three of the four arrays: refused
    cache.apx_row_start = None
    with pytest.raises(vb.VectorError) as ei:
        vb.vector_decode_attn(cache, t["q"], scale, torch.empty((B, Hq, d), dtype=torch.float32, device="cuda:0"), ws,
                              flags=vb.VECTOR_DECODE_OUT_F32)
    assert ei.value.code == vb.VECTOR_ERR_ARG


@pytest.mark.parametrize("explicit", [False, True], ids=["row_index_positions", "position_array"])
def test_compress_batch_on_rotated_keys(explicit):
    """The batch call on post-RoPE keys: unequal sequences around a run of equal ones, positions
    either implied (row index plus one offset for all) or given as an array ragged like the keys
    (every sequence with an offset of its own).  Bit for bit vector_compress_rope per sequence,
    and the residual is the oracle's with the keys turned back."""
    theta = 500000.0
    cfg = dg.scaled(dg.CONFIGS["cfg2"], n_kv_heads=2, n_q_heads=8, window=32)
    lens = [700, 1200, 1200, 333, 2100]
    offsets = [11 + 1000 * b for b in range(len(lens))] if explicit else [40] * len(lens)
    H, d = cfg.n_kv_heads, cfg.head_dim
    layers = [wl.make_layer(dg.scaled(cfg, seq_len=n), layer=b, rope_theta=theta, rope_interleaved=False, pos_offset=offsets[b])
              for b, n in enumerate(lens)]
    inv_freq = layers[0].extra["inv_freq"]
    W = layers[0].w_cal
    counts = [vo.budget_counts_frac(n, cfg.f_retain, cfg.f_approx) for n in lens]
    n_pool, n_approx = [c[0] for c in counts], [c[1] for c in counts]
    n_ret = [p - a for p, a in zip(n_pool, n_approx)]
    tok0 = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ret0 = np.concatenate([[0], np.cumsum(n_ret)]).astype(np.int64)
    apx0 = np.concatenate([[0], np.cumsum(n_approx)]).astype(np.int64)
    T, R, A = int(tok0[-1]), int(ret0[-1]), int(apx0[-1])
    dev = dict(q=pl.to_device(np.stack([li.q_win for li in layers])), k=pl.to_device(np.concatenate([li.k for li in layers], axis=1)),
               v=pl.to_device(np.concatenate([li.v for li in layers], axis=1)), W=pl.to_device(W))
    pos_all = pl.to_device(np.concatenate([li.extra["pos"] for li in layers]).astype(np.int32)) if explicit else None
    rope, keep_r = vb.make_rope(inv_freq, pos_all, False, 0 if explicit else offsets[0])
    shape = pl.shape_of(cfg, seq_len=1)
    batch, keep = vb.make_batch(lens, n_pool, n_approx, n_ret)
    ws = pl.alloc_workspace(vb.vector_compress_batch_workspace_bytes(shape, batch))
    out = dict(score=torch.full((H * T,), -1.0, device="cuda:0"), eps=torch.full((H * T,), -1.0, device="cuda:0"),
               tier=torch.full((H * T,), 9, dtype=torch.uint8, device="cuda:0"),
               ir=torch.full((H * R,), -1, dtype=torch.int32, device="cuda:0"), ia=torch.full((H * A,), -1, dtype=torch.int32, device="cuda:0"),
               kr=torch.zeros((H * R, d), dtype=torch.bfloat16, device="cuda:0"), vr=torch.zeros((H * R, d), dtype=torch.bfloat16, device="cuda:0"),
               ka=torch.zeros((H * A, d), dtype=torch.bfloat16, device="cuda:0"))
    vb.vector_compress_batch_rope(shape, batch, rope, dev["q"], dev["k"], dev["v"], dev["W"], out["score"], out["eps"], out["tier"],
                                  out["ir"], out["ia"], out["kr"], out["vr"], out["ka"], ws)
    torch.cuda.synchronize()
    w_wide = dg.widen(W)
    for b, li in enumerate(layers):
        n, n_p, n_a, n_r = lens[b], n_pool[b], n_approx[b], n_ret[b]
        t0, r0, a0 = int(tok0[b]), int(ret0[b]), int(apx0[b])
        s1 = pl.shape_of(cfg, seq_len=n)
        one = pl.alloc_outputs(s1, n_p, n_a, n_r, torch.bfloat16)
        ws1 = pl.alloc_workspace(vb.vector_compress_workspace_bytes(s1, n_p, n_a))
        pos_b = pl.to_device(li.extra["pos"].astype(np.int32)) if explicit else None
        rope1, keep1 = vb.make_rope(inv_freq, pos_b, False, 0 if explicit else offsets[b])
        vb.vector_compress_rope(s1, rope1, pl.to_device(li.q_win), pl.to_device(li.k), pl.to_device(li.v), dev["W"], n_p, n_a, one.score,
                                one.eps, one.tier, one.idx_retain, one.idx_approx, one.k_ret, one.v_ret, one.k_apx, n_r, ws1)
        torch.cuda.synchronize()
        what = f"sequence {b}"
        assert torch.equal(out["score"][H * t0: H * (t0 + n)].view(H, n), one.score), what
        assert torch.equal(out["eps"][H * t0: H * (t0 + n)].view(H, n), one.eps), what
        assert torch.equal(out["tier"][H * t0: H * (t0 + n)].view(H, n), one.tier), what
        assert torch.equal(out["ir"][H * r0: H * (r0 + n_r)].view(H, n_r), one.idx_retain), what
        assert torch.equal(out["ia"][H * a0: H * (a0 + n_a)].view(H, n_a), one.idx_approx), what
        assert torch.equal(out["kr"][H * r0: H * (r0 + n_r)].view(torch.int16), one.k_ret.view(torch.int16).reshape(H * n_r, d)), what
        assert torch.equal(out["ka"][H * a0: H * (a0 + n_a)].view(torch.int16), one.k_apx.view(torch.int16).reshape(H * n_a, d)), what
        ref_eps = vo.residual(dg.widen(li.k), dg.widen(li.v), w_wide, pos=li.extra["pos"], inv_freq=inv_freq, interleaved=False)
        close(one.eps.cpu().numpy(), ref_eps, what + " eps")
    del keep, keep_r
