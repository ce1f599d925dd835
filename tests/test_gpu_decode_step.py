"""GPU parity of vector_decode_step: decode attention with the step's own token appended.

The oracle has no append of its own: Section 3.2 keeps generated tokens exactly, so a step is
decode attention over the cache with the new (key, value) row placed after the live retained rows.
The test builds that cache on the host for the oracle, and checks the library's output (tolerance
of the decode tests), the rows it stored (bit for bit) and the lengths it advanced."""
import zlib

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
from paper_2605_23258_amd import pipeline as pl
from parity_util import ATOL, RTOL, BF16_HALF_ULP, close

pytestmark = pytest.mark.gpu

CASES = {
    # dtype, d, Hq, Hkv, capacity, live lengths per sequence, approximated rows, flags
    "bf16_d128": ("bf16", 128, 8, 2, 300, (290, 0, 298, 37), 150, 0),
    "bf16_d128_literal": ("bf16", 128, 8, 2, 300, (290, 0, 298, 37), 150, vb.VECTOR_DECODE_LITERAL),
    "bf16_d64_g8": ("bf16", 64, 8, 1, 130, (5, 128), 40, 0),
    "bf16_nothing_approximated": ("bf16", 128, 4, 2, 200, (100, 198), 0, 0),
    "f32_d64": ("f32", 64, 6, 2, 260, (257, 100, 0), 77, 0),
    "f32_d128": ("f32", 128, 2, 2, 90, (10, 88), 33, 0),
}


def _store(dtype):
    return (lambda a: dg.f32_to_bf16_bits(a.astype(np.float32))) if dtype == "bf16" else (lambda a: a.astype(np.float32))


def _oracle_step(q, k_ret, v_ret, length, k_new, v_new, k_apx, W, scale):
    """Decode attention over the cache with (k_new, v_new) as row length[b] of every sequence."""
    B, H, cap, d = k_ret.shape
    kk = np.concatenate([k_ret, np.zeros((B, H, 1, d), k_ret.dtype)], axis=2)
    vv = np.concatenate([v_ret, np.zeros((B, H, 1, d), v_ret.dtype)], axis=2)
    for b in range(B):
        kk[b, :, length[b]] = k_new[b]
        vv[b, :, length[b]] = v_new[b]
    return vo.decode_attn(dg.widen(q), dg.widen(kk), dg.widen(vv), np.asarray(length) + 1, dg.widen(k_apx), dg.widen(W), scale)


@pytest.mark.parametrize("name", list(CASES))
def test_two_steps_with_append(name):
    dtype, d, Hq, H, cap, lens, n_a, flags = CASES[name]
    B = len(lens)
    is_bf = dtype == "bf16"
    store = _store(dtype)
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    k_ret, v_ret = store(rng.standard_normal((B, H, cap, d))), store(rng.standard_normal((B, H, cap, d)))
    k_apx = store(rng.standard_normal((B, H, max(n_a, 1), d)))[:, :, :n_a]
    W = store(rng.standard_normal((H, d, d)) / np.sqrt(d))
    length = np.array(lens, dtype=np.int32)
    for b in range(B):                      # rows beyond the live length must never reach the result
        k_ret[b, :, length[b]:] = store(np.full((1,), 1e30))[0]
        v_ret[b, :, length[b]:] = store(np.full((1,), -1e30))[0]
    scale = 1.0 / np.sqrt(d)
    t = dict(len=pl.to_device(length), k_ret=pl.to_device(k_ret), v_ret=pl.to_device(v_ret),
             k_apx=pl.to_device(np.ascontiguousarray(k_apx)) if n_a else None, W=pl.to_device(W))
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16 if is_bf else vb.VECTOR_F32,
                     cap_retain=cap, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret = t["len"].data_ptr(), t["k_ret"].data_ptr(), t["v_ret"].data_ptr()
    cache.k_apx = t["k_apx"].data_ptr() if n_a else None
    cache.W = t["W"].data_ptr()
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=H, head_dim=d, seq_len=max(cap, 64), window=1, pool_kernel=1, dtype=cache.dtype)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, cap, 0, B) + (1 << 20))
    host_k, host_v, host_len = k_ret.copy(), v_ret.copy(), length.copy()
    for step in range(2):
        q = store(rng.standard_normal((B, Hq, d)))
        k_new, v_new = store(rng.standard_normal((B, H, d))), store(rng.standard_normal((B, H, d)))
        ref = _oracle_step(q, host_k, host_v, host_len, k_new, v_new, k_apx, W, scale)
        out = torch.full((B, Hq, d), 7.0, dtype=torch.float32, device="cuda:0")
        vb.vector_decode_step(cache, pl.to_device(q), pl.to_device(k_new), pl.to_device(v_new), scale, out, ws,
                              flags=flags | vb.VECTOR_DECODE_OUT_F32)
        torch.cuda.synchronize()
        close(out.cpu().numpy(), ref, f"{name} step {step}")
        # the host's picture of the cache after the step
        for b in range(B):
            if host_len[b] < cap:
                host_k[b, :, host_len[b]] = k_new[b]
                host_v[b, :, host_len[b]] = v_new[b]
                host_len[b] += 1
        assert np.array_equal(t["len"].cpu().numpy(), host_len), f"{name} step {step}: lengths"
        got_k, got_v = pl.to_host(t["k_ret"]), pl.to_host(t["v_ret"])
        for b in range(B):                   # live rows bit for bit; rows beyond them untouched
            assert np.array_equal(got_k[b, :, : host_len[b]], host_k[b, :, : host_len[b]]), f"{name} step {step}: k rows"
            assert np.array_equal(got_v[b, :, : host_len[b]], host_v[b, :, : host_len[b]]), f"{name} step {step}: v rows"
            assert np.array_equal(got_k[b, :, host_len[b]:], host_k[b, :, host_len[b]:])
    # afterwards plain decode attention sees the appended rows through the cache alone
    q = store(rng.standard_normal((B, Hq, d)))
    ref = vo.decode_attn(dg.widen(q), dg.widen(host_k), dg.widen(host_v), host_len, dg.widen(k_apx), dg.widen(W), scale)
    out = torch.full((B, Hq, d), 7.0, dtype=torch.float32, device="cuda:0")
    vb.vector_decode_attn(cache, pl.to_device(q), scale, out, ws, flags=flags | vb.VECTOR_DECODE_OUT_F32)
    torch.cuda.synchronize()
    close(out.cpu().numpy(), ref, f"{name} attention after the steps")


def test_full_block_attends_without_storing_and_bf16_output_is_the_rounding():
    d, Hq, H, cap, n_a, B = 128, 4, 1, 64, 20, 2
    store = _store("bf16")
    rng = np.random.default_rng(77)
    k_ret, v_ret = store(rng.standard_normal((B, H, cap, d))), store(rng.standard_normal((B, H, cap, d)))
    k_apx, W = store(rng.standard_normal((B, H, n_a, d))), store(rng.standard_normal((H, d, d)) / np.sqrt(d))
    length = np.array([cap, cap - 1], dtype=np.int32)           # the first block is full
    q, k_new, v_new = store(rng.standard_normal((B, Hq, d))), store(rng.standard_normal((B, H, d))), store(rng.standard_normal((B, H, d)))
    scale = 1.0 / np.sqrt(d)
    ref = _oracle_step(q, k_ret, v_ret, length, k_new, v_new, k_apx, W, scale)
    t = dict(len=pl.to_device(length), k_ret=pl.to_device(k_ret), v_ret=pl.to_device(v_ret), k_apx=pl.to_device(k_apx), W=pl.to_device(W))
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=cap, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret = t["len"].data_ptr(), t["k_ret"].data_ptr(), t["v_ret"].data_ptr()
    cache.k_apx, cache.W = t["k_apx"].data_ptr(), t["W"].data_ptr()
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=H, head_dim=d, seq_len=cap, window=1, pool_kernel=1, dtype=cache.dtype)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, cap, 0, B) + (1 << 20))
    dev = [pl.to_device(x) for x in (q, k_new, v_new)]
    # fp32 output first, on a copy of the lengths so that the bf16 call below starts from the same state
    out32 = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda:0")
    vb.vector_decode_step(cache, *dev, scale, out32, ws, flags=vb.VECTOR_DECODE_OUT_F32)
    torch.cuda.synchronize()
    close(out32.cpu().numpy(), ref, "full block, fp32 out")
    assert t["len"].cpu().numpy().tolist() == [cap, cap]
    got_k = pl.to_host(t["k_ret"])
    assert np.array_equal(got_k[0], k_ret[0]), "a full block must not be written"
    assert np.array_equal(got_k[1, :, cap - 1], k_new[1])
    # same step again with the native output: sequence 1 is full now, so restore its length first
    t["len"].copy_(torch.from_numpy(length))
    out16 = torch.empty((B, Hq, d), dtype=torch.bfloat16, device="cuda:0")
    vb.vector_decode_step(cache, *dev, scale, out16, ws)
    torch.cuda.synchronize()
    bits = pl.to_host(out16)
    assert np.array_equal(bits, dg.f32_to_bf16_bits(out32.cpu().numpy()))
    err = np.abs(dg.widen(bits) - ref)
    assert (err <= ATOL + (RTOL + BF16_HALF_ULP) * np.abs(ref)).all()


def test_step_over_per_sequence_blocks_and_bad_arguments():
    d, Hq, H = 128, 8, 2
    caps, lens, n_as = (70, 200, 33), (69, 150, 0), (30, 64, 10)
    B = len(caps)
    store = _store("bf16")
    rng = np.random.default_rng(5)
    ret0 = np.concatenate([[0], np.cumsum([H * c for c in caps])]).astype(np.int64)
    apx0 = np.concatenate([[0], np.cumsum([H * a for a in n_as])]).astype(np.int64)
    k_ret, v_ret = store(rng.standard_normal((int(ret0[-1]), d))), store(rng.standard_normal((int(ret0[-1]), d)))
    k_apx, W = store(rng.standard_normal((int(apx0[-1]), d))), store(rng.standard_normal((H, d, d)) / np.sqrt(d))
    q, k_new, v_new = store(rng.standard_normal((B, Hq, d))), store(rng.standard_normal((B, H, d))), store(rng.standard_normal((B, H, d)))
    scale = 1.0 / np.sqrt(d)
    ref = np.zeros((B, Hq, d))
    for b in range(B):
        kr = k_ret[ret0[b]: ret0[b + 1]].reshape(1, H, caps[b], d)
        vr = v_ret[ret0[b]: ret0[b + 1]].reshape(1, H, caps[b], d)
        ka = k_apx[apx0[b]: apx0[b + 1]].reshape(1, H, n_as[b], d)
        ref[b] = _oracle_step(q[b: b + 1], kr, vr, np.array([lens[b]]), k_new[b: b + 1], v_new[b: b + 1], ka, W, scale)[0]
    i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device="cuda:0")
    t = dict(len=i32(lens), cap=i32(caps), n_a=i32(n_as), k_ret=pl.to_device(k_ret), v_ret=pl.to_device(v_ret), k_apx=pl.to_device(k_apx),
             W=pl.to_device(W), ret0=torch.from_numpy(ret0[:-1].copy()).cuda(), apx0=torch.from_numpy(apx0[:-1].copy()).cuda())
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16, cap_retain=max(caps), n_approx=max(n_as))
    cache.len_retain, cache.k_ret, cache.v_ret = t["len"].data_ptr(), t["k_ret"].data_ptr(), t["v_ret"].data_ptr()
    cache.k_apx, cache.W = t["k_apx"].data_ptr(), t["W"].data_ptr()
    cache.cap_retain_seq, cache.n_approx_seq = t["cap"].data_ptr(), t["n_a"].data_ptr()
    cache.ret_row_start, cache.apx_row_start = t["ret0"].data_ptr(), t["apx0"].data_ptr()
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=H, head_dim=d, seq_len=max(caps), window=1, pool_kernel=1, dtype=cache.dtype)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, max(caps), 0, B) + (1 << 20))
    dq, dk, dv = (pl.to_device(x) for x in (q, k_new, v_new))
    out = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda:0")
    vb.vector_decode_step(cache, dq, dk, dv, scale, out, ws, flags=vb.VECTOR_DECODE_OUT_F32)
    torch.cuda.synchronize()
    close(out.cpu().numpy(), ref, "per-sequence blocks")
    assert t["len"].cpu().numpy().tolist() == [l + 1 for l in lens]
    got_k = pl.to_host(t["k_ret"])
    for b in range(B):
        for h in range(H):
            assert np.array_equal(got_k[ret0[b] + h * caps[b] + lens[b]], k_new[b, h])
    # a step needs its token and a retained block
    with pytest.raises(vb.VectorError) as ei:
        vb.vector_decode_step(cache, dq, None, dv, scale, out, ws, flags=vb.VECTOR_DECODE_OUT_F32)
    assert ei.value.code == vb.VECTOR_ERR_ARG
    cache.cap_retain = 0
    with pytest.raises(vb.VectorError) as ei:
        vb.vector_decode_step(cache, dq, dk, dv, scale, out, ws, flags=vb.VECTOR_DECODE_OUT_F32)
    assert ei.value.code == vb.VECTOR_ERR_ARG


@pytest.mark.parametrize("dtype,d,block_rows", [("bf16", 128, 64), ("bf16", 64, 16), ("f32", 64, 32)])
def test_paged_retained_segments(dtype, d, block_rows):
    """Retained segments scattered over a pool of blocks: attention and two steps with appends give
    what the oracle gives on the same rows laid out contiguously; new rows land in the right blocks."""
    Hq, H, B, n_a = 8, 2, 3, 50
    blocks_per_seq = 5
    cap = blocks_per_seq * block_rows
    lens = np.array([block_rows * 2 - 1, 0, cap - 2], dtype=np.int32)       # a block boundary, an empty and a nearly full sequence
    is_bf = dtype == "bf16"
    store = _store(dtype)
    rng = np.random.default_rng(zlib.crc32(f"paged {dtype} {d} {block_rows}".encode()))
    k_lin, v_lin = store(rng.standard_normal((B, H, cap, d))), store(rng.standard_normal((B, H, cap, d)))
    k_apx, W = store(rng.standard_normal((B, H, n_a, d))), store(rng.standard_normal((H, d, d)) / np.sqrt(d))
    # a shuffled block table over a pool with some blocks nobody owns
    n_blocks = B * H * blocks_per_seq + 7
    table = rng.permutation(n_blocks)[: B * H * blocks_per_seq].astype(np.int32).reshape(B, H, blocks_per_seq)
    k_pool = store(np.full((n_blocks, block_rows, d), 3e30))
    v_pool = store(np.full((n_blocks, block_rows, d), -3e30))
    for b in range(B):
        for h in range(H):
            for j in range(blocks_per_seq):
                k_pool[table[b, h, j]] = k_lin[b, h, j * block_rows: (j + 1) * block_rows]
                v_pool[table[b, h, j]] = v_lin[b, h, j * block_rows: (j + 1) * block_rows]
    t = dict(len=pl.to_device(lens), k=pl.to_device(k_pool), v=pl.to_device(v_pool), k_apx=pl.to_device(k_apx), W=pl.to_device(W),
             table=pl.to_device(table))
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16 if is_bf else vb.VECTOR_F32,
                     cap_retain=cap, n_approx=n_a)
    cache.len_retain, cache.k_ret, cache.v_ret = t["len"].data_ptr(), t["k"].data_ptr(), t["v"].data_ptr()
    cache.k_apx, cache.W = t["k_apx"].data_ptr(), t["W"].data_ptr()
    cache.ret_block_table, cache.ret_block_rows, cache.ret_blocks_per_seq = t["table"].data_ptr(), block_rows, blocks_per_seq
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=H, head_dim=d, seq_len=max(cap, 64), window=1, pool_kernel=1, dtype=cache.dtype)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, cap, 0, B) + (1 << 20))
    scale = 1.0 / np.sqrt(d)
    host_k, host_v, host_len = k_lin.copy(), v_lin.copy(), lens.copy()
    q = store(rng.standard_normal((B, Hq, d)))
    ref = vo.decode_attn(dg.widen(q), dg.widen(host_k), dg.widen(host_v), host_len, dg.widen(k_apx), dg.widen(W), scale)
    out = torch.full((B, Hq, d), 7.0, dtype=torch.float32, device="cuda:0")
    vb.vector_decode_attn(cache, pl.to_device(q), scale, out, ws, flags=vb.VECTOR_DECODE_OUT_F32)
    torch.cuda.synchronize()
    close(out.cpu().numpy(), ref, "paged attention")
    for step in range(2):
        q = store(rng.standard_normal((B, Hq, d)))
        k_new, v_new = store(rng.standard_normal((B, H, d))), store(rng.standard_normal((B, H, d)))
        ref = _oracle_step(q, host_k, host_v, host_len, k_new, v_new, k_apx, W, scale)
        vb.vector_decode_step(cache, pl.to_device(q), pl.to_device(k_new), pl.to_device(v_new), scale, out, ws,
                              flags=vb.VECTOR_DECODE_OUT_F32)
        torch.cuda.synchronize()
        close(out.cpu().numpy(), ref, f"paged step {step}")
        got_k, got_v = pl.to_host(t["k"]), pl.to_host(t["v"])
        for b in range(B):
            r = int(host_len[b])
            assert r < cap
            for h in range(H):
                blk, off = table[b, h, r // block_rows], r % block_rows
                assert np.array_equal(got_k[blk, off], k_new[b, h]) and np.array_equal(got_v[blk, off], v_new[b, h])
            host_k[b, :, r], host_v[b, :, r] = k_new[b], v_new[b]
            host_len[b] += 1
        assert np.array_equal(t["len"].cpu().numpy(), host_len)
    # blocks nobody owns are untouched
    owned = set(table.reshape(-1).tolist())
    got_k = pl.to_host(t["k"])
    for blk in range(n_blocks):
        if blk not in owned:
            assert np.array_equal(got_k[blk], k_pool[blk])
    # a block table excludes per-sequence arrays, and needs a power-of-two block
    cache.ret_block_rows = 48
    with pytest.raises(vb.VectorError) as ei:
        vb.vector_decode_attn(cache, pl.to_device(q), scale, out, ws, flags=vb.VECTOR_DECODE_OUT_F32)
    assert ei.value.code == vb.VECTOR_ERR_ARG
    cache.ret_block_rows = block_rows
    cache.cap_retain = cap + 1
    with pytest.raises(vb.VectorError) as ei:
        vb.vector_decode_attn(cache, pl.to_device(q), scale, out, ws, flags=vb.VECTOR_DECODE_OUT_F32)
    assert ei.value.code == vb.VECTOR_ERR_ARG


def _random_step_cases():
    rng = np.random.default_rng(4242)
    out = []
    for i in range(18):
        dtype = "bf16" if rng.random() < 0.65 else "f32"
        d = int(rng.choice([64, 128]))
        hkv = int(rng.integers(1, 4))
        g = int(rng.integers(1, 9))
        B = int(rng.integers(1, 5))
        layout = ["uniform", "per_sequence", "paged"][i % 3]
        out.append((i, dtype, d, hkv, g, B, layout))
    return out


@pytest.mark.parametrize("case", _random_step_cases(), ids=lambda c: f"{c[0]}-{c[1]}-d{c[2]}-h{c[3]}g{c[4]}-B{c[5]}-{c[6]}")
def test_random_decode_steps(case):
    """Seeded sweep: three steps with appends over caches of random sizes in each of the three
    layouts of the retained segment (one capacity, per-sequence blocks, paged), every group size."""
    i, dtype, d, H, g, B, layout = case
    Hq = H * g
    is_bf = dtype == "bf16"
    store = _store(dtype)
    rng = np.random.default_rng(9000 + i)
    block_rows = int(rng.choice([16, 32, 64]))
    if layout == "per_sequence":
        caps = [int(rng.integers(4, 400)) for _ in range(B)]
        n_as = [int(rng.integers(0, 300)) for _ in range(B)]
    elif layout == "paged":
        bps = int(rng.integers(1, 7))
        caps = [bps * block_rows] * B
        n_as = [int(rng.integers(0, 300))] * B
    else:
        caps = [int(rng.integers(4, 400))] * B
        n_as = [int(rng.integers(0, 300))] * B
    lens = np.array([int(rng.integers(0, c - 2)) if c > 3 else 0 for c in caps], dtype=np.int32)
    # the oracle's picture: one (k, v, k_apx) set per sequence, contiguous
    ks = [store(rng.standard_normal((H, c, d))) for c in caps]
    vs = [store(rng.standard_normal((H, c, d))) for c in caps]
    kas = [store(rng.standard_normal((H, max(a, 1), d)))[:, :a] for a in n_as]
    W = store(rng.standard_normal((H, d, d)) / np.sqrt(d))
    scale = 1.0 / np.sqrt(d)
    cache = vb.Cache(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, dtype=vb.VECTOR_BF16 if is_bf else vb.VECTOR_F32,
                     cap_retain=max(caps), n_approx=max(n_as))
    keep = {}
    if layout == "paged":
        n_blocks = B * H * bps + 3
        table = rng.permutation(n_blocks)[: B * H * bps].astype(np.int32).reshape(B, H, bps)
        k_pool, v_pool = store(np.zeros((n_blocks, block_rows, d))), store(np.zeros((n_blocks, block_rows, d)))
        for b in range(B):
            for h in range(H):
                for j in range(bps):
                    k_pool[table[b, h, j]] = ks[b][h, j * block_rows: (j + 1) * block_rows]
                    v_pool[table[b, h, j]] = vs[b][h, j * block_rows: (j + 1) * block_rows]
        keep.update(k=pl.to_device(k_pool), v=pl.to_device(v_pool), table=pl.to_device(table),
                    ka=pl.to_device(np.ascontiguousarray(np.stack(kas))) if n_as[0] else None)
        cache.ret_block_table, cache.ret_block_rows, cache.ret_blocks_per_seq = keep["table"].data_ptr(), block_rows, bps
    else:
        keep.update(k=pl.to_device(np.concatenate([x.reshape(-1, d) for x in ks])), v=pl.to_device(np.concatenate([x.reshape(-1, d) for x in vs])),
                    ka=pl.to_device(np.concatenate([x.reshape(-1, d) for x in kas])) if sum(n_as) else None)
        if layout == "per_sequence":
            i32 = lambda x: torch.tensor(list(x), dtype=torch.int32, device="cuda:0")
            i64 = lambda x: torch.tensor(list(x), dtype=torch.int64, device="cuda:0")
            keep.update(cap=i32(caps), na=i32(n_as), r0=i64(np.concatenate([[0], np.cumsum([H * c for c in caps])])[:-1]),
                        a0=i64(np.concatenate([[0], np.cumsum([H * a for a in n_as])])[:-1]))
            cache.cap_retain_seq, cache.n_approx_seq = keep["cap"].data_ptr(), keep["na"].data_ptr()
            cache.ret_row_start, cache.apx_row_start = keep["r0"].data_ptr(), keep["a0"].data_ptr()
    keep["len"], keep["W"] = pl.to_device(lens), pl.to_device(W)
    cache.len_retain, cache.k_ret, cache.v_ret = keep["len"].data_ptr(), keep["k"].data_ptr(), keep["v"].data_ptr()
    cache.k_apx = keep["ka"].data_ptr() if keep["ka"] is not None else None
    cache.W = keep["W"].data_ptr()
    shape = vb.Shape(n_q_heads=Hq, n_kv_heads=H, head_dim=d, seq_len=max(max(caps), 64), window=1, pool_kernel=1, dtype=cache.dtype)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, max(caps), 0, B) + (1 << 20))
    host_len = lens.copy()
    out = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda:0")
    for step in range(3):
        q = store(rng.standard_normal((B, Hq, d)))
        k_new, v_new = store(rng.standard_normal((B, H, d))), store(rng.standard_normal((B, H, d)))
        ref = np.zeros((B, Hq, d))
        for b in range(B):
            ref[b] = _oracle_step(q[b: b + 1], ks[b][None], vs[b][None], np.array([host_len[b]]), k_new[b: b + 1], v_new[b: b + 1],
                                  kas[b][None], W, scale)[0]
        vb.vector_decode_step(cache, pl.to_device(q), pl.to_device(k_new), pl.to_device(v_new), scale, out, ws, flags=vb.VECTOR_DECODE_OUT_F32)
        torch.cuda.synchronize()
        close(out.cpu().numpy(), ref, f"case {i} step {step}")
        for b in range(B):
            if host_len[b] < caps[b]:
                ks[b][:, host_len[b]], vs[b][:, host_len[b]] = k_new[b], v_new[b]
                host_len[b] += 1
        assert np.array_equal(keep["len"].cpu().numpy(), host_len)
