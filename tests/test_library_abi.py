"""The C-ABI library loads and exports every symbol include/vector.h declares;
host-only helpers agree with the oracle.  No GPU needed."""
import os
import re

import pytest

from oracle import vector_oracle as vo
from paper_2605_23258_amd import binding as vb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "vector.h")).read()
    return sorted(set(re.findall(r"VECTOR_API\s+[\w\s\*]+?\b(vector_\w+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared()
    assert len(names) >= 11 and set(names) == set(vb.EXPORTS)
    L = vb.lib()
    for name in names:
        assert hasattr(L, name), name


def test_struct_sizes_match_header_layout():
    import ctypes
    assert ctypes.sizeof(vb.Shape) == 8 * 4 + 5 * 8 + 2 * 4
    assert ctypes.sizeof(vb.Cache) == 8 * 4 + 5 * 8 + 4 * 8 + 8 + 2 * 4
    assert ctypes.sizeof(vb.Batch) == 8 + 4 * 8
    assert ctypes.sizeof(vb.CompressOptions) == 3 * 8


def test_budget_helpers_match_oracle():
    for n in (1024, 8192, 32768, 131072, 999):
        for fr, fa in ((0.25, 0.25), (0.15, 0.15), (0.10, 0.10), (0.05, 0.05), (0.0, 0.3), (1.0, 0.0)):
            assert vb.vector_budget_counts_frac(n, fr, fa) == vo.budget_counts_frac(n, fr, fa)
        for p_c in (0.25, 0.5, 0.75, 0.9):
            p_a = vb.vector_pa_deploy(p_c, 0.0)
            assert p_a == pytest.approx(vo.pa_deploy(p_c))
            assert vb.vector_budget_counts(n, p_c, p_a) == vo.budget_counts(n, p_c, p_a)


def test_budget_counts_hand_values():
    """The library against hand-computed counts, not against the oracle: Section 5's p_c = 0.9,
    p_a = 0.05 keeps 5 % of the tokens and approximates 10 %."""
    assert vb.vector_budget_counts(1000, 0.9, 0.05) == (150, 100)
    assert vb.vector_budget_counts(30000, 0.9, 0.05) == (4500, 3000)
    assert vb.vector_budget_counts(1000, 0.8, 0.1) == (300, 200)
    assert vb.vector_budget_counts(1001, 0.9, 0.05) == (150, 100)
    assert vb.vector_budget_counts_frac(10, 0.29, 0.0) == (2, 0)


def test_bad_arguments_are_rejected_on_the_host():
    with pytest.raises(vb.VectorError):
        vb.vector_budget_counts_frac(100, 0.8, 0.5)
    with pytest.raises(vb.VectorError):
        vb.vector_budget_counts(100, 0.5, 0.6)
    s = vb.Shape(n_q_heads=4, n_kv_heads=1, head_dim=96, seq_len=64, window=8, pool_kernel=7, dtype=0)
    assert vb.vector_workspace_bytes(s, 10, 5, 1) == 0          # unsupported head_dim
    s.head_dim = 64
    assert vb.vector_workspace_bytes(s, 10, 5, 1) > 0
    # null pointers / bad counts never reach a launch
    L = vb.lib()
    import ctypes as C
    assert L.vector_score(C.byref(s), None, None, None, None, 0, None) == -1
    assert L.vector_route(1, 64, None, None, 10, 20, None, None, None, None, 0, None) == -1
    s.pool_kernel = 4
    assert L.vector_score(C.byref(s), None, None, None, None, 0, None) == -2
    assert vb.strerror(-3).startswith("workspace")


def test_batch_workspace_follows_how_the_sequences_share_launches():
    """Host-side planning of a batch: a run of equal sequences needs what one call on the stacked
    heads needs; unequal neighbours run together, each in its own piece of the workspace after
    their parameter tables; the batch needs the largest part."""
    s = vb.Shape(n_q_heads=8, n_kv_heads=2, head_dim=128, seq_len=1, window=32, pool_kernel=7, dtype=vb.VECTOR_BF16)

    def one(n, heads_times=1):
        t = vb.Shape(n_q_heads=8 * heads_times, n_kv_heads=2 * heads_times, head_dim=128, seq_len=n, window=32, pool_kernel=7,
                     dtype=vb.VECTOR_BF16)
        n_p, n_a = vb.vector_budget_counts_frac(n, 0.15, 0.15)
        return vb.vector_compress_workspace_bytes(t, n_p, n_a)

    def batch_bytes(lens):
        counts = [vb.vector_budget_counts_frac(n, 0.15, 0.15) for n in lens]
        b, keep = vb.make_batch(lens, [c[0] for c in counts], [c[1] for c in counts], [c[0] - c[1] for c in counts])
        return vb.vector_compress_batch_workspace_bytes(s, b)

    assert batch_bytes([4096]) == one(4096)
    assert batch_bytes([4096, 4096, 4096]) == one(4096, 3)
    ragged = batch_bytes([4096, 1000, 2500])
    pieces = sum((one(n) + 255) // 256 * 256 for n in (4096, 1000, 2500))
    assert pieces < ragged <= pieces + 65536                   # the tables are a few hundred bytes per sequence and kernel
    assert batch_bytes([700, 4096, 4096, 4096, 900]) == one(4096, 3)      # singles around a run: the run is the largest part
    assert batch_bytes([4096, 1000, 2500, 8192, 8192]) == max(ragged, one(8192, 2))


def test_batch_and_option_arguments_are_rejected_on_the_host():
    import ctypes as C
    L = vb.lib()
    s = vb.Shape(n_q_heads=8, n_kv_heads=2, head_dim=128, seq_len=1, window=32, pool_kernel=7, dtype=vb.VECTOR_BF16)
    good, keep = vb.make_batch([100, 200], [30, 60], [10, 20], [20, 40])
    assert vb.vector_compress_batch_workspace_bytes(s, good) > 0
    for lens, pool, apx, cap in (([100, 20], [30, 6], [10, 2], [20, 4]),          # shorter than the window
                                 ([100, 200], [30, 260], [10, 20], [20, 240]),     # pool larger than the sequence
                                 ([100, 200], [30, 60], [40, 20], [20, 40]),       # more approximated than pooled
                                 ([100, 200], [30, 60], [10, 20], [19, 40])):      # capacity below the retained count
        bad, keep_b = vb.make_batch(lens, pool, apx, cap)
        assert vb.vector_compress_batch_workspace_bytes(s, bad) == 0
        assert L.vector_compress_batch(C.byref(s), C.byref(bad), *([None] * 13), 0, None) < 0
    # null tensors with a valid batch; a null shape; a stride for a log-sum-exp that is not there
    assert L.vector_compress_batch(C.byref(s), C.byref(good), *([None] * 13), 0, None) == -1
    assert L.vector_compress_ex(None, None, *([None] * 4), 1, 0, *([None] * 8), 0, None, 0, None) == -1
    opt = vb.CompressOptions()
    opt.rope, opt.lse, opt.lse_stride_head = None, None, 64
    assert L.vector_compress_batch_ex(C.byref(s), C.byref(good), C.byref(opt), *([None] * 13), 0, None) == -1


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more ends with a message and a non-zero status
    before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
