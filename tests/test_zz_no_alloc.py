"""The allocation-free routing entry point (vector_route_static) against vector_route: same
tiers and index lists, bit for bit, on two calls in a row through the C ABI, the second on a
smaller input (the library's scratch array keeps the first call's contents)."""
import ctypes as C

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import pipeline as pl

pytestmark = pytest.mark.gpu


def _route_both(H, n, n_pool, n_approx, seed):
    rng = np.random.default_rng(seed)
    score = np.exp(rng.standard_normal((H, n))).astype(np.float32) / n
    score[:, n - 8:] = np.inf
    at = np.arange(0, n - 16, 97)
    score[:, at] = score[:, at + 5]                  # some exact ties
    eps = (rng.random((H, n)) ** 4).astype(np.float32)
    d_score, d_eps = pl.to_device(score), pl.to_device(eps)
    n_r = n_pool - n_approx

    def outputs():
        return (torch.full((H, n), 77, dtype=torch.uint8, device="cuda:0"),
                torch.full((H, max(n_r, 1)), -1, dtype=torch.int32, device="cuda:0"),
                torch.full((H, max(n_approx, 1)), -1, dtype=torch.int32, device="cuda:0"))
    ref = outputs()
    shape = vb.Shape(n_q_heads=H, n_kv_heads=H, head_dim=64, seq_len=n, window=1, pool_kernel=1, dtype=0)
    ws = pl.alloc_workspace(vb.vector_workspace_bytes(shape, n_pool, n_approx, 1))
    vb.vector_route(H, n, d_score, d_eps, n_pool, n_approx, ref[0], ref[1], ref[2], ws)
    got = outputs()
    stream = torch.cuda.current_stream().cuda_stream
    rc = vb.lib().vector_route_static(H, n, C.c_void_p(d_score.data_ptr()), C.c_void_p(d_eps.data_ptr()), n_pool, n_approx,
                                      C.c_void_p(got[0].data_ptr()), C.c_void_p(got[1].data_ptr()), C.c_void_p(got[2].data_ptr()),
                                      C.c_void_p(stream) if stream else None)
    assert rc == vb.VECTOR_OK, vb.strerror(rc)
    torch.cuda.synchronize()
    for g, r, what in zip(got, ref, ("tier", "idx_retain", "idx_approx")):
        assert torch.equal(g, r), f"{what} differs (n={n}, n_pool={n_pool}, n_approx={n_approx})"
    assert (ref[0] == vb.TIER_RETAIN).sum().item() == H * n_r and (ref[0] == vb.TIER_APPROX).sum().item() == H * n_approx


def test_static_scratch_matches_workspace_variant_twice():
    _route_both(8, 32768, 6552, 3276, seed=1)       # a benchmark-sized layer first
    _route_both(3, 5001, 1234, 600, seed=2)         # then a smaller, ragged one on the same scratch
    _route_both(2, 70000, 9000, 0, seed=3)          # nothing approximated: the split step only copies


def test_static_scratch_rejects_what_does_not_fit():
    L = vb.lib()
    assert L.vector_route_static_scratch_bytes() == 16 << 20
    H, n = 64, 1 << 20                                # needs far more than the array holds
    x = torch.zeros(16, device="cuda:0")
    rc = L.vector_route_static(H, n, C.c_void_p(x.data_ptr()), C.c_void_p(x.data_ptr()), 10, 5, C.c_void_p(x.data_ptr()),
                               C.c_void_p(x.data_ptr()), C.c_void_p(x.data_ptr()), None)
    assert rc == vb.VECTOR_ERR_WORKSPACE
    assert L.vector_route_static(1, 64, None, None, 10, 20, None, None, None, None) == vb.VECTOR_ERR_ARG
