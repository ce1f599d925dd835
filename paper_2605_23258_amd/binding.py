"""ctypes binding of libvector.so: the same entry points as include/vector.h.

Argument marshalling only -- every step of the path runs in the HIP kernels.
Tensors are torch tensors used as device memory; the stream defaults to torch's
current stream.  A missing library is an error: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libvector.so")

VECTOR_F32, VECTOR_BF16 = 0, 1
VECTOR_POOL_AVG, VECTOR_POOL_MAX = 0, 1
VECTOR_DECODE_LITERAL = 1
VECTOR_DECODE_OUT_F32 = 2
VECTOR_OK, VECTOR_ERR_ARG, VECTOR_ERR_SHAPE, VECTOR_ERR_WORKSPACE, VECTOR_ERR_DTYPE, VECTOR_ERR_HIP = 0, -1, -2, -3, -4, -5
TIER_EVICT, TIER_APPROX, TIER_RETAIN = 0, 1, 2

EXPORTS = (
    "vector_budget_counts", "vector_budget_counts_frac", "vector_pa_deploy", "vector_workspace_bytes",
    "vector_strerror", "vector_score", "vector_residual", "vector_score_residual", "vector_route",
    "vector_route_static", "vector_route_static_scratch_bytes", "vector_compact", "vector_decode_attn", "vector_compress_workspace_bytes", "vector_compress",
    "vector_compress_batch_workspace_bytes", "vector_compress_batch",
    "vector_score_residual_lse", "vector_compress_lse", "vector_compress_rope", "vector_compress_batch_rope",
    "vector_compress_ex", "vector_compress_batch_ex",
    "vector_timing_enable", "vector_timing_kernels", "vector_timing_name", "vector_timing_read",
    "vector_probe_residual_mfma", "vector_probe_mfma_loop", "vector_probe_read_stream",
    "vector_residual_rope", "vector_score_residual_rope", "vector_decode_attn_rope",
    "vector_decode_step", "vector_decode_step_rope",
    "vector_calibrate_workspace_bytes", "vector_calibrate",
    "vector_distortion_workspace_bytes", "vector_distortion",
    "vector_r2_workspace_bytes", "vector_r2",
    "vector_score_key_diversity_workspace_bytes", "vector_score_key_diversity",
)


class VectorError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class Shape(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("seq_len", C.c_int32),
        ("window", C.c_int32), ("pool_kernel", C.c_int32), ("dtype", C.c_int32), ("pool_mode", C.c_int32),
        ("k_stride_head", C.c_int64), ("k_stride_tok", C.c_int64),
        ("v_stride_head", C.c_int64), ("v_stride_tok", C.c_int64),
        ("w_stride_head", C.c_int64), ("w_shared", C.c_int32), ("reserved2", C.c_int32),
    ]


class Rope(C.Structure):
    """vector_rope: inv_freq is HOST memory (keep the array it points into alive during the call)."""
    _fields_ = [("inv_freq", C.POINTER(C.c_double)), ("interleaved", C.c_int32), ("pos_offset", C.c_int32),
                ("positions", C.c_void_p)]


class CompressOptions(C.Structure):
    """vector_compress_options: any of a rotary description and the window rows' log-sum-exp."""
    _fields_ = [("rope", C.POINTER(Rope)), ("lse", C.c_void_p), ("lse_stride_head", C.c_int64)]



def make_rope(inv_freq, positions=None, interleaved: bool = False, pos_offset: int = 0):
    """(Rope, keep-alive) from a float64 host array of head_dim/2 frequencies and an optional
    device int32 tensor of positions."""
    import numpy as np
    arr = np.ascontiguousarray(inv_freq, dtype=np.float64)
    r = Rope(inv_freq=arr.ctypes.data_as(C.POINTER(C.c_double)), interleaved=int(bool(interleaved)),
             pos_offset=int(pos_offset), positions=_ptr(positions))
    return r, (arr, positions)


class Cache(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("dtype", C.c_int32), ("cap_retain", C.c_int32), ("n_approx", C.c_int32), ("w_shared", C.c_int32),
        ("len_retain", C.c_void_p), ("k_ret", C.c_void_p), ("v_ret", C.c_void_p), ("k_apx", C.c_void_p),
        ("W", C.c_void_p),
        ("cap_retain_seq", C.c_void_p), ("n_approx_seq", C.c_void_p), ("ret_row_start", C.c_void_p),
        ("apx_row_start", C.c_void_p),
        ("ret_block_table", C.c_void_p), ("ret_block_rows", C.c_int32), ("ret_blocks_per_seq", C.c_int32),
    ]


class Batch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("seq_len", C.POINTER(C.c_int32)), ("n_pool", C.POINTER(C.c_int32)),
                ("n_approx", C.POINTER(C.c_int32)), ("cap_retain", C.POINTER(C.c_int32))]


def make_batch(seq_len, n_pool, n_approx, cap_retain):
    """(Batch, keep-alive) from four host sequences of equal length."""
    arrs = [(C.c_int32 * len(seq_len))(*[int(x) for x in a]) for a in (seq_len, n_pool, n_approx, cap_retain)]
    assert len({len(a) for a in arrs}) == 1
    return Batch(len(seq_len), *[C.cast(a, C.POINTER(C.c_int32)) for a in arrs]), arrs


_lib = None


def lib() -> C.CDLL:
    """Load libvector.so (built by paper_2605_23258_amd.build); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2605_23258_amd.build` "
                "(there is no CPU fallback for the hot path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.vector_budget_counts.argtypes = [i32, C.c_double, C.c_double, C.POINTER(i32), C.POINTER(i32)]
        L.vector_budget_counts_frac.argtypes = [i32, C.c_double, C.c_double, C.POINTER(i32), C.POINTER(i32)]
        L.vector_pa_deploy.argtypes = [C.c_double, C.c_double]
        L.vector_pa_deploy.restype = C.c_double
        L.vector_workspace_bytes.argtypes = [C.POINTER(Shape), i32, i32, i32]
        L.vector_workspace_bytes.restype = sz
        L.vector_strerror.argtypes = [C.c_int]
        L.vector_strerror.restype = C.c_char_p
        L.vector_score.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, sz, vp]
        L.vector_residual.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, vp, sz, vp]
        L.vector_score_residual.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vector_route.argtypes = [i32, i32, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
        L.vector_compress_ex.argtypes = [C.POINTER(Shape), C.POINTER(CompressOptions), vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp,
                                         vp, vp, i32, vp, sz, vp]
        L.vector_compress_batch_ex.argtypes = [C.POINTER(Shape), C.POINTER(Batch), C.POINTER(CompressOptions), vp, vp, vp, vp, vp, vp,
                                               vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vector_compress_batch_rope.argtypes = [C.POINTER(Shape), C.POINTER(Batch), C.POINTER(Rope), vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                 vp, vp, vp, vp, sz, vp]
        L.vector_compress_rope.argtypes = [C.POINTER(Shape), C.POINTER(Rope), vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp,
                                           i32, vp, sz, vp]
        L.vector_score_residual_lse.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, vp, C.c_int64, vp, vp, vp, sz, vp]
        L.vector_compress_lse.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, vp, C.c_int64, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp,
                                          i32, vp, sz, vp]
        L.vector_route_static.argtypes = [i32, i32, vp, vp, i32, i32, vp, vp, vp, vp]
        L.vector_route_static_scratch_bytes.argtypes = []
        L.vector_route_static_scratch_bytes.restype = sz
        L.vector_compact.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, i32, i32, vp, vp, vp, i32, vp]
        L.vector_decode_attn.argtypes = [C.POINTER(Cache), vp, C.c_float, vp, i32, vp, sz, vp]
        L.vector_decode_step.argtypes = [C.POINTER(Cache), vp, vp, vp, C.c_float, vp, i32, vp, sz, vp]
        L.vector_decode_step_rope.argtypes = [C.POINTER(Cache), C.POINTER(Rope), vp, vp, vp, C.c_float, vp, i32, vp, sz, vp]
        L.vector_timing_enable.argtypes = [C.c_int]
        L.vector_timing_name.argtypes = [C.c_int]
        L.vector_timing_name.restype = C.c_char_p
        L.vector_timing_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.vector_probe_residual_mfma.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, i32, vp]
        L.vector_probe_mfma_loop.argtypes = [vp, i32, C.POINTER(C.c_int64), vp]
        L.vector_probe_read_stream.argtypes = [vp, sz, vp, C.POINTER(C.c_int64), vp]
        L.vector_calibrate_workspace_bytes.argtypes = [C.POINTER(Shape)]
        L.vector_calibrate_workspace_bytes.restype = sz
        L.vector_calibrate.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, sz, vp]
        L.vector_distortion_workspace_bytes.argtypes = [C.POINTER(Shape)]
        L.vector_distortion_workspace_bytes.restype = sz
        L.vector_distortion.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, vp, vp, sz, vp]
        L.vector_r2_workspace_bytes.argtypes = [C.POINTER(Shape)]
        L.vector_r2_workspace_bytes.restype = sz
        L.vector_r2.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, vp, sz, vp]
        L.vector_compress_workspace_bytes.argtypes = [C.POINTER(Shape), i32, i32]
        L.vector_compress_workspace_bytes.restype = sz
        L.vector_compress.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        L.vector_compress_batch_workspace_bytes.argtypes = [C.POINTER(Shape), C.POINTER(Batch)]
        L.vector_compress_batch_workspace_bytes.restype = sz
        L.vector_compress_batch.argtypes = [C.POINTER(Shape), C.POINTER(Batch), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vector_score_key_diversity_workspace_bytes.argtypes = [C.POINTER(Shape)]
        L.vector_score_key_diversity_workspace_bytes.restype = sz
        L.vector_score_key_diversity.argtypes = [C.POINTER(Shape), vp, vp, vp, sz, vp]
        L.vector_residual_rope.argtypes = [C.POINTER(Shape), vp, vp, vp, C.POINTER(Rope), vp, vp, sz, vp]
        L.vector_score_residual_rope.argtypes = [C.POINTER(Shape), vp, vp, vp, vp, C.POINTER(Rope), vp, vp, vp, sz, vp]
        L.vector_decode_attn_rope.argtypes = [C.POINTER(Cache), C.POINTER(Rope), vp, C.c_float, vp, i32, vp, sz, vp]
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a tensor, None for None."""
    if t is None:
        return None
    return int(t.data_ptr())


def _nbytes(t) -> int:
    return 0 if t is None else int(t.numel() * t.element_size())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    return int(getattr(stream, "cuda_stream", stream)) or None


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise VectorError(rc, where)


def strerror(code: int) -> str:
    return lib().vector_strerror(code).decode()


def vector_budget_counts(n: int, p_c: float, p_a: float):
    a, b = C.c_int32(), C.c_int32()
    _check(lib().vector_budget_counts(n, p_c, p_a, C.byref(a), C.byref(b)), "vector_budget_counts")
    return a.value, b.value


def vector_budget_counts_frac(n: int, f_retain: float, f_approx: float):
    a, b = C.c_int32(), C.c_int32()
    _check(lib().vector_budget_counts_frac(n, f_retain, f_approx, C.byref(a), C.byref(b)), "vector_budget_counts_frac")
    return a.value, b.value


def vector_pa_deploy(p_c: float, eps: float = 0.0) -> float:
    return lib().vector_pa_deploy(p_c, eps)


def vector_workspace_bytes(shape: Shape, n_pool: int, n_approx: int, batch: int = 1) -> int:
    return int(lib().vector_workspace_bytes(C.byref(shape), n_pool, n_approx, batch))


def vector_score(shape: Shape, q_win, k, score, ws, stream=None) -> None:
    _check(lib().vector_score(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(score), _ptr(ws), _nbytes(ws),
                              _stream(stream)), "vector_score")


def vector_residual(shape: Shape, k, v, W, eps, ws=None, stream=None) -> None:
    _check(lib().vector_residual(C.byref(shape), _ptr(k), _ptr(v), _ptr(W), _ptr(eps), _ptr(ws), _nbytes(ws),
                                 _stream(stream)), "vector_residual")


def vector_score_residual(shape: Shape, q_win, k, v, W, score, eps, ws, stream=None) -> None:
    _check(lib().vector_score_residual(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(v), _ptr(W), _ptr(score),
                                       _ptr(eps), _ptr(ws), _nbytes(ws), _stream(stream)), "vector_score_residual")


def vector_score_residual_lse(shape: Shape, q_win, k, v, W, lse, lse_stride_head: int, score, eps, ws, stream=None) -> None:
    _check(lib().vector_score_residual_lse(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(v), _ptr(W), _ptr(lse), lse_stride_head,
                                           _ptr(score), _ptr(eps), _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_score_residual_lse")


def vector_compress_lse(shape: Shape, q_win, k, v, W, lse, lse_stride_head: int, n_pool: int, n_approx: int, score, eps, tier,
                        idx_retain, idx_approx, k_ret, v_ret, k_apx, cap_retain: int, ws, stream=None) -> None:
    _check(lib().vector_compress_lse(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(v), _ptr(W), _ptr(lse), lse_stride_head,
                                     n_pool, n_approx, _ptr(score), _ptr(eps), _ptr(tier), _ptr(idx_retain), _ptr(idx_approx),
                                     _ptr(k_ret), _ptr(v_ret), _ptr(k_apx), cap_retain, _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_compress_lse")


def vector_route(n_kv_heads: int, seq_len: int, score, eps, n_pool: int, n_approx: int, tier, idx_retain,
                 idx_approx, ws, stream=None) -> None:
    _check(lib().vector_route(n_kv_heads, seq_len, _ptr(score), _ptr(eps), n_pool, n_approx, _ptr(tier),
                              _ptr(idx_retain), _ptr(idx_approx), _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_route")


def vector_route_static(n_kv_heads: int, seq_len: int, score, eps, n_pool: int, n_approx: int, tier, idx_retain,
                        idx_approx, stream=None) -> None:
    """vector_route on the library's own scratch array (no workspace, no allocation)."""
    _check(lib().vector_route_static(n_kv_heads, seq_len, _ptr(score), _ptr(eps), n_pool, n_approx, _ptr(tier),
                                     _ptr(idx_retain), _ptr(idx_approx), _stream(stream)), "vector_route_static")


def vector_compact(shape: Shape, k, v, idx_retain, idx_approx, n_retain: int, n_approx: int, k_ret, v_ret, k_apx,
                   cap_retain: int, stream=None) -> None:
    _check(lib().vector_compact(C.byref(shape), _ptr(k), _ptr(v), _ptr(idx_retain), _ptr(idx_approx), n_retain,
                                n_approx, _ptr(k_ret), _ptr(v_ret), _ptr(k_apx), cap_retain, _stream(stream)),
           "vector_compact")


def vector_decode_attn(cache: Cache, q, scale: float, out, ws, flags: int = 0, stream=None) -> None:
    _check(lib().vector_decode_attn(C.byref(cache), _ptr(q), float(scale), _ptr(out), flags, _ptr(ws), _nbytes(ws),
                                    _stream(stream)), "vector_decode_attn")


def vector_decode_step(cache: Cache, q, k_new, v_new, scale: float, out, ws, flags: int = 0, stream=None) -> None:
    """Decode attention with the step's own token appended to the retained segments (cache rows and
    len_retain are written)."""
    _check(lib().vector_decode_step(C.byref(cache), _ptr(q), _ptr(k_new), _ptr(v_new), float(scale), _ptr(out), flags,
                                    _ptr(ws), _nbytes(ws), _stream(stream)), "vector_decode_step")


def vector_decode_step_rope(cache: Cache, rope: Rope, q, k_new, v_new, scale: float, out, ws, flags: int = 0, stream=None) -> None:
    _check(lib().vector_decode_step_rope(C.byref(cache), C.byref(rope), _ptr(q), _ptr(k_new), _ptr(v_new), float(scale),
                                         _ptr(out), flags, _ptr(ws), _nbytes(ws), _stream(stream)), "vector_decode_step_rope")


def vector_timing_enable(on: bool) -> None:
    _check(lib().vector_timing_enable(1 if on else 0), "vector_timing_enable")


def vector_timing_read() -> dict:
    """{kernel name: (total milliseconds, launches)} since the last read; waits for the launches."""
    L = lib()
    out = {}
    for i in range(L.vector_timing_kernels()):
        ms, cnt = C.c_double(), C.c_int64()
        _check(L.vector_timing_read(i, C.byref(ms), C.byref(cnt)), "vector_timing_read")
        out[L.vector_timing_name(i).decode()] = (ms.value, cnt.value)
    return out


def vector_probe_residual_mfma(shape: Shape, k, v, W, eps, repeat: int, stream=None) -> None:
    _check(lib().vector_probe_residual_mfma(C.byref(shape), _ptr(k), _ptr(v), _ptr(W), _ptr(eps), repeat,
                                            _stream(stream)), "vector_probe_residual_mfma")


def vector_probe_mfma_loop(out, iters: int, stream=None) -> int:
    """Launch the register-only MFMA loop; returns the flops of the launch."""
    flops = C.c_int64()
    _check(lib().vector_probe_mfma_loop(_ptr(out), iters, C.byref(flops), _stream(stream)), "vector_probe_mfma_loop")
    return flops.value


def vector_probe_read_stream(src, out, stream=None) -> int:
    """Launch the read-only streaming kernel over `src`; returns the bytes the launch reads."""
    n = C.c_int64()
    _check(lib().vector_probe_read_stream(_ptr(src), _nbytes(src), _ptr(out), C.byref(n), _stream(stream)), "vector_probe_read_stream")
    return n.value


def vector_residual_rope(shape: Shape, k, v, W, rope: Rope, eps, ws=None, stream=None) -> None:
    _check(lib().vector_residual_rope(C.byref(shape), _ptr(k), _ptr(v), _ptr(W), C.byref(rope), _ptr(eps), _ptr(ws),
                                      _nbytes(ws), _stream(stream)), "vector_residual_rope")


def vector_score_residual_rope(shape: Shape, q_win, k, v, W, rope: Rope, score, eps, ws, stream=None) -> None:
    _check(lib().vector_score_residual_rope(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(v), _ptr(W), C.byref(rope),
                                            _ptr(score), _ptr(eps), _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_score_residual_rope")


def vector_decode_attn_rope(cache: Cache, rope: Rope, q, scale: float, out, ws, flags: int = 0, stream=None) -> None:
    _check(lib().vector_decode_attn_rope(C.byref(cache), C.byref(rope), _ptr(q), scale, _ptr(out), flags, _ptr(ws),
                                         _nbytes(ws), _stream(stream)), "vector_decode_attn_rope")


def vector_calibrate_workspace_bytes(shape: Shape) -> int:
    return int(lib().vector_calibrate_workspace_bytes(C.byref(shape)))


def vector_calibrate(shape: Shape, k, v, W, ws, stream=None) -> None:
    _check(lib().vector_calibrate(C.byref(shape), _ptr(k), _ptr(v), _ptr(W), _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_calibrate")


DISTORTION_FIELDS = ("E", "w_evict", "w_approx", "mu_approx", "r2_approx", "w_bar", "w_star", "threshold", "n_approx", "n_evict")


def vector_distortion_workspace_bytes(shape: Shape) -> int:
    return int(lib().vector_distortion_workspace_bytes(C.byref(shape)))


def vector_distortion(shape: Shape, weights, tier, eps, v, out, ws, stream=None) -> None:
    _check(lib().vector_distortion(C.byref(shape), _ptr(weights), _ptr(tier), _ptr(eps), _ptr(v), _ptr(out), _ptr(ws),
                                   _nbytes(ws), _stream(stream)), "vector_distortion")


R2_FIELDS = ("r2_centered", "r2_uncentered", "sse", "sst_centered", "sst_raw")


def vector_r2_workspace_bytes(shape: Shape) -> int:
    return int(lib().vector_r2_workspace_bytes(C.byref(shape)))


def vector_r2(shape: Shape, k, v, W, out, ws, stream=None) -> None:
    _check(lib().vector_r2(C.byref(shape), _ptr(k), _ptr(v), _ptr(W), _ptr(out), _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_r2")


def vector_compress_workspace_bytes(shape: Shape, n_pool: int, n_approx: int) -> int:
    return int(lib().vector_compress_workspace_bytes(C.byref(shape), n_pool, n_approx))


def vector_compress(shape: Shape, q_win, k, v, W, n_pool: int, n_approx: int, score, eps, tier, idx_retain, idx_approx,
                    k_ret, v_ret, k_apx, cap_retain: int, ws, stream=None) -> None:
    _check(lib().vector_compress(C.byref(shape), _ptr(q_win), _ptr(k), _ptr(v), _ptr(W), n_pool, n_approx, _ptr(score),
                                 _ptr(eps), _ptr(tier), _ptr(idx_retain), _ptr(idx_approx), _ptr(k_ret), _ptr(v_ret),
                                 _ptr(k_apx), cap_retain, _ptr(ws), _nbytes(ws), _stream(stream)), "vector_compress")


def vector_compress_rope(shape: Shape, rope: Rope, q_win, k, v, W, n_pool: int, n_approx: int, score, eps, tier, idx_retain,
                         idx_approx, k_ret, v_ret, k_apx, cap_retain: int, ws, stream=None) -> None:
    _check(lib().vector_compress_rope(C.byref(shape), C.byref(rope), _ptr(q_win), _ptr(k), _ptr(v), _ptr(W), n_pool, n_approx,
                                      _ptr(score), _ptr(eps), _ptr(tier), _ptr(idx_retain), _ptr(idx_approx), _ptr(k_ret),
                                      _ptr(v_ret), _ptr(k_apx), cap_retain, _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_compress_rope")


def vector_compress_batch_workspace_bytes(shape: Shape, batch: Batch) -> int:
    return int(lib().vector_compress_batch_workspace_bytes(C.byref(shape), C.byref(batch)))


def vector_compress_batch(shape: Shape, batch: Batch, q_win, k, v, W, score, eps, tier, idx_retain, idx_approx,
                          k_ret, v_ret, k_apx, ws, stream=None) -> None:
    _check(lib().vector_compress_batch(C.byref(shape), C.byref(batch), _ptr(q_win), _ptr(k), _ptr(v), _ptr(W), _ptr(score),
                                       _ptr(eps), _ptr(tier), _ptr(idx_retain), _ptr(idx_approx), _ptr(k_ret), _ptr(v_ret),
                                       _ptr(k_apx), _ptr(ws), _nbytes(ws), _stream(stream)), "vector_compress_batch")


def make_options(rope: Optional[Rope] = None, lse=None, lse_stride_head: int = 0) -> CompressOptions:
    o = CompressOptions()
    o.rope = C.pointer(rope) if rope is not None else None
    o.lse = _ptr(lse)
    o.lse_stride_head = lse_stride_head
    return o


def vector_compress_ex(shape: Shape, options: Optional[CompressOptions], q_win, k, v, W, n_pool: int, n_approx: int, score, eps, tier,
                       idx_retain, idx_approx, k_ret, v_ret, k_apx, cap_retain: int, ws, stream=None) -> None:
    _check(lib().vector_compress_ex(C.byref(shape), C.byref(options) if options is not None else None, _ptr(q_win), _ptr(k), _ptr(v),
                                    _ptr(W), n_pool, n_approx, _ptr(score), _ptr(eps), _ptr(tier), _ptr(idx_retain), _ptr(idx_approx),
                                    _ptr(k_ret), _ptr(v_ret), _ptr(k_apx), cap_retain, _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_compress_ex")


def vector_compress_batch_ex(shape: Shape, batch: Batch, options: Optional[CompressOptions], q_win, k, v, W, score, eps, tier, idx_retain,
                             idx_approx, k_ret, v_ret, k_apx, ws, stream=None) -> None:
    _check(lib().vector_compress_batch_ex(C.byref(shape), C.byref(batch), C.byref(options) if options is not None else None, _ptr(q_win),
                                          _ptr(k), _ptr(v), _ptr(W), _ptr(score), _ptr(eps), _ptr(tier), _ptr(idx_retain),
                                          _ptr(idx_approx), _ptr(k_ret), _ptr(v_ret), _ptr(k_apx), _ptr(ws), _nbytes(ws),
                                          _stream(stream)), "vector_compress_batch_ex")


def vector_compress_batch_rope(shape: Shape, batch: Batch, rope: Rope, q_win, k, v, W, score, eps, tier, idx_retain, idx_approx,
                               k_ret, v_ret, k_apx, ws, stream=None) -> None:
    _check(lib().vector_compress_batch_rope(C.byref(shape), C.byref(batch), C.byref(rope), _ptr(q_win), _ptr(k), _ptr(v), _ptr(W),
                                            _ptr(score), _ptr(eps), _ptr(tier), _ptr(idx_retain), _ptr(idx_approx), _ptr(k_ret),
                                            _ptr(v_ret), _ptr(k_apx), _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_compress_batch_rope")


def vector_score_key_diversity_workspace_bytes(shape: Shape) -> int:
    return int(lib().vector_score_key_diversity_workspace_bytes(C.byref(shape)))


def vector_score_key_diversity(shape: Shape, k, score, ws, stream=None) -> None:
    _check(lib().vector_score_key_diversity(C.byref(shape), _ptr(k), _ptr(score), _ptr(ws), _nbytes(ws), _stream(stream)),
           "vector_score_key_diversity")
