"""Buffer management around the C ABI: device tensors, workspaces and the order
of calls of one compression pass.  No arithmetic of the method happens here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding as vb
from .datagen import Config


def to_device(arr: np.ndarray, device="cuda:0") -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bf16 bit patterns."""
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16).copy()).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(arr)).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> numpy; bf16 comes back as uint16 bit patterns."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def shape_of(cfg: Config, seq_len: Optional[int] = None) -> vb.Shape:
    return vb.Shape(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                    seq_len=seq_len or cfg.seq_len, window=cfg.window, pool_kernel=cfg.pool_kernel,
                    pool_mode=vb.VECTOR_POOL_MAX if cfg.pool_mode == "max" else vb.VECTOR_POOL_AVG,
                    dtype=vb.VECTOR_BF16 if cfg.dtype == "bf16" else vb.VECTOR_F32)


def alloc_workspace(nbytes: int, device="cuda:0") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


@dataclass
class Compressed:
    score: torch.Tensor        # [Hkv, n] fp32
    eps: torch.Tensor          # [Hkv, n] fp32
    tier: torch.Tensor         # [Hkv, n] u8
    idx_retain: torch.Tensor   # [Hkv, n_r] i32
    idx_approx: torch.Tensor   # [Hkv, n_a] i32
    k_ret: torch.Tensor        # [Hkv, cap, d]
    v_ret: torch.Tensor
    k_apx: torch.Tensor        # [Hkv, n_a, d]


def alloc_outputs(shape: vb.Shape, n_pool: int, n_approx: int, cap_retain: int, dtype: torch.dtype,
                  device="cuda:0") -> Compressed:
    H, n, d = shape.n_kv_heads, shape.seq_len, shape.head_dim
    n_r = n_pool - n_approx
    f32, dev = torch.float32, device
    return Compressed(
        score=torch.empty((H, n), dtype=f32, device=dev), eps=torch.empty((H, n), dtype=f32, device=dev),
        tier=torch.empty((H, n), dtype=torch.uint8, device=dev),
        idx_retain=torch.empty((H, max(n_r, 1)), dtype=torch.int32, device=dev)[:, :n_r],
        idx_approx=torch.empty((H, max(n_approx, 1)), dtype=torch.int32, device=dev)[:, :n_approx],
        k_ret=torch.zeros((H, max(cap_retain, 1), d), dtype=dtype, device=dev),
        v_ret=torch.zeros((H, max(cap_retain, 1), d), dtype=dtype, device=dev),
        k_apx=torch.zeros((H, max(n_approx, 1), d), dtype=dtype, device=dev))


def compress_layer(shape: vb.Shape, q_win, k, v, W, n_pool: int, n_approx: int, out: Compressed, ws,
                   cap_retain: Optional[int] = None, fused: bool = True, stream=None, one_call: bool = False) -> Compressed:
    """One compression pass: score + residual -> route -> compact, all enqueued on one stream.
    `one_call` uses vector_compress (ws of vector_compress_workspace_bytes) instead of the three calls."""
    n_r = n_pool - n_approx
    cap = cap_retain if cap_retain is not None else out.k_ret.shape[1]
    if one_call:
        vb.vector_compress(shape, q_win, k, v, W, n_pool, n_approx, out.score, out.eps, out.tier,
                           out.idx_retain if n_r else None, out.idx_approx if n_approx else None,
                           out.k_ret, out.v_ret, out.k_apx, cap, ws, stream)
        return out
    if fused:
        vb.vector_score_residual(shape, q_win, k, v, W, out.score, out.eps, ws, stream)
    else:
        vb.vector_score(shape, q_win, k, out.score, ws, stream)
        vb.vector_residual(shape, k, v, W, out.eps, ws, stream)
    vb.vector_route(shape.n_kv_heads, shape.seq_len, out.score, out.eps, n_pool, n_approx, out.tier,
                    out.idx_retain if n_r else None, out.idx_approx if n_approx else None, ws, stream)
    vb.vector_compact(shape, k, v, out.idx_retain if n_r else None, out.idx_approx if n_approx else None,
                      n_r, n_approx, out.k_ret, out.v_ret, out.k_apx, cap, stream)
    return out
