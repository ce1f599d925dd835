"""Seeded synthetic inputs for the VECTOR compression pass and decode attention.

This module only draws numbers. It holds none of the method's arithmetic (no
scoring, residual, routing, attention or least-squares fit): it produces the
planted-regression K/V tensors and observation-window queries, and the separate
seeded calibration draw from which the caller fits the value map that the paper's
Section 3.1 obtains offline (the fit itself is passed in as a callable).

Every stream is a counter-based Philox generator keyed by
(master seed, config id, layer, tag), so any tensor can be regenerated on its
own and the same bits reach the CPU oracle and the HIP path.  Master seed 42
is the seed the paper's reproducibility appendix uses.

bf16 tensors are carried as uint16 bit patterns (round-to-nearest-even from
fp32); `widen()` turns either representation into exact float64.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

MASTER_SEED = 42

# tensor tags (Philox key lanes)
_TAG_K, _TAG_WTRUE, _TAG_SIGMA, _TAG_NOISE, _TAG_Q, _TAG_HEAVY = 1, 2, 3, 4, 5, 6
_TAG_CAL = 32          # added to the tags above for the calibration draw
_TAG_DECODE = 64       # per-step decode draws


def _rng(cfg_id: int, layer: int, tag: int, sub: int = 0, seed: int = MASTER_SEED) -> np.random.Generator:
    key0 = np.uint64(seed)
    key1 = (np.uint64(cfg_id) << np.uint64(48)) | (np.uint64(layer) << np.uint64(32)) \
        | (np.uint64(tag) << np.uint64(20)) | np.uint64(sub)
    return np.random.Generator(np.random.Philox(key=np.array([key0, key1], dtype=np.uint64)))


# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit handling (format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = (b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def widen(x: np.ndarray) -> np.ndarray:
    """Exact float64 view of a stored tensor (uint16 = bf16 bits, else float)."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


# ----------------------------------------------------------------------------
# workload descriptions
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    cfg_id: int
    name: str
    dtype: str                 # "f32" | "bf16"
    layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    window: int
    pool_kernel: int
    f_retain: float
    f_approx: float
    sigma_law: str             # "loguniform" | "bimodal"
    heavy_frac: float          # fraction of tokens whose keys are scaled
    heavy_scale: float = 4.0
    cal_tokens: int = 4096
    decode_steps: int = 0
    pool_mode: str = "avg"     # "avg" | "max"

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def counts(self):
        """(n_retain, n_approx, n_pool): floor of the token fractions, in double."""
        n_r = int(np.floor(self.f_retain * self.seq_len))
        n_a = int(np.floor(self.f_approx * self.seq_len))
        return n_r, n_a, n_r + n_a


CONFIGS: Dict[str, Config] = {
    "cfg1": Config(1, "tiny-f32", "f32", 1, 1, 4, 1, 64, 1024, 32, 7, 0.25, 0.25, "loguniform", 0.0),
    "cfg2": Config(2, "llama3-8b-layer", "bf16", 1, 1, 32, 8, 128, 8192, 32, 7, 0.15, 0.15, "loguniform", 0.05),
    "cfg3": Config(3, "prefill-32layer-32k", "bf16", 32, 1, 32, 8, 128, 32768, 64, 7, 0.10, 0.10, "loguniform", 0.05),
    "cfg4": Config(4, "long-context-128k", "bf16", 1, 1, 32, 8, 128, 131072, 32, 7, 0.05, 0.05, "bimodal", 0.05),
    "cfg5": Config(5, "decode-b16-32k", "bf16", 1, 16, 32, 8, 128, 32768, 64, 7, 0.10, 0.10, "loguniform", 0.05,
                   decode_steps=256),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a config with some fields replaced (smaller parity-test cases)."""
    d = {f: getattr(cfg, f) for f in cfg.__dataclass_fields__}
    d.update(kw)
    return Config(**d)


@dataclass
class LayerInputs:
    """One layer (or one sequence) worth of inputs.  Arrays are fp32 or bf16 bits."""
    cfg: Config
    layer: int
    q_win: np.ndarray          # [Hq, w, d]
    k: np.ndarray              # [Hkv, n, d]
    v: np.ndarray              # [Hkv, n, d]
    w_cal: np.ndarray          # [Hkv, d, d]  (v_hat = k @ w_cal)
    w_true: np.ndarray         # [Hkv, d, d]  float64, for tests of the recipe only
    sigma: np.ndarray          # [Hkv, n]     float64
    heavy: np.ndarray          # [Hkv, n]     bool
    extra: dict = field(default_factory=dict)


def _sigma(cfg: Config, rng: np.random.Generator, shape) -> np.ndarray:
    u = rng.random(shape)
    if cfg.sigma_law == "loguniform":          # log-uniform on [1e-3, 1]
        return 10.0 ** (-3.0 * u)
    if cfg.sigma_law == "bimodal":             # 70 % at 1e-2, 30 % at 1.0
        return np.where(u < 0.7, 1e-2, 1.0)
    raise ValueError(cfg.sigma_law)


def _store(cfg: Config, x: np.ndarray) -> np.ndarray:
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    return f32_to_bf16_bits(x32) if cfg.dtype == "bf16" else x32


def _draw_kv(cfg: Config, layer: int, n: int, w_true: np.ndarray, tag_off: int, sub: int = 0):
    """K ~ N(0,1) with heavy-hitter rows scaled, V = K W_true + sigma_t N(0,1)."""
    H, d = cfg.n_kv_heads, cfg.head_dim
    k = _rng(cfg.cfg_id, layer, _TAG_K + tag_off, sub).standard_normal((H, n, d), dtype=np.float32)
    heavy = np.zeros((H, n), dtype=bool)
    if cfg.heavy_frac > 0.0:
        heavy = _rng(cfg.cfg_id, layer, _TAG_HEAVY + tag_off, sub).random((H, n)) < cfg.heavy_frac
        k[heavy] *= np.float32(cfg.heavy_scale)
    sigma = _sigma(cfg, _rng(cfg.cfg_id, layer, _TAG_SIGMA + tag_off, sub), (H, n))
    noise = _rng(cfg.cfg_id, layer, _TAG_NOISE + tag_off, sub).standard_normal((H, n, d), dtype=np.float32)
    v = np.matmul(k, w_true.astype(np.float32)) + sigma.astype(np.float32)[..., None] * noise
    return k, v, sigma, heavy


def rotary_inv_freq(head_dim: int, theta: float) -> np.ndarray:
    """Angular frequency of pair i: theta^(-2i/d), float64 [d/2]."""
    return np.asarray(theta, dtype=np.float64) ** (-np.arange(head_dim // 2, dtype=np.float64) * 2.0 / head_dim)


def apply_rotary(x: np.ndarray, pos: np.ndarray, inv_freq: np.ndarray, interleaved: bool = False) -> np.ndarray:
    """Rows of x [..., n, d] as a model with rotary position embedding would cache them:
    pair i of row t turned forward by pos[t] * inv_freq[i].  float64 in, float64 out."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    ang = np.asarray(pos, dtype=np.float64)[..., None] * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    if interleaved:
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2], out[..., 1::2] = a * c - b * s, a * s + b * c
    else:
        a, b = x[..., : d // 2], x[..., d // 2:]
        out[..., : d // 2], out[..., d // 2:] = a * c - b * s, a * s + b * c
    return out


def make_layer(cfg: Config, fit, layer: int = 0, sub: int = 0, rope_theta: Optional[float] = None,
               rope_interleaved: bool = False, pos_offset: int = 0) -> LayerInputs:
    """Inputs of one compression pass: one layer of one sequence (`sub` = sequence id).

    `fit(k_cal, v_cal) -> W [Hkv, d, d]` is the caller's offline calibration of the value map
    (Section 3.1), run on a separate draw of `cfg.cal_tokens` tokens of the same law; this module
    draws numbers and does none of the method's arithmetic itself.

    With `rope_theta` the stored keys are post-RoPE: the values (and the calibrated map) belong
    to the keys as drawn, and row t of the stored keys is that key turned by position
    pos_offset + t.  `extra` then holds inv_freq (float64 [d/2]), the positions, and the flag."""
    H, d, n, w = cfg.n_kv_heads, cfg.head_dim, cfg.seq_len, cfg.window
    w_true = _rng(cfg.cfg_id, layer, _TAG_WTRUE, sub).standard_normal((H, d, d)) / np.sqrt(d)
    k, v, sigma, heavy = _draw_kv(cfg, layer, n, w_true, 0, sub)
    k_cal, v_cal, _, _ = _draw_kv(cfg, layer, cfg.cal_tokens, w_true, _TAG_CAL, sub)
    w_cal = fit(k_cal, v_cal)
    q = _rng(cfg.cfg_id, layer, _TAG_Q, sub).standard_normal((cfg.n_q_heads, w, d), dtype=np.float32)
    extra = {}
    if rope_theta is not None:
        inv_freq = rotary_inv_freq(d, rope_theta)
        pos = np.arange(n, dtype=np.int64) + pos_offset
        k = apply_rotary(k, pos, inv_freq, rope_interleaved)
        extra = {"inv_freq": inv_freq, "pos": pos.astype(np.int32), "interleaved": rope_interleaved}
    return LayerInputs(cfg, layer, _store(cfg, q), _store(cfg, k), _store(cfg, v), _store(cfg, w_cal),
                       w_true, sigma, heavy, extra)


def make_decode_step(cfg: Config, step: int, w_true_per_seq: Optional[np.ndarray] = None):
    """Per decode step: one query per (sequence, query head) and the new token's
    exact (k, v) per (sequence, kv head), drawn by the same law as the context."""
    B, Hq, H, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    q = _rng(cfg.cfg_id, 0, _TAG_DECODE + _TAG_Q, step).standard_normal((B, Hq, d), dtype=np.float32)
    k = _rng(cfg.cfg_id, 0, _TAG_DECODE + _TAG_K, step).standard_normal((B, H, d), dtype=np.float32)
    sig = _sigma(cfg, _rng(cfg.cfg_id, 0, _TAG_DECODE + _TAG_SIGMA, step), (B, H)).astype(np.float32)
    noise = _rng(cfg.cfg_id, 0, _TAG_DECODE + _TAG_NOISE, step).standard_normal((B, H, d), dtype=np.float32)
    if w_true_per_seq is None:
        v = sig[..., None] * noise
    else:                                          # [B, H, d, d]
        v = np.einsum("bhi,bhij->bhj", k, w_true_per_seq.astype(np.float32)) + sig[..., None] * noise
    return _store(cfg, q), _store(cfg, k), _store(cfg, v)
