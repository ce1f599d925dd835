"""CPU oracle for VECTOR's three-way KV-cache routing.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy statement of what the hot path computes.  It is
imported by tests, by the smoke check and by the benchmark's CPU-baseline leg,
never by the product path, and it shares no code with the HIP kernels.

Each function follows the paper's definition directly (Section 3.2, Steps 1-3;
Section 3.1 for the least-squares value map; Section 4 for the deployment rule
and the distortion measure).  The paper names its base scorer (SnapKV) without
defining it; the scorer written here is the observation-window reading fixed by
this build: causal softmax attention of the last `window` queries over all
keys, averaged over window rows and over the query heads that share a KV head,
then average-pooled along the sequence.

Row convention throughout: v_hat = k @ W, i.e. W here is the transpose of the
paper's column-convention W_OLS (footnote in Section 3.1).

Keys cached after rotary position embedding (Section 3.1, "RoPE Decoupling") are
turned back by the inverse rotation of their position before the value map is
applied; attention logits always use the cached (rotated) keys.

Pins (tests/test_oracle_*.py): softmax-row mass conservation, the q = 0 closed
form, reduction to a textbook softmax, brute-force routing on tiny inputs, the
truncated-Gaussian closed form of Example 1, planted-map recovery by the
least-squares fit, the printed p_a table, identities of decode attention, and for
the rotary un-rotation its dense block-rotation matrix, R^-1 R = I, the relative-
position property of rotated dot products and a hand-computed quarter turn.
Not pinned against the authors' own code (none is published with the paper):
the scorer reading (mean vs sum, pooling pad, window handling) is this build's.
"""
from __future__ import annotations

import math
from typing import Tuple

import numpy as np

EVICT, APPROX, RETAIN = 0, 1, 2


# ----------------------------------------------------------------------------
# budget arithmetic (Section 3.2 last paragraph; Section 4, deployment formula)
# ----------------------------------------------------------------------------
def pa_deploy(p_c: float, eps: float = 0.0) -> float:
    """Approximation ratio used at deployment: the smaller of half the
    compression ratio and half the head-room left for the retention tier."""
    return min(p_c / 2.0, (1.0 - p_c - eps) / 2.0)


def tier_fractions(p_c: float, p_a: float) -> Tuple[float, float, float, float]:
    """(evict, approximate, retain, pool) token fractions of Section 3.2."""
    return p_c - p_a, 2.0 * p_a, 1.0 - p_c - p_a, 1.0 - p_c + p_a


def budget_counts(n: int, p_c: float, p_a: float) -> Tuple[int, int]:
    """(n_pool, n_approx) from the paper's ratios; counts are floors, and the
    pool is the sum of the floored retain and approximate counts."""
    _, f_a, f_r, _ = tier_fractions(p_c, p_a)
    return budget_counts_frac(n, f_r, f_a)


def budget_counts_frac(n: int, f_retain: float, f_approx: float) -> Tuple[int, int]:
    """Floors of fraction * n.  The paper's ratios are decimals (Section 5 uses p_c = 0.9 with
    p_a = 0.05) that doubles only approximate, so a product within 1e-9 of an integer is taken
    as that integer: 5 % of 1000 tokens is 50 tokens."""
    def count(f: float) -> int:
        x = f * n
        r = round(x)
        return int(r) if abs(x - r) <= 1e-9 else int(math.floor(x))
    n_r, n_a = count(f_retain), count(f_approx)
    return n_r + n_a, n_a


# ----------------------------------------------------------------------------
# Section 3.1: least-squares value map (no intercept), row convention
# ----------------------------------------------------------------------------
def ols_fit(k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """argmin_W || k W - v ||_F^2 through the normal equations, per head.
    k [H, m, d_k], v [H, m, d_v] -> W [H, d_k, d_v]."""
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    out = np.empty((k.shape[0], k.shape[2], v.shape[2]))
    for h in range(k.shape[0]):
        gram = k[h].T @ k[h]
        out[h] = np.linalg.solve(gram, k[h].T @ v[h])
    return out


def r2_global(k: np.ndarray, v: np.ndarray, w: np.ndarray) -> dict:
    """Section 3.1, predictability of values from keys on a set of tokens (the paper reports
    it on held-out sequences), per head:
      sse           sum_t || v_t - k_t W ||^2
      sst_centered  sum_t || v_t - mean_t v ||^2      r2_centered   = 1 - sse / sst_centered
      sst_raw       sum_t || v_t ||^2                 r2_uncentered = 1 - sse / sst_raw
    The centred form is the usual coefficient of determination (all value dimensions pooled);
    the other is one minus the mean relative error that Section 4 uses."""
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    diff = v - np.einsum("hti,hij->htj", k, w)
    sse = (diff * diff).sum(axis=(1, 2))
    sst_c = ((v - v.mean(axis=1, keepdims=True)) ** 2).sum(axis=(1, 2))
    sst_r = (v * v).sum(axis=(1, 2))
    return {"r2_centered": 1.0 - sse / sst_c, "r2_uncentered": 1.0 - sse / sst_r, "sse": sse, "sst_centered": sst_c,
            "sst_raw": sst_r}


# ----------------------------------------------------------------------------
# base scorer (observation-window attention mass, pooled)
# ----------------------------------------------------------------------------
def attention_mass(q_win: np.ndarray, k: np.ndarray) -> np.ndarray:
    """mass[h, t]: mean over the G query heads of KV head h and over the w
    window rows of the causal softmax probability put on key t.
    q_win [Hq, w, d], k [Hkv, n, d]; window row r sits at position n - w + r."""
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    n_q, w, d = q_win.shape
    n_kv, n, _ = k.shape
    group = n_q // n_kv
    mass = np.zeros((n_kv, n))
    for h in range(n_kv):
        for g in range(group):
            s = (q_win[h * group + g] @ k[h].T) / math.sqrt(d)        # [w, n]
            for r in range(w):
                s[r, n - w + r + 1:] = -np.inf                        # causal mask
            s -= s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p /= p.sum(axis=1, keepdims=True)
            mass[h] += p.sum(axis=0)
        mass[h] /= group * w
    return mass


def score_key_diversity(k: np.ndarray) -> np.ndarray:
    """A query-agnostic importance score (Section 5 names scorers that rank tokens by the
    geometric diversity of their keys, without giving a formula; this is this build's reading):
    with a_h the direction of the mean of the head's unit-normalised keys,
        score[h, t] = - cos(k[h, t], a_h),
    so keys that point away from the common direction rank highest.  k [H, n, d] -> float32 [H, n]."""
    k = np.asarray(k, dtype=np.float64)
    unit = k / np.linalg.norm(k, axis=-1, keepdims=True)
    anchor = unit.sum(axis=1)
    anchor /= np.linalg.norm(anchor, axis=-1, keepdims=True)
    return (-(unit * anchor[:, None, :]).sum(axis=-1)).astype(np.float32)


def pool_scores(mass: np.ndarray, window: int, pool_kernel: int, pool_mode: str = "avg") -> np.ndarray:
    """1-D pooling (stride 1, odd kernel, centred) over the prefix columns [0, n - w); window
    columns get +inf.  "avg": zero padding, divisor always the kernel size.  "max": the largest
    mass among the columns of the kernel that lie inside the prefix (mass is never negative, so
    this equals padding with zeros)."""
    assert pool_mode in ("avg", "max")
    n_kv, n = mass.shape
    n_prefix = n - window
    half = pool_kernel // 2
    score = np.full((n_kv, n), np.inf)
    for h in range(n_kv):
        for t in range(n_prefix):
            lo, hi = max(0, t - half), min(n_prefix, t + half + 1)
            if pool_mode == "avg":
                score[h, t] = mass[h, lo:hi].sum() / pool_kernel
            else:
                score[h, t] = mass[h, lo:hi].max()
    return score


def score(q_win: np.ndarray, k: np.ndarray, window: int, pool_kernel: int, pool_mode: str = "avg") -> np.ndarray:
    """Importance score per KV head and token, float32 as the routing consumes it."""
    assert q_win.shape[1] == window
    return pool_scores(attention_mass(q_win, k), window, pool_kernel, pool_mode).astype(np.float32)


# ----------------------------------------------------------------------------
# Step 2: reconstruction residual
# ----------------------------------------------------------------------------
def rope_unrotate(k_post: np.ndarray, pos: np.ndarray, inv_freq: np.ndarray, interleaved: bool = False) -> np.ndarray:
    """Section 3.1, RoPE decoupling: R_m^{-1} applied to each cached key row.

    R_m turns pair i of a row, (a_i, b_i), by the angle m * inv_freq[i]:
    (a, b) -> (a cos - b sin, a sin + b cos); its inverse turns it back by the
    same angle.  Pair i is (x[i], x[i + d/2]), or (x[2i], x[2i+1]) when
    `interleaved`.  k_post [..., n, d], pos [..., n] (integers), inv_freq [d/2].
    Returns float64."""
    x = np.asarray(k_post, dtype=np.float64)
    d = x.shape[-1]
    ang = np.asarray(pos, dtype=np.float64)[..., None] * np.asarray(inv_freq, dtype=np.float64)
    c, s_ = np.cos(ang), np.sin(ang)
    if interleaved:
        a, b = x[..., 0::2], x[..., 1::2]
    else:
        a, b = x[..., : d // 2], x[..., d // 2:]
    a_pre = a * c + b * s_
    b_pre = -a * s_ + b * c
    out = np.empty_like(x)
    if interleaved:
        out[..., 0::2], out[..., 1::2] = a_pre, b_pre
    else:
        out[..., : d // 2], out[..., d // 2:] = a_pre, b_pre
    return out


def residual(k: np.ndarray, v: np.ndarray, w: np.ndarray, pos: np.ndarray = None, inv_freq: np.ndarray = None,
             interleaved: bool = False) -> np.ndarray:
    """eps[h, t] = || v[h,t] - k[h,t] @ W[h] ||_2^2 (squared, un-normalised),
    for every token; float32 as the routing consumes it.  With `inv_freq` the
    keys are post-RoPE and are un-rotated by their positions first (pos [n] or
    [H, n]; None = the row index)."""
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    if inv_freq is not None:
        if pos is None:
            pos = np.arange(k.shape[1])
        k = rope_unrotate(k, np.broadcast_to(pos, k.shape[:2]), inv_freq, interleaved)
    eps = np.empty(k.shape[:2])
    for h in range(k.shape[0]):
        diff = v[h] - k[h] @ w[h]
        eps[h] = (diff * diff).sum(axis=1)
    return eps.astype(np.float32)


# ----------------------------------------------------------------------------
# Steps 1 and 3: pool by importance, then split the pool by residual
# ----------------------------------------------------------------------------
def route(score_: np.ndarray, eps: np.ndarray, n_pool: int, n_approx: int):
    """Per head: pool = the n_pool tokens of highest score; approx = the
    n_approx pool tokens of lowest eps; retain = the rest of the pool.
    Ties go to the lower token index in both selections.
    Returns tier [H, n] uint8, idx_retain [H, n_pool - n_approx] int32 ascending,
    idx_approx [H, n_approx] int32 ascending."""
    score_ = np.asarray(score_, dtype=np.float32)
    eps = np.asarray(eps, dtype=np.float32)
    n_kv, n = score_.shape
    assert 0 <= n_approx <= n_pool <= n
    tier = np.zeros((n_kv, n), dtype=np.uint8)
    idx_r = np.empty((n_kv, n_pool - n_approx), dtype=np.int32)
    idx_a = np.empty((n_kv, n_approx), dtype=np.int32)
    for h in range(n_kv):
        by_score = sorted(range(n), key=lambda t: (-float(score_[h, t]), t))
        pool = sorted(by_score[:n_pool])
        by_eps = sorted(pool, key=lambda t: (float(eps[h, t]), t))
        approx = sorted(by_eps[:n_approx])
        retain = sorted(by_eps[n_approx:])
        tier[h, approx] = APPROX
        tier[h, retain] = RETAIN
        idx_a[h] = approx
        idx_r[h] = retain
    return tier, idx_r, idx_a


# ----------------------------------------------------------------------------
# packed cache: keys of the whole pool, values of retained tokens only
# ----------------------------------------------------------------------------
def compact(k: np.ndarray, v: np.ndarray, idx_retain: np.ndarray, idx_approx: np.ndarray):
    """Gather k_ret, v_ret [H, n_r, d] and k_apx [H, n_a, d] by the index lists.
    Works on any element type (rows are copied, not converted)."""
    n_kv = k.shape[0]
    k_ret = np.stack([k[h][idx_retain[h]] for h in range(n_kv)])
    v_ret = np.stack([v[h][idx_retain[h]] for h in range(n_kv)])
    k_apx = np.stack([k[h][idx_approx[h]] for h in range(n_kv)])
    return k_ret, v_ret, k_apx


# ----------------------------------------------------------------------------
# decode attention over the packed cache, approximated values rebuilt as k @ W
# ----------------------------------------------------------------------------
def decode_attn(q: np.ndarray, k_ret: np.ndarray, v_ret: np.ndarray, len_retain: np.ndarray,
                k_apx: np.ndarray, w: np.ndarray, scale: float, pos_apx: np.ndarray = None,
                inv_freq: np.ndarray = None, interleaved: bool = False) -> np.ndarray:
    """q [B, Hq, d]; k_ret, v_ret [B, Hkv, cap, d] of which the first
    len_retain[b] rows are live; k_apx [B, Hkv, n_a, d]; W [Hkv, d, d].
    One softmax over retained and approximated tokens together;
    out = sum_ret p_t v_t + sum_apx p_t (k_t @ W).  With `inv_freq` the cached keys
    are post-RoPE: logits use them as they are, and the rebuilt value of an
    approximated token comes from its key un-rotated by its original position
    pos_apx [B, Hkv, n_a].  Returns float64 [B, Hq, d]."""
    q = np.asarray(q, dtype=np.float64)
    k_ret = np.asarray(k_ret, dtype=np.float64)
    v_ret = np.asarray(v_ret, dtype=np.float64)
    k_apx = np.asarray(k_apx, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    n_b, n_q, d = q.shape
    n_kv = k_ret.shape[1]
    group = n_q // n_kv
    out = np.zeros((n_b, n_q, d))
    for b in range(n_b):
        length = int(len_retain[b])
        for h in range(n_kv):
            keys = np.concatenate([k_ret[b, h, :length], k_apx[b, h]], axis=0)
            k_lin = k_apx[b, h]
            if inv_freq is not None:
                k_lin = rope_unrotate(k_lin, np.asarray(pos_apx)[b, h], inv_freq, interleaved)
            v_hat = k_lin @ w[h]                          # rebuilt values
            vals = np.concatenate([v_ret[b, h, :length], v_hat], axis=0)
            for g in range(group):
                qh = h * group + g
                s = (keys @ q[b, qh]) * scale
                s -= s.max()
                p = np.exp(s)
                p /= p.sum()
                out[b, qh] = p @ vals
    return out


# ----------------------------------------------------------------------------
# Section 4: distortion measure (diagnostic; used by tests of the routing)
# ----------------------------------------------------------------------------
def distortion(weights: np.ndarray, tier: np.ndarray, eps: np.ndarray, v_sqnorm: np.ndarray) -> np.ndarray:
    """E = sum_evicted w_i + sum_approx w_i * eps_i / ||v_i||^2, per head."""
    weights = np.asarray(weights, dtype=np.float64)
    rel = np.asarray(eps, dtype=np.float64) / np.asarray(v_sqnorm, dtype=np.float64)
    return (weights * (tier == EVICT)).sum(axis=1) + (weights * rel * (tier == APPROX)).sum(axis=1)


def distortion_report(weights: np.ndarray, tier: np.ndarray, eps: np.ndarray, v: np.ndarray) -> dict:
    """The quantities of Section 4 per head, from importance weights w [H, n] (summing to one
    per head), the routing, the residuals and the values v [H, n, d]:

      E          the distortion above
      w_evict    sum of w over evicted tokens;  w_approx  the same over approximated tokens
      mu_approx  mean over approximated tokens of eps_i / ||v_i||^2;  r2_approx = 1 - mu_approx
      w_bar      (1 - w_evict) / (pool fraction): mean pool weight relative to the uniform 1/n
      w_star     n * (largest weight among evicted tokens): the token at the truncation boundary
                 of the eviction set, on the same scale (0 when nothing is evicted)
      threshold  w_bar / (w_star + w_bar): Proposition 1 says that growing the approximation
                 tier lowers E when r2_approx exceeds it."""
    w = np.asarray(weights, dtype=np.float64)
    e = np.asarray(eps, dtype=np.float64)
    vsq = (np.asarray(v, dtype=np.float64) ** 2).sum(axis=-1)
    n = w.shape[1]
    ev, ap = tier == EVICT, tier == APPROX
    rel = e / vsq
    n_ap = ap.sum(axis=1)
    w_evict = (w * ev).sum(axis=1)
    mu = np.where(n_ap > 0, (rel * ap).sum(axis=1) / np.maximum(n_ap, 1), 0.0)
    pool_frac = (~ev).sum(axis=1) / n
    w_bar = (1.0 - w_evict) / pool_frac
    w_star = n * np.where(ev, w, 0.0).max(axis=1)
    return {"E": w_evict + (w * rel * ap).sum(axis=1), "w_evict": w_evict, "w_approx": (w * ap).sum(axis=1),
            "mu_approx": mu, "r2_approx": 1.0 - mu, "w_bar": w_bar, "w_star": w_star,
            "threshold": w_bar / (w_star + w_bar), "n_approx": n_ap, "n_evict": ev.sum(axis=1)}
