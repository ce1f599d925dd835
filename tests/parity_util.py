"""Shared checks of the GPU parity tests.

Floating-point bar (scores scaled by n, residuals, attention outputs): |g - o| <= 1e-3 + 2e-3 |o|
element by element against the float64 oracle.  Decode attention accumulates in fp32 and, for a
bf16 cache, rounds its result to bf16 on store.  The bar is applied to the fp32 result
(VECTOR_DECODE_OUT_F32); the bf16 output must then be exactly the round-to-nearest-even bf16 of
that fp32 result, so its own distance to the oracle is at most the bar plus half a bf16 ulp
(2^-9 relative), which is also asserted."""
import numpy as np
import torch

from paper_2605_23258_amd import binding as vb
from paper_2605_23258_amd import datagen as dg
from paper_2605_23258_amd import pipeline as pl

ATOL, RTOL = 1e-3, 2e-3
BF16_HALF_ULP = 2.0 ** -9


def close(got, ref, what):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"


def decode_check(cache, q_dev, scale, ws, ref, what="decode", flags=0, rope=None):
    """Run decode attention with fp32 output (and, for bf16 caches, with the native bf16 output)
    and hold both against the oracle's `ref` [B, Hq, d].  Returns the fp32 result."""
    B, Hq, d = ref.shape
    is_bf = cache.dtype == vb.VECTOR_BF16

    def run(out, fl):
        if rope is None:
            vb.vector_decode_attn(cache, q_dev, scale, out, ws, flags=fl)
        else:
            vb.vector_decode_attn_rope(cache, rope, q_dev, scale, out, ws, flags=fl)
        torch.cuda.synchronize()

    out32 = torch.full((B, Hq, d), 7.0, dtype=torch.float32, device="cuda:0")
    run(out32, flags | vb.VECTOR_DECODE_OUT_F32)
    got32 = out32.cpu().numpy()
    close(got32, ref, f"{what} (fp32 out)")
    native = torch.full((B, Hq, d), 7.0, dtype=torch.bfloat16 if is_bf else torch.float32, device="cuda:0")
    run(native, flags)
    if is_bf:
        bits = pl.to_host(native)
        assert np.array_equal(bits, dg.f32_to_bf16_bits(got32)), f"{what}: bf16 output is not the rounding of the fp32 result"
        err = np.abs(dg.widen(bits) - ref)
        assert (err <= ATOL + (RTOL + BF16_HALF_ULP) * np.abs(ref)).all(), f"{what} (bf16 out): max err {err.max():.3e}"
    else:
        assert np.array_equal(native.cpu().numpy(), got32), f"{what}: the flag must not change an fp32 cache's output"
    return got32


def band_check(score_ref, eps_ref, n_p, n_a, got_tier, ref_tier, n, what):
    """Tokens routed differently must sit within float tolerance of the oracle's own
    selection thresholds (GPU and oracle scores differ in the last bits)."""
    flips = 0
    for h in range(score_ref.shape[0]):
        diff = np.flatnonzero(got_tier[h] != ref_tier[h])
        if not len(diff):
            continue
        flips += len(diff)
        s = score_ref[h].astype(np.float64) * n
        thr_s = np.sort(s)[::-1][n_p - 1]
        pool_ref = ref_tier[h] != 0
        e = eps_ref[h].astype(np.float64)
        thr_e = np.sort(e[pool_ref])[n_a - 1] if n_a else 0.0
        for t in diff:
            near_s = abs(s[t] - thr_s) <= 2 * (ATOL + RTOL * abs(thr_s))
            near_e = abs(e[t] - thr_e) <= 2 * (ATOL + RTOL * abs(thr_e))
            assert near_s or near_e, f"{what}: head {h} token {t} flipped far from both thresholds"
    return flips
