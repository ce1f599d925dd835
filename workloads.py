"""Harness: the five synthetic workloads as the tests, the smoke check and the benchmark use them.

The compression pass takes the calibrated value map W as an input: the paper fits it offline,
once per model, by ordinary least squares (Section 3.1).  The harness plays that offline step
with a library least-squares call on a separate seeded draw of 4096 tokens, and hands the
result to both the HIP path and the CPU oracle.  Nothing here is part of the product path, and
neither the oracle's own normal-equation fit nor the library's GPU calibration is used for it
(the oracle's fit is pinned to agree with this one in tests/test_oracle_residual_ols.py).
"""
from __future__ import annotations

import numpy as np

from paper_2605_23258_amd import datagen as dg


def fit_w(k_cal: np.ndarray, v_cal: np.ndarray) -> np.ndarray:
    """Least-squares value map per head on a calibration draw (library lstsq, fp64):
    k_cal [H, m, d], v_cal [H, m, d] -> W [H, d, d] with v_hat = k @ W."""
    out = np.empty((k_cal.shape[0], k_cal.shape[2], v_cal.shape[2]), dtype=np.float64)
    for h in range(k_cal.shape[0]):
        out[h] = np.linalg.lstsq(k_cal[h].astype(np.float64), v_cal[h].astype(np.float64), rcond=None)[0]
    return out


def make_layer(cfg: dg.Config, layer: int = 0, **kw) -> dg.LayerInputs:
    """datagen.make_layer with the harness's calibration."""
    return dg.make_layer(cfg, fit_w, layer, **kw)
