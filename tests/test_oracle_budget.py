"""Pins for the budget arithmetic against the values the paper prints."""
import os

import numpy as np
import pytest

from oracle import vector_oracle as vo
from paper_2605_23258_amd import datagen as dg


def _rows(path):
    with open(path) as f:
        return [tuple(float(x) for x in line.split()) for line in f if line.strip() and not line.startswith("#")]


def test_printed_pa_table(golden_dir):
    for p_c, p_a in _rows(os.path.join(golden_dir, "pa_table.txt")):
        assert vo.pa_deploy(p_c, 0.0) == pytest.approx(p_a, abs=1e-12)
        # a small positive epsilon only matters where the second term binds
        assert vo.pa_deploy(p_c, 1e-6) <= p_a


def test_tier_fractions(golden_dir):
    for p_c, p_a, ev, ap, re, pool in _rows(os.path.join(golden_dir, "tier_fractions.txt")):
        got = vo.tier_fractions(p_c, p_a)
        assert got == pytest.approx((ev, ap, re, pool), abs=1e-12)
        assert sum(got[:3]) == pytest.approx(1.0)
        # memory identity: pool keys + retained values = 2 (1 - p_c) half-pairs
        assert got[3] + got[2] == pytest.approx(2 * (1 - p_c))


def test_counts_of_the_five_workloads():
    expect = {"cfg1": (256, 256, 512), "cfg2": (1228, 1228, 2456), "cfg3": (3276, 3276, 6552),
              "cfg4": (6553, 6553, 13106), "cfg5": (3276, 3276, 6552)}
    for name, cfg in dg.CONFIGS.items():
        assert cfg.counts() == expect[name]
        n_pool, n_approx = vo.budget_counts_frac(cfg.seq_len, cfg.f_retain, cfg.f_approx)
        assert (n_pool - n_approx, n_approx, n_pool) == expect[name]


def test_counts_from_paper_ratios():
    n = 30000
    for p_c in (0.25, 0.5, 0.75, 0.9):
        p_a = vo.pa_deploy(p_c)
        n_pool, n_approx = vo.budget_counts(n, p_c, p_a)
        assert abs(n_approx - 2 * p_a * n) <= 1 and abs(n_pool - (1 - p_c + p_a) * n) <= 2
        assert n_pool + (n_pool - n_approx) <= 2 * (1 - p_c) * n + 1e-9


def test_exact_counts_at_decimal_ratios():
    """Hand values.  Section 5 runs p_c = 0.9 with p_a = 0.05: of 1000 tokens 5 % = 50 are retained and
    10 % = 100 approximated, although 1 - 0.9 - 0.05 is a hair below 0.05 in binary floating point.
    Products that are not integers are still floored."""
    assert vo.budget_counts(1000, 0.9, 0.05) == (150, 100)
    assert vo.budget_counts(30000, 0.9, 0.05) == (4500, 3000)
    assert vo.budget_counts(1000, 0.8, 0.1) == (300, 200)
    assert vo.budget_counts(1001, 0.9, 0.05) == (150, 100)          # 50.05 -> 50, 100.1 -> 100
    assert vo.budget_counts(7, 0.5, 0.25) == (4, 3)                 # 1.75 -> 1, 3.5 -> 3
    assert vo.budget_counts_frac(10, 0.29, 0.0) == (2, 0)           # 2.9 stays 2
