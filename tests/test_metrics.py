"""The reporting helpers against the numbers the paper prints.  CPU only."""
import os

import pytest

from paper_2511_20340_amd import metrics

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_numbers.txt")


def gold():
    rows = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if line:
            key, *vals = line.split()
            rows.setdefault(key, []).append([float(v) for v in vals])
    return rows


def test_a100_arithmetic_intensity():
    (flops, bw, want), = gold()["ai_c_a100"]
    assert metrics.chip_ai(flops * 1e12, bw * 1e12) == pytest.approx(want, abs=5e-3)
    assert metrics.model_ai(2.0) == 1.0                       # AI_m = 2M / (2 bytes * M) = 1
    assert metrics.redundancy_ratio(flops * 1e12, bw * 1e12) == pytest.approx(want, abs=5e-3)


def test_theta_reproduces_the_model_size_table():
    for kap, speed, want in gold()["theta"]:
        assert metrics.theta(kap, speed) == pytest.approx(want, abs=0.0151)   # table prints 2 decimals


def test_kappa_and_cost_factor():
    assert metrics.kappa(1.0, 1, 0) == 1.0                     # W/o SD rows: kappa = 1
    assert metrics.kappa(1.75, 4, 4) == 1.75                   # no tree: l_d == k
    shared, per_pos = metrics.draft_param_counts(4096, 32, 8, 128, 14336, 4)
    assert per_pos == 4096 * 4096 + 4096                       # l_d * d_h^2 position-specific weights
    M = metrics.target_param_count(32, 4096, 32, 8, 128, 14336, 128256)
    assert 7.9e9 < M < 8.1e9                                   # an 8B-class decoder
    p = metrics.cost_factor(shared, per_pos, 4, M)
    assert 1.0 < p < 1.1
