"""Pins for the oracle's elementwise / linear primitives: closed forms, invariants and special
cases that reduce to a numpy / torch library routine.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import sfo


def test_round_bf16_known_values():
    # bf16 keeps 8 significant bits: spacing 2^-7 at 1.0; ties go to the even mantissa
    assert sfo.round_bf16(1.0) == 1.0
    assert sfo.round_bf16(1.0 + 2.0 ** -8) == 1.0                      # tie -> even (mantissa 0)
    assert sfo.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6      # tie -> even (mantissa 2)
    assert sfo.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert sfo.round_bf16(-0.3) == -sfo.round_bf16(0.3)
    assert sfo.round_bf16(0.0) == 0.0


def test_round_bf16_matches_torch_cast():
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32) * 3.0
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(sfo.round_bf16(x), want)


def test_rmsnorm_constant_input_closed_form():
    d, c, eps = 64, 3.0, 1e-6
    g = np.linspace(0.5, 1.5, d).astype(np.float32)
    y = sfo.rmsnorm(np.full((2, d), c), g, eps)
    np.testing.assert_allclose(y, np.broadcast_to(g.astype(np.float64) * c / math.sqrt(c * c + eps), (2, d)), rtol=1e-14)


def test_rmsnorm_matches_definition_and_scale_invariance():
    rs = np.random.default_rng(1)
    x = rs.standard_normal((5, 48))
    g = rs.standard_normal(48).astype(np.float32)
    want = g * x / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6)
    np.testing.assert_allclose(sfo.rmsnorm(x, g, 1e-6), want, rtol=1e-13)
    np.testing.assert_allclose(sfo.rmsnorm(7.0 * x, g, 0.0), sfo.rmsnorm(x, g, 0.0), rtol=1e-13)
    # unit gains: every output row has RMS 1 (eps -> 0)
    y = sfo.rmsnorm(x, np.ones(48, np.float32), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(-1)), 1.0, rtol=1e-13)
    # library routine
    t = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g).double(), 1e-6)
    np.testing.assert_allclose(sfo.rmsnorm(x, g, 1e-6), t.numpy(), rtol=1e-12)


def test_group_rmsnorm_is_four_independent_norms():
    rs = np.random.default_rng(2)
    x = rs.standard_normal((3, 4, 32)) * np.array([1.0, 10.0, 0.1, 5.0])[None, :, None]
    g = rs.standard_normal((4, 32)).astype(np.float32)
    y = sfo.group_rmsnorm(x, g, 1e-6)
    for s in range(4):
        np.testing.assert_allclose(y[:, s], sfo.rmsnorm(x[:, s], g[s], 1e-6), rtol=1e-14)
    # a slice's scale does not leak into another slice: group statistics are per slice
    x2 = x.copy(); x2[:, 1] *= 100.0
    y2 = sfo.group_rmsnorm(x2, g, 1e-6)
    np.testing.assert_array_equal(y2[:, [0, 2, 3]], y[:, [0, 2, 3]])
    # identical groups with identical gains == RMSNorm tiled; gains of one (the paper's init)
    xi = np.repeat(rs.standard_normal((3, 1, 32)), 4, axis=1)
    yi = sfo.group_rmsnorm(xi, np.ones((4, 32), np.float32), 1e-6)
    for s in range(4):
        np.testing.assert_array_equal(yi[:, s], yi[:, 0])
    np.testing.assert_allclose(yi[:, 0], sfo.rmsnorm(xi[:, 0], np.ones(32, np.float32)), rtol=1e-14)


def test_linear_matches_matmul_and_onehot():
    rs = np.random.default_rng(3)
    x = rs.standard_normal((7, 33))
    w = rs.standard_normal((19, 33)).astype(np.float32)
    b = rs.standard_normal(19).astype(np.float32)
    np.testing.assert_allclose(sfo.linear(x, w), x @ w.astype(np.float64).T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sfo.linear(x, w, b), x @ w.astype(np.float64).T + b, rtol=1e-12, atol=1e-12)
    # one-hot rows select input features: w is [out, in]
    sel = np.zeros((3, 33), np.float32); sel[0, 5] = 1; sel[1, 0] = 1; sel[2, 32] = 1
    np.testing.assert_array_equal(sfo.linear(x, sel), x[:, [5, 0, 32]])
    # non-square identity catches a transposed operand
    eye = np.eye(33, dtype=np.float32)[:10]
    np.testing.assert_array_equal(sfo.linear(x, eye), x[:, :10])


def test_rope_closed_forms():
    rs = np.random.default_rng(4)
    M, H, hd, theta = 6, 3, 16, 10000.0
    x = rs.standard_normal((M, H, hd))
    pos = np.array([0, 1, 2, 17, 100, 4000], np.int32)
    y = sfo.rope(x, pos, theta)
    np.testing.assert_array_equal(y[0], x[0])                                  # position 0 = identity
    np.testing.assert_allclose((y * y).sum(-1), (x * x).sum(-1), rtol=1e-12)   # rotation: norm kept
    # complex form: (x_i + j x_{i+hd/2}) * exp(j * pos * theta^(-2i/hd))
    half = hd // 2
    z = x[..., :half] + 1j * x[..., half:]
    ang = pos[:, None, None] * theta ** (-2.0 * np.arange(half) / hd)[None, None, :]
    zr = z * np.exp(1j * ang)
    np.testing.assert_allclose(y[..., :half], zr.real, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(y[..., half:], zr.imag, rtol=1e-10, atol=1e-12)
    # hd = 2: a single plane rotated by exactly `pos` radians
    v = sfo.rope(np.array([[[1.0, 0.0]]]), np.array([3], np.int32), theta)
    np.testing.assert_allclose(v[0, 0], [math.cos(3.0), math.sin(3.0)], rtol=1e-14)


def test_rope_scores_depend_on_relative_position_only():
    rs = np.random.default_rng(5)
    q = rs.standard_normal((1, 1, 32)); k = rs.standard_normal((1, 1, 32))
    def score(m, n):
        return float((sfo.rope(q, np.array([m], np.int32)) * sfo.rope(k, np.array([n], np.int32))).sum())
    assert score(10, 3) == pytest.approx(score(107, 100), rel=1e-10)
    assert score(10, 3) != pytest.approx(score(10, 4), rel=1e-6)


def test_silu_mul():
    g = np.array([0.0, 1.0, -1.0, 20.0, -20.0]); u = np.array([5.0, 2.0, 2.0, 1.0, 1.0])
    y = sfo.silu_mul(g, u)
    assert y[0] == 0.0                                             # silu(0) = 0: closed gate
    assert y[1] == pytest.approx(2.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    assert y[2] == pytest.approx(-2.0 / (1.0 + math.e), rel=1e-15)
    assert y[3] == pytest.approx(20.0, rel=1e-8) and abs(y[4]) < 1e-7
    rs = np.random.default_rng(6)
    g, u = rs.standard_normal(100), rs.standard_normal(100)
    want = (torch.nn.functional.silu(torch.from_numpy(g)) * torch.from_numpy(u)).numpy()
    np.testing.assert_allclose(sfo.silu_mul(g, u), want, rtol=1e-13)


def test_argmax_ties_and_nan():
    assert sfo.argmax(np.array([1.0, 3.0, 3.0, 2.0])) == 1          # lowest index among maxima
    assert sfo.argmax(np.array([np.nan, 1.0, np.nan, 1.0])) == 1    # NaN never wins
    assert sfo.argmax(np.array([-np.inf, -np.inf])) == 0
    assert sfo.argmax(np.array([-5.0, -2.0, -9.0])) == 1


# ---- the norm + linear pair, exact and as a bf16 pipeline computes it ---------------------------------
def _bf16(a):
    """bf16 rounding through torch's cast (an implementation other than the oracle's)."""
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def test_norm_linear_exact_mode_is_norm_then_linear():
    rs = np.random.default_rng(3)
    x = rs.standard_normal((5, 24)); g = rs.uniform(0.5, 1.5, 24).astype(np.float32)
    w = rs.standard_normal((7, 24)).astype(np.float32)
    want = (x / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6) * g) @ w.astype(np.float64).T
    np.testing.assert_allclose(sfo.norm_linear(x, g, w), want, rtol=1e-12, atol=1e-12)


def test_norm_linear_bf16_mode_rounding_points():
    """round_bf16 mode: the gains are folded into the weight (w*g rounded to bf16 once), the product
    runs on the bf16 copy of the raw row, the row factor comes from that same copy and is applied
    unrounded.  Pinned against a numpy composition with torch's bf16 cast."""
    rs = np.random.default_rng(4)
    M, K, N = 6, 40, 9
    x = rs.standard_normal((M, K)) * 3.0                       # fp32-like values, not bf16-representable
    w = _bf16(rs.standard_normal((N, K)) * 0.05).astype(np.float32)
    for g in (np.ones(K, np.float32), _bf16(rs.uniform(0.25, 2.0, K)).astype(np.float32)):
        rinv = 1.0 / np.sqrt((_bf16(x) ** 2).mean(-1, keepdims=True) + 1e-6)
        want = (_bf16(x) @ _bf16(w.astype(np.float64) * g).T) * rinv
        got = sfo.norm_linear(x, g, w, round_bf16=True)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    # unit gains and bf16-valued rows: the emulation rounds nothing at all -> equals the exact mode
    xb = _bf16(x)
    np.testing.assert_allclose(sfo.norm_linear(xb, np.ones(K, np.float32), w, round_bf16=True),
                               sfo.norm_linear(xb, np.ones(K, np.float32), w), rtol=1e-12, atol=1e-13)


def test_norm_linear_bf16_mode_stays_within_the_rounding_bound_of_exact():
    """Each product x_k * (w g)_k is perturbed by two bf16 roundings (unit roundoff u = 2^-8) and the
    row factor, a function of sum x_k^2 with every term within (1 +- u)^2, by at most a factor
    (1 + u), so |y_rb - y_exact| <= ((1+u)^3 - 1) * rinv * sum_k |x_k w_k g_k|, element by element."""
    rs = np.random.default_rng(5)
    M, K, N = 8, 96, 12
    x = rs.standard_normal((M, K)) * 0.7
    g = rs.uniform(0.25, 2.0, K).astype(np.float32)
    w = (rs.standard_normal((N, K)) * 0.05).astype(np.float32)
    exact = sfo.norm_linear(x, g, w)
    got = sfo.norm_linear(x, g, w, round_bf16=True)
    u = 2.0 ** -8
    rinv = 1.0 / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6)
    bound = ((1 + u) ** 3 - 1) * (np.abs(x) @ np.abs(w.astype(np.float64) * g).T) * rinv
    assert np.all(np.abs(got - exact) <= bound * (1 + 1e-9))
    assert np.abs(got - exact).max() > 0                       # and the rounding really happens
