"""Pins for the oracle's GELU and its derivative (the activation whose input Sec. 4 caches in 4 bits) -- CPU only."""
import numpy as np
from scipy import stats

from oracle import ref


def test_textbook_values():
    x = np.array([0.0, 1.0, -1.0, 2.0, -2.0, 0.5, 10.0, -10.0, 40.0, -40.0], dtype=np.float32)
    y = ref.gelu(x)
    # x * Phi(x) with the standard normal CDF to 16 digits
    phi = {1.0: 0.8413447460685429, 2.0: 0.9772498680518208, 0.5: 0.6914624612740131}
    want = [0.0, phi[1.0], -(1 - phi[1.0]), 2 * phi[2.0], -2 * (1 - phi[2.0]), 0.5 * phi[0.5], 10.0, 0.0, 40.0, 0.0]
    np.testing.assert_allclose(y[:7], np.float32(want[:7]), rtol=1e-7, atol=0)
    assert abs(float(y[7])) < 1e-20 and y[8] == 40.0 and y[9] == 0.0
    assert y[0] == 0.0


def test_against_library_normal_cdf_and_reflection_identity():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(20000) * 3).astype(np.float32)
    y = ref.gelu(x).astype(np.float64)
    want = x.astype(np.float64) * stats.norm.cdf(x.astype(np.float64))
    np.testing.assert_allclose(y, want, rtol=1.2e-7, atol=1e-45)          # one rounding to fp32
    ym = ref.gelu(-x).astype(np.float64)
    np.testing.assert_allclose(y - ym, x.astype(np.float64), rtol=3e-7, atol=1e-7)     # GELU(x) - GELU(-x) = x


def test_minimum_and_monotone_right_branch():
    x = np.linspace(-6, 6, 24001).astype(np.float32)
    y = ref.gelu(x)
    i = int(np.argmin(y))
    assert abs(float(x[i]) + 0.7517916) < 1e-3 and abs(float(y[i]) + 0.16997121) < 1e-6
    assert np.all(np.diff(y[i:].astype(np.float64)) >= 0)


def test_derivative_matches_numerical_differentiation():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(5000) * 2.5).astype(np.float32)
    ones = np.ones_like(x)
    g = ref.gelu_backward(x, ones).astype(np.float64)
    xd = x.astype(np.float64)
    h = 1e-5
    f = lambda t: t * stats.norm.cdf(t)
    num = (f(xd + h) - f(xd - h)) / (2 * h)
    np.testing.assert_allclose(g, num, rtol=0, atol=5e-7)
    assert ref.gelu_backward(np.zeros(1, np.float32), np.ones(1, np.float32))[0] == 0.5
    big = ref.gelu_backward(np.array([30.0, -30.0], np.float32), np.ones(2, np.float32))
    assert big[0] == 1.0 and abs(float(big[1])) < 1e-30


def test_backward_is_linear_in_dy_and_handles_bf16():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(4096).astype(np.float32)
    dy = rng.standard_normal(4096).astype(np.float32)
    g1 = ref.gelu_backward(x, np.ones_like(dy)).astype(np.float64)
    g = ref.gelu_backward(x, dy).astype(np.float64)
    np.testing.assert_allclose(g, dy.astype(np.float64) * g1, rtol=3e-7, atol=1e-38)
    # bf16 in / out: widened exactly, one rounding to bf16
    dyb = (dy.view(np.uint32) >> 16).astype(np.uint16)
    gb = ref.gelu_backward(x, dyb)
    dyw = (dyb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    exact = dyw * g1
    got = (gb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.all(np.abs(got - exact) <= np.abs(exact) * 2.0 ** -8 + 1e-38)
    yb = ref.gelu((x.view(np.uint32) >> 16).astype(np.uint16))
    xw = ((x.view(np.uint32) >> 16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    yw = (yb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.all(np.abs(yw - xw * stats.norm.cdf(xw)) <= np.abs(xw * stats.norm.cdf(xw)) * 2.0 ** -8 + 1e-38)
