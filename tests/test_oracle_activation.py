"""Pins for the reference's batch-norm based activation range (Section 4 set-up).  The paper
names the approach only; the closed form below is the reading this library takes."""
import numpy as np
import pytest

import oracle


def closed_form(gamma, beta, n_sigma, relu, bits):
    g, b, n = gamma.astype(np.float32), beta.astype(np.float32), np.float32(n_sigma)
    t = n * np.abs(g)
    lo, hi = (b - t).min(), (b + t).max()
    if relu:
        lo, hi = max(lo, np.float32(0)), max(hi, np.float32(0))
    lo, hi = np.float32(lo) + np.float32(0), np.float32(hi) + np.float32(0)
    q = np.float32((1 << bits) - 1)
    span = np.float32(hi - lo)
    scale = np.float32(span / q) if span > 0 else np.float32(1)
    z = int(np.clip(np.rint(np.float32(-lo) / scale), 0, q))
    return lo, hi, scale, z


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("bits", [2, 4, 8, 16])
@pytest.mark.parametrize("channels", [1, 7, 64, 2048])
def test_matches_numpy_closed_form(channels, bits, relu):
    rng = np.random.default_rng(channels * 31 + bits)
    gamma = (rng.standard_normal(channels) * 0.7 + 1.0).astype(np.float32)
    beta = (rng.standard_normal(channels) * 0.4).astype(np.float32)
    for n_sigma in (0.0, 3.0, 6.0):
        got = oracle.activation_range(gamma, beta, n_sigma, relu, bits)
        want = closed_form(gamma, beta, n_sigma, relu, bits)
        assert np.float32(got[0]).tobytes() == np.float32(want[0]).tobytes()
        assert np.float32(got[1]).tobytes() == np.float32(want[1]).tobytes()
        assert np.float32(got[2]).tobytes() == np.float32(want[2]).tobytes()
        assert got[3] == want[3]


def test_hand_worked_example():
    # channels: 0.1 -/+ 6, -0.3 -/+ 3, 0.2 -/+ 12  ->  [-11.8, 12.2]; 8 bit: step 24/255, zero at 125
    g = np.array([1.0, 0.5, 2.0], np.float32)
    b = np.array([0.1, -0.3, 0.2], np.float32)
    lo, hi, scale, z = oracle.activation_range(g, b, 6.0, False, 8)
    assert lo == np.float32(-11.8) and hi == np.float32(12.2)
    assert abs(float(scale) - 24.0 / 255.0) < 1e-6 and z == 125
    lo, hi, scale, z = oracle.activation_range(g, b, 6.0, True, 8)       # ReLU: from 0
    assert lo == 0 and hi == np.float32(12.2) and z == 0
    assert abs(float(scale) - 12.2 / 255.0) < 1e-6


def test_properties():
    rng = np.random.default_rng(9)
    g = rng.standard_normal(300).astype(np.float32)
    b = rng.standard_normal(300).astype(np.float32)
    lo0, hi0, _, _ = oracle.activation_range(g, b, 0.0, False, 8)
    assert lo0 == b.min() and hi0 == b.max()                             # no spread: the biases
    prev = (lo0, hi0)
    for n in (1.0, 2.0, 6.0):                                            # wider with n_sigma
        lo, hi, scale, z = oracle.activation_range(g, b, n, False, 8)
        assert lo <= prev[0] and hi >= prev[1]
        prev = (lo, hi)
        assert 0 <= z <= 255
        assert abs(z * float(scale) + float(lo)) <= float(scale)          # code z sits on 0
    a = oracle.activation_range(g, b, 6.0, False, 8)
    assert a == oracle.activation_range(-g, b, 6.0, False, 8)            # the sign of gamma is immaterial
    # all-negative outputs under a ReLU: the empty range [0, 0]
    lo, hi, scale, z = oracle.activation_range(np.zeros(4, np.float32), np.full(4, -1, np.float32), 6.0, True, 8)
    assert (lo, hi, scale, z) == (0.0, 0.0, 1.0, 0)
    assert np.signbit(np.float32(lo)) == False                           # +0, not -0


def test_bad_arguments():
    g = np.ones(3, np.float32)
    with pytest.raises(ValueError):
        oracle.activation_range(g, g, 6.0, False, 1)
    with pytest.raises(ValueError):
        oracle.activation_range(g, g, 6.0, False, 17)
