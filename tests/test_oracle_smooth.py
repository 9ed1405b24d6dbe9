"""Pins of the smoothing oracle (oracle/hp_smooth_oracle.c): a library separable correlation, impulse responses,
constants, identity, border replication and separability."""
import numpy as np
import pytest
from scipy import ndimage

import oracle
from synth import gaussian_taps


def test_gaussian_taps_are_a_normalised_sampled_gaussian():
    t = gaussian_taps(3.0, 8)
    assert t.dtype == np.float32 and len(t) == 17 and abs(float(t.astype(np.float64).sum()) - 1) < 1e-6
    assert np.array_equal(t, t[::-1]) and np.all(np.diff(t[:9]) > 0)
    assert abs(t[8] / t[5] - np.exp(9 / 18.0)) < 1e-5          # exp(-0 / 2s^2) / exp(-9 / 2s^2)


@pytest.mark.parametrize("shape,taps", [((3, 37, 53), gaussian_taps(3.0, 8)), ((1, 9, 200), gaussian_taps(1.0, 2)),
                                        ((2, 64, 5), gaussian_taps(2.0, 12)), ((1, 1, 1), gaussian_taps(3.0, 8)),
                                        ((1, 40, 40), np.array([0.25, -0.5, 2.0, 0.125, 0.5], np.float32))])
def test_matches_a_library_separable_correlation(shape, taps):
    rng = np.random.default_rng(1)
    m = rng.random(shape, dtype=np.float32)
    got = oracle.smooth(m, taps)
    want = ndimage.correlate1d(m.astype(np.float64), taps.astype(np.float64), axis=-1, mode="nearest")
    want = ndimage.correlate1d(want, taps.astype(np.float64), axis=-2, mode="nearest")
    assert got.shape == m.shape and np.allclose(got, want, rtol=2e-6, atol=1e-7)


def test_impulse_response_is_the_outer_product_of_the_taps():
    taps = np.array([0.5, 0.25, 0.125, 2.0, 4.0], np.float32)       # asymmetric: an impulse spreads the taps mirrored
    m = np.zeros((21, 23), np.float32)
    m[10, 11] = 1.0
    got = oracle.smooth(m, taps)
    want = np.zeros_like(m)
    want[8:13, 9:14] = np.outer(taps[::-1], taps[::-1])               # products of powers of two: exact
    assert np.array_equal(got, want)


def test_constants_and_identity():
    taps = gaussian_taps(3.0, 8)
    c = np.full((4, 30, 30), 0.75, np.float32)
    assert np.allclose(oracle.smooth(c, taps), 0.75, rtol=0, atol=2e-7)
    m = np.random.default_rng(2).random((2, 17, 19), dtype=np.float32)
    assert np.array_equal(oracle.smooth(m, np.array([1.0], np.float32)), m)
    assert np.array_equal(oracle.smooth(m, np.array([0.0, 1.0, 0.0], np.float32)), m)


def test_borders_repeat_the_edge_pixel_and_axes_are_not_swapped():
    # taps (1, 0, 0) read the pixel to the left / above: a shift by one with the first column / row repeated
    m = np.arange(6 * 8, dtype=np.float32).reshape(6, 8)
    got = oracle.smooth(m, np.array([1.0, 0.0, 0.0], np.float32))
    want = np.pad(m, ((1, 0), (1, 0)), mode="edge")[:-1, :-1]
    assert np.array_equal(got, want)
    got = oracle.smooth(m, np.array([0.0, 0.0, 1.0], np.float32))
    want = np.pad(m, ((0, 1), (0, 1)), mode="edge")[1:, 1:]
    assert np.array_equal(got, want)
    # a row vector smoothed only spreads along x
    row = np.zeros((5, 9), np.float32)
    row[2, :] = 1.0
    out = oracle.smooth(row, np.array([0.25, 0.5, 0.25], np.float32))
    assert np.array_equal(out[:, 4], np.array([0, 0.25, 0.5, 0.25, 0], np.float32))


def test_separable_equals_direct_two_dimensional_sum():
    rng = np.random.default_rng(4)
    taps = rng.random(7).astype(np.float32)
    m = rng.random((12, 14)).astype(np.float32)
    got = oracle.smooth(m, taps)
    pad = np.pad(m.astype(np.float64), 3, mode="edge")
    k2 = np.outer(taps.astype(np.float64), taps.astype(np.float64))
    want = np.array([[np.sum(k2 * pad[y:y + 7, x:x + 7]) for x in range(14)] for y in range(12)])
    assert np.allclose(got, want, rtol=2e-6)
