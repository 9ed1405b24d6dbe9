"""Pins of the sub-pixel refinement oracle (oracle/hp_refine_oracle.c)."""
import numpy as np
import pytest

import oracle


def test_parabola_vertex_is_recovered():
    # u = 5 - 0.3 (x - x*)^2 - 0.2 (y - y*)^2 sampled on the grid: the parabola through three samples is u itself
    rng = np.random.default_rng(0)
    for _ in range(50):
        xs, ys = rng.uniform(3.6, 8.4), rng.uniform(3.6, 8.4)
        yy, xx = np.mgrid[0:12, 0:12].astype(np.float64)
        u = (5 - 0.3 * (xx - xs) ** 2 - 0.2 * (yy - ys) ** 2).astype(np.float32)
        px, py = int(round(xs)), int(round(ys))
        xf, yf = oracle.refine_peaks(u, [px], [py])
        assert abs(xf[0] - xs) < 2e-5 and abs(yf[0] - ys) < 2e-5


def test_hand_values_symmetry_plateaus_and_borders():
    u = np.zeros((5, 7), np.float32)
    u[2, 2:5] = [1.0, 3.0, 2.0]          # a=1, b=3, c=2: den = 3 - 6 = -3, off = 0.5 * (1 - 2) / -3 = 1/6
    u[1, 3], u[3, 3] = 2.0, 2.0          # symmetric above and below: no vertical offset
    xf, yf = oracle.refine_peaks(u, [3], [2])
    assert xf[0] == np.float32(3) + np.float32(0.5 * -1.0) / np.float32(-3.0) and yf[0] == 2.0
    flat = np.full((4, 4), 0.5, np.float32)                     # den = 0: a plateau stays where it is
    xf, yf = oracle.refine_peaks(flat, [1, 2], [1, 2])
    assert xf.tolist() == [1.0, 2.0] and yf.tolist() == [1.0, 2.0]
    ramp = np.tile(np.arange(6, dtype=np.float32), (6, 1))     # first / last column and row: no neighbours, no offset
    xf, yf = oracle.refine_peaks(ramp, [0, 5, 3], [0, 5, 0])
    assert xf.tolist() == [0.0, 5.0, 3.0] and yf.tolist() == [0.0, 5.0, 0.0]
    valley = np.array([[4, 1, 3]], np.float32).repeat(3, axis=0)   # den = 5 > 0: not a maximum of the parabola
    assert oracle.refine_peaks(valley, [1], [1])[0][0] == 1.0


def test_offsets_stay_within_half_a_pixel_and_follow_the_larger_neighbour():
    rng = np.random.default_rng(1)
    u = rng.random((40, 40)).astype(np.float32)
    ys, xs = np.mgrid[1:39, 1:39]
    xf, yf = oracle.refine_peaks(u, xs.ravel(), ys.ravel())
    assert np.all(np.abs(xf - xs.ravel()) <= 0.5) and np.all(np.abs(yf - ys.ravel()) <= 0.5)
    a, b, c = u[ys, xs - 1].ravel(), u[ys, xs].ravel(), u[ys, xs + 1].ravel()
    peak = (b > a) & (b > c)
    assert np.all(np.sign(xf - xs.ravel())[peak] == np.sign(c - a)[peak])


@pytest.mark.parametrize("sigma", [2.0, 3.0, 5.0])
def test_gaussian_centre_within_the_interpolation_error(sigma):
    # for a Gaussian sampled at x* + {-1, 0, 1} - d the parabola's vertex misses the centre by less than
    # d (1 - d^2) / (6 sigma^2) ... bounded here by 0.02 px for sigma >= 2
    rng = np.random.default_rng(2)
    for _ in range(30):
        xs, ys = rng.uniform(10, 20), rng.uniform(10, 20)
        yy, xx = np.mgrid[0:32, 0:32].astype(np.float64)
        u = np.exp(-((xx - xs) ** 2 + (yy - ys) ** 2) / (2 * sigma * sigma)).astype(np.float32)
        xf, yf = oracle.refine_peaks(u, [int(round(xs))], [int(round(ys))])
        assert abs(xf[0] - xs) < 0.02 and abs(yf[0] - ys) < 0.02
        assert abs(xf[0] - xs) <= abs(round(xs) - xs) + 1e-6     # never worse than the whole pixel
