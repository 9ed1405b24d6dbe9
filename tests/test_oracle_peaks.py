"""Pins for the oracle's peak step (reading P: thresholded 3x3 maximum, raster-first tie-break)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st
from scipy.ndimage import maximum_filter

import oracle


def brute_peaks(u, thr):
    """Independent formulation: a pixel is a peak iff it exceeds thr and the pair
    (value, -raster index) is the strict lexicographic maximum of its in-bounds 3x3 window."""
    H, W = u.shape
    out = []
    for y in range(H):
        for x in range(W):
            if not u[y, x] > thr:
                continue
            me = (float(u[y, x]), -(y * W + x))
            best = max((float(u[yy, xx]), -(yy * W + xx))
                       for yy in range(max(y - 1, 0), min(y + 2, H))
                       for xx in range(max(x - 1, 0), min(x + 2, W)))
            if best == me:
                out.append((x, y))
    return out


def as_list(res):
    return list(zip(res[0].tolist(), res[1].tolist()))


@settings(max_examples=150, deadline=None)
@given(st.integers(1, 12), st.integers(1, 12), st.integers(0, 2 ** 31 - 1), st.sampled_from([2, 4, 1000]))
def test_brute_force_tiny_maps(H, W, seed, levels):
    rng = np.random.default_rng(seed)
    # few quantisation levels -> many exact ties and plateaus
    u = (rng.integers(0, levels, (H, W)) / levels).astype(np.float32)
    res = oracle.find_peaks(u, 0.3)
    assert as_list(res) == brute_peaks(u, 0.3)
    assert np.array_equal(res[2], u[res[1], res[0]])


def test_matches_maximum_filter_without_ties():
    """Library pin: with distinct values a peak is a pixel equal to its 3x3 maximum filter."""
    rng = np.random.default_rng(7)
    u = rng.permutation(40 * 53).reshape(40, 53).astype(np.float32) / (40 * 53)
    mf = maximum_filter(u, size=3, mode="constant", cval=-np.inf)
    ys, xs = np.nonzero((u == mf) & (u > 0.5))
    res = oracle.find_peaks(u, 0.5)
    assert as_list(res) == list(zip(xs.tolist(), ys.tolist()))     # np.nonzero is raster order


def test_plateaus_and_borders():
    u = np.full((5, 6), 0.7, np.float32)
    assert as_list(oracle.find_peaks(u, 0.05)) == [(0, 0)]          # one plateau -> its raster-first pixel
    assert as_list(oracle.find_peaks(u, 0.7)) == []                  # threshold is strict
    u = np.zeros((6, 6), np.float32)
    u[5, 5] = 1.0                                                    # corner pixel, 3 in-bounds neighbours
    u[0, 3] = 0.5
    u[2, 2] = u[2, 3] = u[3, 2] = u[3, 3] = 0.9                      # 2x2 plateau
    assert as_list(oracle.find_peaks(u, 0.05)) == [(3, 0), (2, 2), (5, 5)]


def test_never_adjacent_and_monotone_in_threshold():
    rng = np.random.default_rng(11)
    u = (rng.integers(0, 6, (64, 80)) / 6).astype(np.float32)
    lo = as_list(oracle.find_peaks(u, 0.1))
    hi = as_list(oracle.find_peaks(u, 0.6))
    assert set(hi) <= set(lo) and len(hi) < len(lo)
    pts = np.array(lo)
    d = np.abs(pts[:, None, :] - pts[None, :, :]).max(axis=2)
    np.fill_diagonal(d, 9)
    assert d.min() >= 2
    keys = [y * 80 + x for x, y in lo]
    assert keys == sorted(keys)


def test_single_gaussian_through_resize():
    gy, gx = np.meshgrid(8 * np.arange(20) + 3.5, 8 * np.arange(24) + 3.5, indexing="ij")
    for cx, cy in [(75.5, 83.5), (70.2, 91.9), (100.0, 60.0)]:
        lo = np.exp(-((gx - cx) ** 2 + (gy - cy) ** 2) / 98.0).astype(np.float32)
        x, y, s = oracle.find_peaks(oracle.resize(lo, 8), 0.05)
        assert len(x) == 1
        assert abs(x[0] - cx) <= 4.5 and abs(y[0] - cy) <= 4.5
    # node-centred: exact 2x2 plateau, the top-left pixel wins
    lo = np.exp(-((gx - 75.5) ** 2 + (gy - 83.5) ** 2) / 98.0).astype(np.float32)
    x, y, s = oracle.find_peaks(oracle.resize(lo, 8), 0.05)
    assert (x[0], y[0]) == (75, 83) and abs(s[0] - 0.94095458) < 2e-6


def test_capacity_reports_required_count():
    rng = np.random.default_rng(5)
    u = rng.random((30, 30)).astype(np.float32)
    full = oracle.find_peaks(u, 0.2)
    n = len(full[0])
    assert n > 8
    import ctypes
    px = np.empty(8, np.int32); py = np.empty(8, np.int32); ps = np.empty(8, np.float32)
    got = oracle.lib().hpo_find_peaks(u.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), 30, 30, 0.2, 8,
                                      px.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                      py.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                      ps.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    assert got == n and np.array_equal(px, full[0][:8]) and np.array_equal(py, full[1][:8])
