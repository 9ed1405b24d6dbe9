"""Pins for the oracle's upsampling step (reading R: half-pixel bilinear, edge clamp)."""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).normal(0.0, 1.0, shape).astype(np.float32)


@pytest.mark.parametrize("shape,s", [((3, 7, 9), 8), ((2, 46, 46), 8), ((1, 5, 3), 4), ((1, 2, 2), 8),
                                     ((2, 1, 6), 8), ((2, 6, 1), 8), ((1, 4, 5), 2)])
def test_matches_torch_bilinear(shape, s):
    """Library special case: torch's CPU bilinear interpolation with
    align_corners=False is the same map up to rounding order."""
    lo = _rand(shape, 1)
    ours = oracle.resize(lo, s)
    ref = torch.nn.functional.interpolate(torch.from_numpy(lo)[None], scale_factor=s, mode="bilinear",
                                          align_corners=False)[0].numpy()
    assert ours.shape == ref.shape == (shape[0], s * shape[1], s * shape[2])
    assert np.abs(ours - ref).max() <= 1e-6


def test_matches_scipy_map_coordinates():
    """Second library pin: order-1 spline sampling at (X+1/2)/s - 1/2 with nearest-edge extension."""
    from scipy.ndimage import map_coordinates
    lo = _rand((11, 6), 2)
    s = 8
    Y, X = np.meshgrid(np.arange(11 * s), np.arange(6 * s), indexing="ij")
    ref = map_coordinates(lo.astype(np.float64), [(Y + 0.5) / s - 0.5, (X + 0.5) / s - 0.5], order=1, mode="nearest")
    assert np.abs(oracle.resize(lo, s) - ref).max() <= 1e-6


def test_constant_map_is_exact():
    for c in (0.5, -2.0, 0.05, 1.0 / 3.0):
        lo = np.full((4, 5), c, np.float32)
        hi = oracle.resize(lo, 8)
        if c in (0.5, -2.0):
            assert np.all(hi == np.float32(c))
        else:
            assert np.abs(hi - np.float32(c)).max() <= 1.2e-7 * abs(c)


def test_affine_ramp_closed_form():
    """In the interior a bilinear map reproduces a*x + b*y + c at the half-pixel sample points."""
    h, w, s = 9, 12, 8
    a, b, c = 0.25, -0.5, 3.0
    yy, xx = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    lo = (a * xx + b * yy + c).astype(np.float32)
    hi = oracle.resize(lo, s)
    Y, X = np.meshgrid(np.arange(h * s), np.arange(w * s), indexing="ij")
    want = a * ((X + 0.5) / s - 0.5) + b * ((Y + 0.5) / s - 0.5) + c
    inner = (slice(s // 2, h * s - s // 2), slice(s // 2, w * s - s // 2))
    assert np.abs(hi[inner] - want[inner]).max() <= 1e-6
    # outside the outermost nodes the map is clamped, not extrapolated
    assert np.all(hi[:, 0] == hi[:, 3]) and np.all(hi[0, :] == hi[3, :])


def test_border_plateaus():
    lo = _rand((6, 7), 3)
    hi = oracle.resize(lo, 8)
    for k in range(1, 4):
        assert np.array_equal(hi[0], hi[k])
        assert np.array_equal(hi[:, 0], hi[:, k])
    # the four corner-most pixels equal the corner node itself
    assert hi[0, 0] == lo[0, 0]
    # bottom / right borders are clamped too (up to one rounding of w*v + (1-w)*v)
    assert np.abs(hi[-1] - hi[-4]).max() <= 2e-7 * np.abs(hi[-1]).max()
    assert np.abs(hi[-1, -1] - lo[-1, -1]) <= 1.2e-7 * abs(lo[-1, -1])


def test_axes_are_not_swapped():
    lo = _rand((5, 9), 4)
    a = oracle.resize(lo, 8)
    b = oracle.resize(np.ascontiguousarray(lo.T), 8).T
    assert np.abs(a - b).max() <= 1e-6
    # one impulse lands where its node is: node (i, j) sits at hi-res (8i+3.5, 8j+3.5)
    lo = np.zeros((5, 9), np.float32)
    lo[3, 7] = 1.0
    hi = oracle.resize(lo, 8)
    Y, X = np.unravel_index(np.argmax(hi), hi.shape)
    assert (Y, X) in [(27, 59), (27, 60), (28, 59), (28, 60)]


def test_pointwise_equals_full():
    lo = _rand((6, 5), 5)
    hi = oracle.resize(lo, 8)
    for Y, X in [(0, 0), (3, 4), (17, 22), (47, 39), (20, 0), (0, 31)]:
        assert np.float32(oracle.up(lo, 8, Y, X)) == hi[Y, X]


def test_fp16_storage_widens_exactly():
    lo16 = _rand((2, 6, 5), 6).astype(np.float16)
    assert np.array_equal(oracle.resize(lo16, 8), oracle.resize(lo16.astype(np.float32), 8))


def test_golden_closed_forms():
    """Values worked out by hand from the definition (see the fixture's header)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "resize_closed_forms.txt")) if l.strip() and l[0] != "#"]
    sigma = 7.0
    h = w = 9
    gy, gx = np.meshgrid(8 * np.arange(h) + 3.5, 8 * np.arange(w) + 3.5, indexing="ij")
    lo = np.exp(-((gx - 35.5) ** 2 + (gy - 35.5) ** 2) / (2 * sigma ** 2)).astype(np.float32)  # centred on node (4, 4)
    hi = oracle.resize(lo, 8)
    for name, Y, X, want in rows:
        assert abs(hi[int(Y), int(X)] - float(want)) <= 2e-6, name
