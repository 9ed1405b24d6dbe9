"""Pins for the oracle's pre-processing operator (readings Q1-Q4: 8-bit interleaved image ->
half-pixel bilinear resize -> channel-first fp32 with a scale and an offset per channel)."""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _images(shape, seed):
    return np.random.default_rng(seed).integers(0, 256, size=shape, dtype=np.uint8)


@pytest.mark.parametrize("src,dst", [((2, 9, 13, 3), (11, 16)), ((1, 36, 64, 3), (46, 82)), ((1, 20, 30, 3), (7, 9)),
                                     ((1, 1, 5, 3), (4, 4)), ((2, 6, 1, 1), (3, 5)), ((1, 17, 23, 4), (17, 23))])
def test_matches_torch_bilinear(src, dst):
    """Library special case: torch's CPU bilinear interpolation (align_corners=False, no
    antialiasing) of the same values, in fp64, is the same map up to rounding."""
    im = _images(src, 3)
    ours = oracle.preprocess(im, dst[0], dst[1], 1.0, 0.0)
    ref = torch.nn.functional.interpolate(torch.from_numpy(im).permute(0, 3, 1, 2).double(), size=dst, mode="bilinear",
                                          align_corners=False, antialias=False).numpy()
    assert ours.shape == ref.shape
    assert np.abs(ours - ref).max() <= 255 * 4e-7


def test_hand_derived_rows():
    rows = 0
    with open(os.path.join(GOLDEN, "preprocess_closed_forms.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            dims, src, want = line.split("|")
            ws, wd = (int(v) for v in dims.split())
            src = np.array(src.split(), np.uint8)
            want = np.array(want.split(), np.float64)
            assert len(src) == ws and len(want) == wd
            got = oracle.preprocess(src.reshape(1, 1, ws, 1), 1, wd, 1.0, 0.0)[0, 0, 0]
            assert np.abs(got - want).max() <= 1e-5, line
            # the same row used as a column
            got = oracle.preprocess(src.reshape(1, ws, 1, 1), wd, 1, 1.0, 0.0)[0, 0, :, 0]
            assert np.abs(got - want).max() <= 1e-5, line
            rows += 1
    assert rows == 5


def test_identity_size_is_an_exact_copy_in_channel_first_layout():
    im = _images((2, 12, 19, 3), 5)
    out = oracle.preprocess(im, 12, 19, 1.0, 0.0)
    assert np.array_equal(out, im.transpose(0, 3, 1, 2).astype(np.float32))


def test_layout_and_channel_order():
    """Per-channel constants come back as constant planes (to rounding: the two weights of a
    cell need not add up to exactly one), in order or reversed."""
    im = np.empty((1, 5, 7, 3), np.uint8)
    im[..., 0], im[..., 1], im[..., 2] = 10, 20, 30
    out = oracle.preprocess(im, 9, 4, 1.0, 0.0)
    assert out.shape == (1, 3, 9, 4)
    for c, v in enumerate((10, 20, 30)):
        assert np.abs(out[0, c] - v).max() <= 2e-6 * v
    rev = oracle.preprocess(im, 9, 4, 1.0, 0.0, reverse_channels=True)
    for c, v in enumerate((30, 20, 10)):
        assert np.abs(rev[0, c] - v).max() <= 2e-6 * v


def test_scale_and_offset_per_channel():
    im = _images((1, 8, 8, 3), 6)
    alpha = np.array([1 / 255.0, 0.5, 2.0], np.float32)
    beta = np.array([-0.5, 3.0, 0.0], np.float32)
    raw = oracle.preprocess(im, 5, 11, 1.0, 0.0).astype(np.float64)
    out = oracle.preprocess(im, 5, 11, alpha, beta)
    want = raw * alpha.astype(np.float64)[None, :, None, None] + beta.astype(np.float64)[None, :, None, None]
    assert np.abs(out - want).max() <= 1e-5
    assert not np.allclose(out[0, 0], out[0, 1])
    # with the colour order reversed, scale and offset still go with the OUTPUT channel
    const = np.empty((1, 4, 4, 3), np.uint8)
    const[..., 0], const[..., 1], const[..., 2] = 10, 20, 30
    rev = oracle.preprocess(const, 4, 4, np.float32([1.0, 2.0, 4.0]), np.float32([0.5, 0.25, 0.125]), reverse_channels=True)
    assert rev[0, :, 0, 0].tolist() == [30.5, 40.25, 40.125]


@pytest.mark.parametrize("hs,ws,hd,wd", [(10, 14, 25, 31), (30, 40, 12, 17)])
def test_affine_ramp_in_closed_form(hs, ws, hd, wd):
    """v = a x + b y + c sampled at (X + 1/2) Ws / Wd - 1/2 (bilinear interpolation reproduces
    affine functions); checked where the sample lies between the outermost nodes."""
    a, b, c = 3, 2, 5
    y, x = np.meshgrid(np.arange(hs), np.arange(ws), indexing="ij")
    im = (a * x + b * y + c).astype(np.uint8).reshape(1, hs, ws, 1)
    assert im.max() < 255
    out = oracle.preprocess(im, hd, wd, 1.0, 0.0)[0, 0]
    sx = (np.arange(wd) + 0.5) * ws / wd - 0.5
    sy = (np.arange(hd) + 0.5) * hs / hd - 0.5
    inside = np.outer((sy >= 0) & (sy <= hs - 1), (sx >= 0) & (sx <= ws - 1))
    want = a * sx[None, :] + b * sy[:, None] + c
    assert inside.sum() > 0.7 * hd * wd
    assert np.abs(out - want)[inside].max() <= 1e-4
    # outside, the clamp replicates the border
    assert np.all(np.abs(out[:, 0] - (a * max(sx[0], 0) + b * np.clip(sy, 0, hs - 1) + c)) <= 1e-4)


def test_values_stay_within_the_source_range():
    im = _images((1, 13, 9, 3), 8)
    out = oracle.preprocess(im, 40, 33, 1.0, 0.0)
    assert out.min() >= im.min() - 1e-4 and out.max() <= im.max() + 1e-4
