"""Pins for the oracle's limb scoring (reading S: sampled PAF line integral)."""
import numpy as np
import pytest

import oracle

S, THR, RATIO = 10, 0.05, 0.8


def score(pafx, pafy, A, B, S=S, thr=THR, ratio=RATIO):
    xA, yA = zip(*A)
    xB, yB = zip(*B)
    return oracle.score_limb(pafx, pafy, 8, xA, yA, xB, yB, S, thr, ratio)


def test_need():
    assert oracle.need(0.8, 10) == 8
    assert oracle.need(0.5, 10) == 5
    assert oracle.need(1.0, 10) == 10
    assert oracle.need(0.75, 10) == 8
    assert oracle.need(0.8, 5) == 4


@pytest.mark.parametrize("phi", [0.0, 0.7, 2.1, -1.3, np.pi])
def test_constant_field_is_cosine(phi):
    """Closed form: in a constant field (cos phi, sin phi) every sample projects to
    cos(theta - phi), so the mean does too, whatever the segment."""
    h, w = 20, 26
    pafx = np.full((h, w), np.cos(phi), np.float32)
    pafy = np.full((h, w), np.sin(phi), np.float32)
    rng = np.random.default_rng(3)
    A = [(int(rng.integers(0, 8 * w)), int(rng.integers(0, 8 * h))) for _ in range(6)]
    B = [(int(rng.integers(0, 8 * w)), int(rng.integers(0, 8 * h))) for _ in range(7)]
    ci, cj, cs = score(pafx, pafy, A, B)
    got = {(i, j): s for i, j, s in zip(ci.tolist(), cj.tolist(), cs.tolist())}
    n_acc = 0
    for i, (xa, ya) in enumerate(A):
        for j, (xb, yb) in enumerate(B):
            theta = np.arctan2(yb - ya, xb - xa)
            c = np.cos(theta - phi)
            if abs(c - THR) < 1e-4 or (xa, ya) == (xb, yb):
                continue
            if c > THR:
                assert abs(got[(i, j)] - c) <= 1e-6
                n_acc += 1
            else:
                assert (i, j) not in got
    assert n_acc > 3
    assert list(got) == sorted(got)                      # (i asc, j asc)


def test_straight_limb_band():
    """A wide straight limb: an on-axis pair scores exactly 1 with all samples valid,
    the reversed pair scores -1 and is rejected, a perpendicular pair scores 0."""
    h, w = 24, 30
    pafx = np.zeros((h, w), np.float32)
    pafy = np.zeros((h, w), np.float32)
    pafx[8:16, 4:26] = 1.0                                # nodes y 67.5..123.5, x 35.5..203.5
    A, B = (60, 90), (180, 90)
    ci, cj, cs = score(pafx, pafy, [A], [B])
    assert ci.tolist() == [0] and cj.tolist() == [0] and cs[0] == np.float32(1.0)
    ci, cj, cs = score(pafx, pafy, [B], [A])
    assert len(ci) == 0
    ci, cj, cs = score(pafx, pafy, [(100, 70)], [(100, 120)])
    assert len(ci) == 0


def test_sample_placement_closed_form():
    """pafx = affine ramp in x (reproduced exactly by the upsampling in the interior), so a
    horizontal pair's score is the mean of the ramp at round(xA + k*dx/(S-1)), k = 0..S-1."""
    h, w = 12, 40
    ramp = (np.arange(w, dtype=np.float64) * 8 + 3.5) / 512.0 + 0.25     # value = X/512 + 0.25 at hi-res X
    pafx = np.tile(ramp.astype(np.float32), (h, 1))
    pafy = np.zeros((h, w), np.float32)
    for xa, xb in [(20, 271), (33, 100), (50, 57), (10, 300)]:
        ci, cj, cs = score(pafx, pafy, [(xa, 40)], [(xb, 44 if xb == 57 else 40)])
        ks = np.arange(S)
        sx = np.floor(xa + ks / (S - 1) * (xb - xa) + 0.5)
        dy = 4 if xb == 57 else 0
        ux = (xb - xa) / np.hypot(xb - xa, dy)
        want = np.mean(sx / 512.0 + 0.25) * ux
        assert len(cs) == 1 and abs(cs[0] - want) <= 1e-6
    # end points included: a pair whose samples all coincide with A or B region values
    ci, cj, cs = score(pafx, pafy, [(100, 40)], [(101, 40)])
    sx = np.floor(100 + np.arange(S) / (S - 1) + 0.5)
    assert abs(cs[0] - np.mean(sx / 512.0 + 0.25)) <= 1e-6


def test_valid_sample_rule():
    """Field 1 on the left, 0 on the right: the number of samples in the left part decides."""
    h, w = 10, 40
    pafx = np.zeros((h, w), np.float32)
    pafx[:, :20] = 1.0                                    # nodes up to X = 155.5 are 1, from 163.5 on 0
    pafy = np.zeros((h, w), np.float32)
    # samples at 10 + 18k: k = 0..8 at X <= 154 (value 1), k = 9 at 172 (value 0) -> 9 valid
    ci, cj, cs = score(pafx, pafy, [(10, 40)], [(172, 40)])
    assert len(ci) == 1 and abs(cs[0] - 0.9) <= 1e-6
    # samples at 10 + 27k: k <= 5 valid (145), k = 6 at 172 -> 6 valid < 8 -> rejected though mean > 0
    ci, cj, cs = score(pafx, pafy, [(10, 40)], [(253, 40)])
    assert len(ci) == 0
    # samples at 10 + 21k: k <= 6 at <= 136 valid, k = 7 at 157 (in the ramp 155.5..163.5: 0.8125 > thr) valid,
    # k = 8, 9 zero -> exactly 8 valid -> accepted
    ci, cj, cs = score(pafx, pafy, [(10, 40)], [(199, 40)])
    assert len(ci) == 1 and abs(cs[0] - (7 + 0.8125) / 10) <= 1e-6
    # same geometry but the rule tightened to 9 of 10 -> rejected
    ci, cj, cs = score(pafx, pafy, [(10, 40)], [(199, 40)], ratio=0.9)
    assert len(ci) == 0


def test_negative_mean_and_degenerate_pairs():
    h, w = 10, 10
    pafx = np.full((h, w), 1.0, np.float32)
    pafy = np.zeros((h, w), np.float32)
    ci, cj, cs = score(pafx, pafy, [(30, 30), (50, 30)], [(30, 30), (50, 30), (70, 30)])
    # (0,0) and (1,1) are zero-length; (1,0) points against the field
    assert list(zip(ci.tolist(), cj.tolist())) == [(0, 1), (0, 2), (1, 2)]
    assert np.all(cs == np.float32(1.0))


def test_capacity_reports_required_count():
    import ctypes
    h, w = 10, 10
    pafx = np.full((h, w), 1.0, np.float32)
    pafy = np.zeros((h, w), np.float32)
    xA = np.arange(5, dtype=np.int32); yA = np.full(5, 20, np.int32)
    xB = np.arange(40, 46, dtype=np.int32); yB = np.full(6, 20, np.int32)
    full = oracle.score_limb(pafx, pafy, 8, xA, yA, xB, yB, 10, 0.05, 0.8)
    assert len(full[0]) == 30
    ci = np.empty(4, np.int32); cj = np.empty(4, np.int32); cs = np.empty(4, np.float32)
    f32 = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
    i32 = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    n = oracle.lib().hpo_score_limb(f32(pafx), f32(pafy), h, w, 8, 5, i32(xA), i32(yA), 6, i32(xB), i32(yB),
                                    10, 0.05, 8, 4, i32(ci), i32(cj), f32(cs))
    assert n == 30 and ci.tolist() == [0, 0, 0, 0] and cj.tolist() == [0, 1, 2, 3]
