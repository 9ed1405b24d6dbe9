"""Pins of the drawing oracle (oracle/hp_draw_oracle.c) to facts outside itself: lattice-point counts, hand-counted
hairlines, capsule areas in closed form, a float64 distance computation, symmetries, and a whole scene drawn by an
independent numpy painter."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "draw_closed_forms.txt")


def golden(kind):
    rows = []
    for line in open(GOLDEN):
        f = line.split()
        if f and f[0] == kind:
            rows.append([int(v) for v in f[1:]])
    assert rows
    return rows


def test_discs_are_gauss_circle_counts():
    for r, want in golden("disc"):
        got = sum(oracle.in_disc(x, y, 3, -2, r) for x in range(-15, 20) for y in range(-20, 15))
        assert got == want, r


def test_hairlines_counted_by_hand():
    for ax, ay, bx, by, want in golden("hairline"):
        got = sum(oracle.in_capsule(x, y, ax, ay, bx, by, 1) for x in range(-3, 14) for y in range(-3, 14))
        assert got == want, (ax, ay, bx, by)


def test_capsule_area_in_closed_form():
    for n, t, want in golden("capsule"):
        for (ax, ay, bx, by) in ((0, 0, n, 0), (n, 0, 0, 0), (0, 0, 0, n), (4, n + 2, 4, 2)):
            got = sum(oracle.in_capsule(x, y, ax, ay, bx, by, t) for x in range(-12, 30) for y in range(-12, 30))
            assert got == want, (n, t, ax, ay, bx, by)
    # odd thickness t = 2r + 1: the band is still 2r + 1 high, the caps are the points with 4 (x^2 + y^2) <= t^2
    for n, t in ((5, 1), (6, 3), (9, 5), (4, 7)):
        r = t // 2
        caps = sum(4 * (x * x + y * y) <= t * t for x in range(-9, 10) for y in range(-9, 10))
        got = sum(oracle.in_capsule(x, y, 0, 0, n, 0, t) for x in range(-12, 30) for y in range(-12, 12))
        assert got == n * (2 * r + 1) + caps


def test_against_float64_distances():
    rng = np.random.default_rng(5)
    checked = 0
    for _ in range(400):
        ax, ay, bx, by = rng.integers(-40, 40, 4)
        t = int(rng.integers(1, 14))
        P = rng.integers(-50, 50, (60, 2))
        a, b = np.array([ax, ay], np.float64), np.array([bx, by], np.float64)
        d = b - a
        for p in P:
            if d @ d == 0:
                dist = np.hypot(*(p - a))
            else:
                s = min(1.0, max(0.0, float((p - a) @ d) / float(d @ d)))
                dist = np.hypot(*(p - (a + s * d)))
            if abs(dist - t / 2) < 1e-9:
                continue
            assert oracle.in_capsule(p[0], p[1], ax, ay, bx, by, t) == (dist < t / 2), (p, ax, ay, bx, by, t)
            checked += 1
    assert checked > 20000


def test_symmetries():
    rng = np.random.default_rng(6)
    for _ in range(300):
        ax, ay, bx, by, px, py = (int(v) for v in rng.integers(-20, 20, 6))
        t = int(rng.integers(0, 9))
        v = oracle.in_capsule(px, py, ax, ay, bx, by, t)
        assert v == oracle.in_capsule(px, py, bx, by, ax, ay, t)            # end points swapped
        assert v == oracle.in_capsule(py, px, ay, ax, by, bx, t)            # transposed
        assert v == oracle.in_capsule(-px, py, -ax, ay, -bx, by, t)         # mirrored
        assert v == oracle.in_capsule(px + 7, py - 3, ax + 7, ay - 3, bx + 7, by - 3, t)
        if v:
            assert oracle.in_capsule(px, py, ax, ay, bx, by, t + 1)         # monotone in thickness
    assert oracle.in_capsule(0, 0, 0, 0, 0, 0, 0) and not oracle.in_capsule(1, 0, 0, 0, 0, 0, 1)


def numpy_painter(frames, H, W, limb_a, limb_b, px, py, slots, limb_rgb, part_rgb, thickness, radius):
    """The same rules written independently: float64 geometry on whole coordinate grids, per primitive, in order."""
    out = frames.copy()
    N, Hf, Wf, C = frames.shape
    yy, xx = np.mgrid[0:Hf, 0:Wf].astype(np.float64)
    fx = lambda x: ((2 * int(x) + 1) * Wf) // (2 * W)
    fy = lambda y: ((2 * int(y) + 1) * Hf) // (2 * H)
    for n in range(N):
        for s in slots[n]:
            for l, (a, b) in enumerate(zip(limb_a, limb_b)):
                if s[a] < 0 or s[b] < 0:
                    continue
                A = np.array([fx(px[n, a, s[a]]), fy(py[n, a, s[a]])], np.float64)
                B = np.array([fx(px[n, b, s[b]]), fy(py[n, b, s[b]])], np.float64)
                d = B - A
                L2 = d @ d
                t = np.zeros_like(xx) if L2 == 0 else np.clip(((xx - A[0]) * d[0] + (yy - A[1]) * d[1]) / L2, 0, 1)
                dist2 = (xx - (A[0] + t * d[0])) ** 2 + (yy - (A[1] + t * d[1])) ** 2
                out[n][dist2 <= thickness * thickness / 4 + 1e-9, :3] = limb_rgb[l]
            for c in range(len(s)):
                if s[c] < 0:
                    continue
                cx, cy = fx(px[n, c, s[c]]), fy(py[n, c, s[c]])
                out[n][(xx - cx) ** 2 + (yy - cy) ** 2 <= radius * radius, :3] = part_rgb[c]
    return out


def random_scene(rng, N, Hf, Wf, C, H, W, K, L, cap, n_persons, missing=0.2):
    frames = rng.integers(0, 256, (N, Hf, Wf, C), dtype=np.uint8)
    limb_a = rng.integers(0, K, L).astype(np.int32)
    limb_b = ((limb_a + 1 + rng.integers(0, K - 1, L)) % K).astype(np.int32)
    px = rng.integers(0, W, (N, K, cap)).astype(np.int32)
    py = rng.integers(0, H, (N, K, cap)).astype(np.int32)
    slots = []
    for n in range(N):
        s = rng.integers(0, cap, (n_persons[n], K)).astype(np.int32)
        s[rng.random(s.shape) < missing] = -1
        slots.append(s)
    limb_rgb = rng.integers(0, 256, (L, 3), dtype=np.uint8)
    part_rgb = rng.integers(0, 256, (K, 3), dtype=np.uint8)
    return frames, limb_a, limb_b, px, py, slots, limb_rgb, part_rgb


@pytest.mark.parametrize("seed,C,scale", [(0, 3, (1, 1)), (1, 4, (2, 2)), (2, 3, (1, 2)), (3, 3, (3, 1)), (4, 4, (1, 1))])
def test_whole_scene_against_a_numpy_painter(seed, C, scale):
    rng = np.random.default_rng(seed)
    H, W = 24, 40
    Hf, Wf = H * scale[0], W * scale[1]
    if seed == 4:
        Hf, Wf = 17, 29                      # a frame smaller than the map, not an integer ratio
    frames, la, lb, px, py, slots, lrgb, prgb = random_scene(rng, 2, Hf, Wf, C, H, W, 5, 6, 7, [4, 0])
    for thickness, radius in ((1, 0), (3, 2), (6, 4)):
        got = oracle.draw_poses(frames, H, W, la, lb, px, py, slots, lrgb, prgb, thickness, radius)
        want = numpy_painter(frames, H, W, la, lb, px, py, slots, lrgb, prgb, thickness, radius)
        assert np.array_equal(got, want)
        assert np.array_equal(got[1], frames[1])                 # no persons: the frame is copied
        if C == 4:
            assert np.array_equal(got[..., 3], frames[..., 3])   # the fourth channel is never touched


def test_painters_order_and_coordinate_map():
    H, W, K = 8, 8, 2
    frames = np.zeros((1, 8, 8, 3), np.uint8)
    la, lb = np.array([0], np.int32), np.array([1], np.int32)
    px = np.array([[[1, 1], [6, 6]]], np.int32)
    py = np.array([[[2, 5], [2, 5]]], np.int32)
    lrgb, prgb = np.array([[9, 9, 9]], np.uint8), np.array([[50, 0, 0], [0, 60, 0]], np.uint8)
    # person 0 on row 2, person 1 on row 5; thickness 1, radius 0: each is a hairline with two coloured end pixels
    out = oracle.draw_poses(frames, H, W, la, lb, px, py, [np.array([[0, 0], [1, 1]])], lrgb, prgb, 1, 0)
    for row in (2, 5):
        assert out[0, row, 1].tolist() == [50, 0, 0] and out[0, row, 6].tolist() == [0, 60, 0]
        assert np.all(out[0, row, 2:6] == 9)
    assert out.sum() == 2 * (4 * 27 + 110)
    # a person drawn later covers an earlier one: both persons on the same peaks, the second one misses part 1, so only
    # its part-0 dot is drawn, on top of the first person's
    prgb2 = prgb.copy()
    out = oracle.draw_poses(frames, H, W, la, lb, px, py, [np.array([[0, 0], [0, -1]])], lrgb, prgb2, 3, 1)
    assert out[0, 2, 1].tolist() == [50, 0, 0] and out[0, 2, 2].tolist() == [50, 0, 0]     # disc of radius 1 over the limb
    assert out[0, 2, 3].tolist() == [9, 9, 9] and out[0, 1, 3].tolist() == [9, 9, 9] and out[0, 0, 3].tolist() == [0, 0, 0]
    # coordinate map: twice the size -> 2x + 1; half the size -> x // 2; same size -> x
    for Wf, want in ((16, [3, 13]), (4, [0, 3]), (8, [1, 6])):
        fr = np.zeros((1, 8, Wf, 3), np.uint8)
        o = oracle.draw_poses(fr, H, W, la, lb, px, py, [np.array([[0, 0]])], lrgb, prgb, 0, 0)
        cols = sorted(int(c) for c in np.nonzero(o[0, 2].sum(axis=1))[0] if o[0, 2, c].tolist() != [9, 9, 9])
        assert cols == want, (Wf, cols)
