"""GPU parity of the visualisation operator (hp_draw_poses) against the drawing oracle: every byte of every frame."""
import numpy as np
import pytest
import torch

import oracle
from synth import CONFIGS, BENCH_CAPS, COCO18, BODY25, SynthConfig, generate, DEFAULT_PARAMS
from parity import run_oracle, caps_for

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def hp():
    import paper_2108_11826_amd as m
    return m


def colours(K, L, seed=3):
    rng = np.random.default_rng(seed)
    return rng.integers(1, 256, (L, 3), dtype=np.uint8), rng.integers(1, 256, (K, 3), dtype=np.uint8)


def dense_peaks(ora, K, cap):
    N = len(ora["peaks"])
    px, py = np.zeros((N, K, cap), np.int32), np.zeros((N, K, cap), np.int32)
    for n in range(N):
        for c in range(K):
            x, y, _ = ora["peaks"][n][c]
            px[n, c, :len(x)], py[n, c, :len(y)] = x, y
    return px, py


@pytest.mark.parametrize("case", [
    dict(ci=2, frame=(360, 640), C=3, thickness=4, radius=4),
    dict(ci=2, frame=(368, 656), C=4, thickness=3, radius=2),
    dict(ci=2, frame=(187, 333), C=3, thickness=1, radius=0),       # rows that are no whole number of 4-pixel groups
    dict(ci=0, frame=(736, 736), C=3, thickness=9, radius=7),       # frame larger than the map
    dict(ci=1, frame=(90, 100), C=4, thickness=0, radius=1, in_place=True),
], ids=lambda c: "cfg%d-%dx%dx%d-t%d-r%d" % (c["ci"], c["frame"][1], c["frame"][0], c["C"], c["thickness"], c["radius"]))
def test_poses_of_the_operator_drawn_on_frames(case):
    m = hp()
    cfg = CONFIGS[case["ci"]]
    sk = cfg.skeleton
    b = generate(cfg)
    ora = run_oracle(b, DEFAULT_PARAMS)
    cap, ccap, pcap = BENCH_CAPS[case["ci"]]
    N = cfg.batch
    buf = m.Buffers(N, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, cap, ccap, pcap, DEV)
    skel = m.Skeleton(sk.n_parts, sk.limb_a, sk.limb_b)
    P = DEFAULT_PARAMS
    prm = m.Params(P.peak_thr, P.paf_thr, P.n_samples, P.min_valid_ratio, P.min_parts, P.scale)
    m.hp_postprocess(torch.from_numpy(b.cm).to(DEV), torch.from_numpy(b.paf).to(DEV), skel, prm, buf)
    Hf, Wf = case["frame"]
    frames = np.random.default_rng(11).integers(0, 256, (N, Hf, Wf, case["C"]), dtype=np.uint8)
    lrgb, prgb = colours(sk.n_parts, sk.n_limbs)
    d_frames = torch.from_numpy(frames).to(DEV)
    out = m.hp_draw_poses(d_frames, cfg.H, cfg.W, skel, buf, lrgb, prgb, case["thickness"], case["radius"],
                          out=d_frames if case.get("in_place") else None)
    got = out.cpu().numpy()
    px, py = dense_peaks(ora, sk.n_parts, cap)
    want = oracle.draw_poses(frames, cfg.H, cfg.W, sk.limb_a, sk.limb_b, px, py, [p[0] for p in ora["poses"]], lrgb, prgb,
                             case["thickness"], case["radius"])
    assert np.array_equal(got, want)
    assert np.any(want != frames)                       # something was drawn
    if not case.get("in_place"):
        assert np.array_equal(d_frames.cpu().numpy(), frames)   # the source is left alone


def scene(rng, N, K, L, cap, pcap, H, W, persons, missing):
    px = rng.integers(0, W, (N, K, cap)).astype(np.int32)
    py = rng.integers(0, H, (N, K, cap)).astype(np.int32)
    slots = np.full((N, pcap, K), -1, np.int32)
    for n in range(N):
        s = rng.integers(0, cap, (persons[n], K)).astype(np.int32)
        s[rng.random(s.shape) < missing] = -1
        slots[n, :persons[n]] = s
    return px, py, slots


@pytest.mark.parametrize("seed,sk,pcap,persons,frame,C,thickness,radius", [
    (0, COCO18, 128, [128, 0, 77], (96, 128), 3, 5, 3),        # 128 x 37 primitives: many chunks, heavy overlap
    (1, BODY25, 40, [40, 1], (61, 83), 3, 2, 2),
    (2, COCO18, 16, [16], (5, 3), 4, 3, 1),
    (3, COCO18, 8, [3], (1, 1), 3, 1, 0),
    (4, BODY25, 64, [64, 64], (200, 300), 4, 40, 25),          # primitives larger than tiles
    (5, COCO18, 32, [9, 32, 0, 5], (48, 64), 3, 0, 0),
    (6, COCO18, 8, [8], (2304, 4096), 3, 6, 5),                # more tiles than the list kernel counts in LDS
])
def test_random_scenes(seed, sk, pcap, persons, frame, C, thickness, radius):
    m = hp()
    rng = np.random.default_rng(seed)
    N, K, L, cap = len(persons), sk.n_parts, sk.n_limbs, 24
    H, W = 40, 56
    Hf, Wf = frame
    px, py, slots = scene(rng, N, K, L, cap, pcap, H, W, persons, 0.25)
    buf = m.Buffers(N, K, L, 5, 7, cap, 32, pcap, DEV)
    buf.px.copy_(torch.from_numpy(px))
    buf.py.copy_(torch.from_numpy(py))
    buf.slots.copy_(torch.from_numpy(slots))
    # a count above the capacity is clamped to it
    count = np.array(persons, np.int32)
    if seed == 0:
        count[0] = pcap + 5
    buf.pose_count.copy_(torch.from_numpy(count))
    skel = m.Skeleton(K, sk.limb_a, sk.limb_b)
    frames = rng.integers(0, 256, (N, Hf, Wf, C), dtype=np.uint8)
    lrgb, prgb = colours(K, L, seed)
    got = m.hp_draw_poses(torch.from_numpy(frames).to(DEV), H, W, skel, buf, lrgb, prgb, thickness, radius).cpu().numpy()
    want = oracle.draw_poses(frames, H, W, sk.limb_a, sk.limb_b, px, py, [slots[n, :persons[n]] for n in range(N)],
                             lrgb, prgb, thickness, radius)
    assert np.array_equal(got, want)


def test_misaligned_frames_take_the_general_path():
    # a frame tensor that starts at an odd address: no 4-byte groups, same result
    m = hp()
    rng = np.random.default_rng(9)
    sk = COCO18
    N, K, L, cap, pcap, H, W, Hf, Wf = 2, sk.n_parts, sk.n_limbs, 16, 8, 32, 32, 40, 64
    px, py, slots = scene(rng, N, K, L, cap, pcap, H, W, [8, 5], 0.2)
    buf = m.Buffers(N, K, L, 4, 4, cap, 32, pcap, DEV)
    buf.px.copy_(torch.from_numpy(px))
    buf.py.copy_(torch.from_numpy(py))
    buf.slots.copy_(torch.from_numpy(slots))
    buf.pose_count.copy_(torch.tensor([8, 5], dtype=torch.int32))
    skel = m.Skeleton(K, sk.limb_a, sk.limb_b)
    frames = rng.integers(0, 256, (N, Hf, Wf, 3), dtype=np.uint8)
    lrgb, prgb = colours(K, L)
    flat = torch.zeros(frames.size + 1, dtype=torch.uint8, device=DEV)
    src = flat[1:].view(N, Hf, Wf, 3)
    src.copy_(torch.from_numpy(frames))
    oflat = torch.zeros(frames.size + 3, dtype=torch.uint8, device=DEV)
    dst = oflat[3:].view(N, Hf, Wf, 3)
    m.hp_draw_poses(src, H, W, skel, buf, lrgb, prgb, 3, 2, out=dst)
    want = oracle.draw_poses(frames, H, W, sk.limb_a, sk.limb_b, px, py, [slots[0, :8], slots[1, :5]], lrgb, prgb, 3, 2)
    assert np.array_equal(dst.cpu().numpy(), want)
    assert oflat[:3].cpu().tolist() == [0, 0, 0]
