"""Random workloads, one seeded and time-bounded run per operator: the HIP library through its C ABI against the CPU
oracle on inputs whose sizes, tables, thresholds and capacities are drawn at random, every output compared (integers
exactly, floats bit for bit).  A run draws workloads from a fixed seed until its time budget is spent (HP_RANDOM_SECONDS,
default 20 s per operator) and stops at its first mismatch, naming the workload."""
import os
import time

import numpy as np
import pytest
import torch

import oracle
from synth import (COCO18, BODY25, SynthConfig, generate, Params, PPConfig, PP_COCO19, generate_pp, CFConfig, CF_COCO17,
                   generate_cf)
from parity import assert_lists_equal, assert_poses_equal, caps_for

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
BUDGET = float(os.environ.get("HP_RANDOM_SECONDS", "20"))


def hp():
    import paper_2108_11826_amd as m
    return m


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def run_until(budget, seed, one, at_least):
    """Calls one(rng, k) with rngs seeded (seed, k) until the budget is spent; `one` returns False for a draw it skipped."""
    t_end = time.time() + budget
    k = done = 0
    while time.time() < t_end or done < at_least:
        if one(np.random.default_rng([seed, k]), k) is not False:
            done += 1
        k += 1
        if k % 25 == 0:
            print(f"  {done} workloads compared", flush=True)
    print(f"  {done} workloads compared, all identical", flush=True)
    return done


def test_main_path_random_workloads():
    """Random sizes, skeleton, people, noise, storage type and parameters; each workload through the fused, the
    materialising and the staged form, half of them with capacities that take the general kernels."""
    m = hp()

    def one(rng, k):
        sk = BODY25 if rng.random() < 0.35 else COCO18
        h, w = int(rng.integers(1, 48)), int(rng.integers(1, 64))
        cfg = SynthConfig(5000 + k, sk, int(rng.integers(1, 6)), h, w, int(rng.integers(0, 14)),
                          scale_lo=float(rng.integers(10, 40)), scale_hi=float(rng.integers(40, 200)),
                          noise_sd=float(rng.choice([0.0, 0.01, 0.03, 0.06, 0.1])),
                          dropout=float(rng.choice([0.0, 0.15, 0.3])), n_spurious=int(rng.integers(0, 20)),
                          truncation=bool(rng.random() < 0.4), clustered=bool(rng.random() < 0.3),
                          dtype="float16" if rng.random() < 0.4 else "float32")
        p = Params(peak_thr=float(rng.choice([0.05, 0.02, 0.1, 0.3, 0.0])), paf_thr=float(rng.choice([0.05, 0.0, 0.2, -0.1])),
                   n_samples=int(rng.choice([10, 2, 3, 7, 16, 33])), min_valid_ratio=float(rng.choice([0.8, 0.0, 0.5, 1.0])),
                   min_parts=int(rng.choice([3, 0, 1, 6])), scale=8)
        b = generate(cfg)
        ora = oracle.postprocess(b.cm, b.paf, sk.limb_a, sk.limb_b, p, threads=8)
        caps = caps_for(ora)
        if rng.random() < 0.5:
            caps = (max(caps[0], 300), max(caps[1], 2048), caps[2])
        skel = m.Skeleton(sk.n_parts, sk.limb_a, sk.limb_b)
        prm = m.Params(p.peak_thr, p.paf_thr, p.n_samples, p.min_valid_ratio, p.min_parts, 8)
        cm, paf = to_dev(b.cm), to_dev(b.paf)
        N = b.cm.shape[0]
        for form in ("fused", "materialised", "staged"):
            where = f"workload {k} ({form}): {cfg}, {p}, capacities {caps}"
            buf = m.Buffers(N, sk.n_parts, sk.n_limbs, h, w, *caps, DEV)
            if form == "staged":
                m.hp_find_peaks(m.hp_resize(cm), sk.n_parts, p.peak_thr, buf)
                m.hp_score_limbs(m.hp_resize(paf), skel, prm, buf)
                m.hp_assemble(skel, prm, buf)
            else:
                his = (None, None)
                if form == "materialised":
                    his = (torch.empty((N, sk.n_parts + 1, 8 * h, 8 * w), dtype=torch.float32, device=DEV),
                           torch.empty((N, 2 * sk.n_limbs, 8 * h, 8 * w), dtype=torch.float32, device=DEV))
                m.hp_postprocess(cm, paf, skel, prm, buf, *his)
            try:
                assert buf.host_status() == 0
                assert_lists_equal("peaks", buf.host_peaks()[0], ora["peaks"])
                assert_lists_equal("candidates", buf.host_cands()[0], ora["candidates"])
                assert_lists_equal("connections", buf.host_conns()[0], ora["conns"])
                assert_poses_equal(buf.host_poses()[0], ora["poses"])
            except AssertionError as e:
                raise AssertionError(f"{where}: {e}") from None

    run_until(BUDGET, 1, one, 10)


def test_pose_proposal_random_workloads():
    """Random grids (up to 32 x 32), neighbourhoods, thresholds, person counts; a third with quantised values (ties)."""
    m = hp()

    def one(rng, k):
        G = int(rng.integers(1, 33))
        Gh, Gw = G, int(rng.integers(1, min(32, 1024 // G) + 1))
        Nh, Nw = int(rng.choice([1, 3, 5, 9, 15])), int(rng.choice([1, 3, 7, 9, 31]))
        batch = int(rng.integers(1, 6))
        img = float(rng.choice([128.0, 384.0, 777.0]))
        cfg = PPConfig(int(rng.integers(1000, 100000)), PP_COCO19, batch, Gh, Gw, int(rng.integers(0, 9)), Nh=Nh, Nw=Nw,
                       img_h=img, img_w=img * 1.5, scale_lo=float(rng.uniform(30, 90)), scale_hi=float(rng.uniform(90, 300)),
                       noise=float(rng.uniform(0.01, 0.12)), dropout=float(rng.uniform(0, 0.4)),
                       det_thr=float(rng.choice([0.0, 0.1, 0.3, 0.6])), nms_thr=float(rng.choice([0.0, 0.3, 0.7, 1.0])),
                       edge_thr=float(rng.choice([0.0, 0.1, 0.3, 0.9])), min_parts=int(rng.integers(1, 6)))
        d = generate_pp(cfg)
        if rng.random() < 0.3:
            d["resp"] = (np.round(d["resp"] * 8) / 8).astype(np.float32)
            d["edge"] = (np.round(d["edge"] * 8) / 8).astype(np.float32)
        sk = cfg.skeleton
        ora = oracle.pp_decode(d["resp"], d["conf"], d["box"], d["edge"], sk.limb_a, sk.limb_b, cfg.img_w, cfg.img_h,
                               cfg.det_thr, cfg.nms_thr, cfg.edge_thr, cfg.min_parts)
        K = sk.n_parts
        need_cap = max(1, max(len(ora["dets"][i][q][0]) for i in range(batch) for q in range(K)))
        need_pcap = max(1, max(len(p[0]) for p in ora["poses"]))
        if need_cap * K > 4096:
            return False
        buf = m.PPBuffers(batch, K, min(need_cap + int(rng.integers(0, 3)), 4096 // K), need_pcap + int(rng.integers(0, 3)), DEV)
        m.hp_pp_decode(to_dev(d["resp"]), to_dev(d["conf"]), to_dev(d["box"]), to_dev(d["edge"]),
                       m.Skeleton(K, sk.limb_a, sk.limb_b), buf, cfg.img_w, cfg.img_h, cfg.det_thr, cfg.nms_thr, cfg.edge_thr,
                       cfg.min_parts)
        torch.cuda.synchronize()
        got = buf.host()
        where = f"workload {k}: {cfg}"
        assert got["status"] == 0, where
        for i in range(batch):
            for q in range(K):
                for a, b in zip(got["dets"][i][q], ora["dets"][i][q]):
                    assert np.array_equal(np.ascontiguousarray(a).view(np.uint32), np.ascontiguousarray(b).view(np.uint32)), \
                        f"{where}: detections of image {i} part {q}"
            for a, b in zip(got["poses"][i], ora["poses"][i]):
                assert np.array_equal(np.ascontiguousarray(a).view(np.uint32), np.ascontiguousarray(b).view(np.uint32)), \
                    f"{where}: persons of image {i}"

    run_until(BUDGET, 2, one, 10)


def test_composite_field_random_workloads():
    """Random grids, strides, thresholds, reverse tolerances, person capacities; permuted limb tables; a third with
    quantised values (ties)."""
    m = hp()

    def one(rng, k):
        Fh, Fw = int(rng.integers(1, 40)), int(rng.integers(1, 60))
        stride = int(rng.choice([2, 4, 8, 8, 8, 16]))
        batch = int(rng.integers(1, 5))
        cfg = CFConfig(int(rng.integers(1000, 100000)), CF_COCO17, batch, Fh, Fw, int(rng.integers(0, 8)), stride=stride,
                       scale_lo=float(rng.uniform(20, 80)), scale_hi=float(rng.uniform(80, 300)),
                       dropout=float(rng.uniform(0, 0.4)), clutter=int(rng.integers(0, 80)),
                       pif_thr=float(rng.choice([0.0, 0.05, 0.1, 0.3])), paf_thr=float(rng.choice([0.0, 0.05, 0.1, 0.3])),
                       seed_thr=float(rng.choice([0.0, 0.1, 0.2, 0.5, 1.0])), grow_thr=float(rng.choice([0.0, 0.01, 0.05, 0.2])),
                       rev_tol=float(rng.choice([0.0, 1.0, 4.0, 8.0, 1e5])), min_parts=int(rng.integers(1, 8)))
        d = generate_cf(cfg)
        if rng.random() < 0.3:
            d["pif"][:, :, 0] = np.round(d["pif"][:, :, 0] * 8) / 8
            d["paf"][:, :, 0] = np.round(d["paf"][:, :, 0] * 8) / 8
            d["pif"][:, :, 1:3] = np.round(d["pif"][:, :, 1:3] * 4) / 4
        sk = cfg.skeleton
        la, lb = sk.limb_a.copy(), sk.limb_b.copy()
        if rng.random() < 0.5:
            perm = rng.permutation(sk.n_limbs)
            la, lb = la[perm], lb[perm]
            d["paf"] = np.ascontiguousarray(d["paf"][:, perm])
        prm = (cfg.stride, cfg.pif_thr, cfg.paf_thr, cfg.seed_thr, cfg.grow_thr, cfg.rev_tol, cfg.min_parts)
        pcap = int(rng.choice([1, 3, 16, 64]))
        ora = oracle.cf_decode(d["pif"], d["paf"], la, lb, *prm, pcap=pcap)
        K, L = sk.n_parts, sk.n_limbs
        need_cap = max(1, max(len(ora["pif"][i][q][0]) for i in range(batch) for q in range(K)))
        need_acap = max(1, max(len(ora["paf"][i][l][0]) for i in range(batch) for l in range(L)))
        if need_cap > 240 or need_cap * K > 4096:
            return False
        buf = m.CFBuffers(batch, K, L, min(240, need_cap + int(rng.integers(0, 4))), need_acap + int(rng.integers(0, 4)), pcap, DEV)
        m.hp_cf_decode(to_dev(d["pif"]), to_dev(d["paf"]), m.Skeleton(K, la, lb), buf, *prm)
        torch.cuda.synchronize()
        got = buf.host()
        where = f"workload {k}: {cfg}, person capacity {pcap}"
        assert got["status"] == (4 if any(ora["overflow"]) else 0), f"{where}: status {got['status']} vs {ora['overflow']}"
        for i in range(batch):
            for q in range(K):
                assert np.array_equal(got["pif"][i][q][0], ora["pif"][i][q][0]) and \
                    np.array_equal(bits(got["pif"][i][q][1]), bits(ora["pif"][i][q][1])), f"{where}: cells of image {i} part {q}"
            for l in range(L):
                assert np.array_equal(got["paf"][i][l][0], ora["paf"][i][l][0]) and \
                    all(np.array_equal(bits(a), bits(b)) for a, b in zip(got["paf"][i][l][1:], ora["paf"][i][l][1:])), \
                    f"{where}: associations of image {i} limb {l}"
            assert np.array_equal(got["poses"][i][1], ora["poses"][i][1]), f"{where}: part counts of image {i}"
            assert np.array_equal(bits(got["poses"][i][0]), bits(ora["poses"][i][0])), f"{where}: joints of image {i}"
            assert np.array_equal(bits(got["poses"][i][2]), bits(ora["poses"][i][2])), f"{where}: scores of image {i}"

    run_until(BUDGET, 3, one, 10)


def test_drawing_random_scenes():
    """Random peak positions and person tables on random frames: sizes, channel counts, thickness and radius vary."""
    m = hp()

    def one(rng, k):
        sk = COCO18 if rng.random() < 0.6 else BODY25
        K, L = sk.n_parts, sk.n_limbs
        N, cap, pcap = int(rng.integers(1, 4)), int(rng.integers(1, 30)), int(rng.integers(1, 60))
        H, W = int(rng.integers(1, 80)), int(rng.integers(1, 100))
        Hf, Wf = int(rng.integers(1, 150)), int(rng.integers(1, 200))
        C, th, rad = int(rng.choice([3, 4])), int(rng.integers(0, 12)), int(rng.integers(0, 9))
        persons = [int(rng.integers(0, pcap + 1)) for _ in range(N)]
        px = rng.integers(0, W, (N, K, cap)).astype(np.int32)
        py = rng.integers(0, H, (N, K, cap)).astype(np.int32)
        slots = np.full((N, pcap, K), -1, np.int32)
        for n in range(N):
            s = rng.integers(0, cap, (persons[n], K)).astype(np.int32)
            s[rng.random(s.shape) < rng.uniform(0, 0.6)] = -1
            slots[n, :persons[n]] = s
        buf = m.Buffers(N, K, L, 4, 4, cap, 32, pcap, DEV)
        buf.px.copy_(torch.from_numpy(px))
        buf.py.copy_(torch.from_numpy(py))
        buf.slots.copy_(torch.from_numpy(slots))
        buf.pose_count.copy_(torch.tensor(persons, dtype=torch.int32))
        frames = rng.integers(0, 256, (N, Hf, Wf, C), dtype=np.uint8)
        lrgb, prgb = rng.integers(0, 256, (L, 3), dtype=np.uint8), rng.integers(0, 256, (K, 3), dtype=np.uint8)
        got = m.hp_draw_poses(to_dev(frames), H, W, m.Skeleton(K, sk.limb_a, sk.limb_b), buf, lrgb, prgb, th, rad).cpu().numpy()
        want = oracle.draw_poses(frames, H, W, sk.limb_a, sk.limb_b, px, py, [slots[n, :persons[n]] for n in range(N)],
                                 lrgb, prgb, th, rad)
        assert np.array_equal(got, want), \
            f"scene {k}: N {N} K {K} cap {cap} pcap {pcap} map {H}x{W} frame {Hf}x{Wf}x{C} thickness {th} radius {rad} persons {persons}"

    run_until(BUDGET, 4, one, 20)


def test_smoothing_and_preprocessing_random_inputs():
    """Random maps smoothed with random taps of 1 to 65, peaks of the smoothed maps refined, and random frames
    pre-processed with random sizes, channel counts, scales and colour order."""
    m = hp()

    def one(rng, k):
        Hm, Wm = int(rng.integers(1, 150)), int(rng.integers(1, 200))
        Cm, Nm = int(rng.integers(1, 5)), int(rng.integers(1, 3))
        T = int(rng.choice([1, 3, 5, 7, 9, 13, 17, 21, 25, 33, 65]))
        taps = rng.normal(0, 1, T).astype(np.float32)
        maps = rng.normal(0, 1, (Nm, Cm, Hm, Wm)).astype(np.float32)
        Cs = int(rng.integers(1, Cm + 1))
        out_t = m.hp_smooth(to_dev(maps), to_dev(taps), channels=Cs, out=to_dev(maps.copy()))
        out = out_t.cpu().numpy()
        want = maps.copy()
        want[:, :Cs] = oracle.smooth(maps[:, :Cs], taps)
        assert np.array_equal(out.view(np.uint32), want.view(np.uint32)), f"smoothing {k}: {Nm}x{Cm} (first {Cs}) maps {Hm}x{Wm}, {T} taps"
        # peaks of the smoothed maps, then their sub-pixel positions
        thr = 0.5
        peaks = [[oracle.find_peaks(want[n, c], thr) for c in range(Cs)] for n in range(Nm)]
        cap = max(8, max(len(p[0]) for im in peaks for p in im) + 2)
        buf = m.Buffers(Nm, Cs, 1, max(1, Hm // 8), max(1, Wm // 8), cap, 16, 16, DEV)
        m.hp_find_peaks(out_t, Cs, thr, buf)
        xf, yf = m.hp_refine_peaks(out_t, Cs, buf)
        assert buf.host_status() == 0
        assert_lists_equal("peaks", buf.host_peaks()[0], peaks)
        xf, yf = xf.cpu().numpy(), yf.cpu().numpy()
        for n in range(Nm):
            for c in range(Cs):
                x, y, _ = peaks[n][c]
                wx, wy = oracle.refine_peaks(want[n, c], x, y)
                assert np.array_equal(bits(xf[n, c, :len(x)]), bits(wx)) and np.array_equal(bits(yf[n, c, :len(x)]), bits(wy)), \
                    f"refinement {k}: map {n},{c} of {Hm}x{Wm}"
        # pre-processing
        Np, Hs, Ws = int(rng.integers(1, 3)), int(rng.integers(1, 120)), int(rng.integers(1, 160))
        Cp, Hd, Wd = int(rng.choice([1, 3, 4])), int(rng.integers(1, 140)), int(rng.integers(1, 180))
        im = rng.integers(0, 256, (Np, Hs, Ws, Cp), dtype=np.uint8)
        alpha, beta = rng.normal(0, 1, Cp).astype(np.float32), rng.normal(0, 1, Cp).astype(np.float32)
        rev = bool(rng.random() < 0.5)
        got = m.hp_preprocess(to_dev(im), Hd, Wd, alpha, beta, rev).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), oracle.preprocess(im, Hd, Wd, alpha, beta, rev).view(np.uint32)), \
            f"pre-processing {k}: {Np} frames {Hs}x{Ws}x{Cp} -> {Hd}x{Wd}, reversed {rev}"

    run_until(BUDGET, 5, one, 20)
