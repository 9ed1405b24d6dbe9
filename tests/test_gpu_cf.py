"""GPU parity of the composite-field decoder (hp_cf_decode, hp_cf_field) against its oracle: cell lists, map values,
persons and the fine maps identical, floats bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from synth import CFConfig, CF_CONFIGS, CF_COCO17, generate_cf

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def hp():
    import paper_2108_11826_amd as m
    return m


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def run_both(cfg, d=None, cap=None, acap=None, pcap=None, limbs=None, **over):
    m = hp()
    d = d or generate_cf(cfg)
    sk = cfg.skeleton
    la, lb = (sk.limb_a, sk.limb_b) if limbs is None else (np.int32([a for a, _ in limbs]), np.int32([b for _, b in limbs]))
    K, L = d["pif"].shape[1], len(la)
    prm = dict(stride=cfg.stride, pif_thr=cfg.pif_thr, paf_thr=cfg.paf_thr, seed_thr=cfg.seed_thr, grow_thr=cfg.grow_thr,
               rev_tol=cfg.rev_tol, min_parts=cfg.min_parts)
    prm.update(over)
    N = d["pif"].shape[0]
    ora = oracle.cf_decode(d["pif"], d["paf"], la, lb, pcap=pcap or 64, **prm)
    need_cap = max(len(ora["pif"][n][k][0]) for n in range(N) for k in range(K))
    need_acap = max(len(ora["paf"][n][l][0]) for n in range(N) for l in range(L))
    need_pcap = max(len(p[1]) for p in ora["poses"])
    buf = m.CFBuffers(N, K, L, cap or max(4, need_cap + 3), acap or max(4, need_acap + 5), pcap or max(2, need_pcap + 2), DEV)
    skel = m.Skeleton(K, la, lb)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    m.hp_cf_decode(t(d["pif"]), t(d["paf"]), skel, buf, prm["stride"], prm["pif_thr"], prm["paf_thr"], prm["seed_thr"],
                   prm["grow_thr"], prm["rev_tol"], prm["min_parts"])
    torch.cuda.synchronize()
    return buf.host(), ora


def assert_same(got, ora, expect_status=0):
    assert got["status"] == expect_status
    for n in range(len(ora["poses"])):
        for k in range(len(ora["pif"][n])):
            (gc, gv), (oc, ov) = got["pif"][n][k], ora["pif"][n][k]
            assert np.array_equal(gc, oc), ("pif cells", n, k)
            assert np.array_equal(bits(gv), bits(ov)), ("pif values", n, k)
        for l in range(len(ora["paf"][n])):
            (gc, g1, g2), (oc, o1, o2) = got["paf"][n][l], ora["paf"][n][l]
            assert np.array_equal(gc, oc), ("paf cells", n, l)
            assert np.array_equal(bits(g1), bits(o1)) and np.array_equal(bits(g2), bits(o2)), ("paf samples", n, l)
        (gx, gn, gs), (ox, on, os_) = got["poses"][n], ora["poses"][n]
        assert np.array_equal(gn, on), ("parts", n, gn, on)
        assert np.array_equal(bits(gx), bits(ox)), ("joints", n)
        assert np.array_equal(bits(gs), bits(os_)), ("scores", n)


@pytest.mark.parametrize("cfg", CF_CONFIGS + [
    CFConfig(220, CF_COCO17, 3, 13, 29, 3, stride=4, scale_lo=40.0, scale_hi=70.0, dropout=0.2, clutter=15),
    CFConfig(221, CF_COCO17, 2, 30, 30, 12, stride=16, scale_lo=150.0, scale_hi=400.0, dropout=0.15, clutter=60),
    CFConfig(222, CF_COCO17, 1, 1, 1, 1, clutter=0),
    CFConfig(223, CF_COCO17, 2, 5, 301, 6, stride=8, scale_lo=20.0, scale_hi=36.0, clutter=30),
], ids=lambda c: "cf%d-%dx%dx%d" % (c.index, c.batch, c.Fh, c.Fw))
def test_decode_matches_oracle(cfg):
    got, ora = run_both(cfg)
    assert_same(got, ora)
    if cfg.index in (200, 201, 202, 220, 221):
        assert sum(len(p[1]) for p in ora["poses"]) > 0


def test_lists_near_the_capacity_limit():
    # 800 active cells per part and 1000-entry lists: the kernels that keep lists in LDS ask for more than 64 KB of it
    m = hp()
    rng = np.random.default_rng(21)
    N, K, L, Fh, Fw = 1, 3, 2, 40, 40
    pif = np.empty((N, K, 5, Fh, Fw), np.float32)
    pif[:, :, 0] = rng.random((N, K, Fh, Fw))
    pif[:, :, 1:3] = rng.normal(0, 0.6, (N, K, 2, Fh, Fw))
    pif[:, :, 3] = 1.0
    pif[:, :, 4] = rng.uniform(0.1, 0.6, (N, K, Fh, Fw))
    paf = np.empty((N, L, 7, Fh, Fw), np.float32)
    paf[:, :, 0] = rng.random((N, L, Fh, Fw))
    paf[:, :, (1, 2, 4, 5)] = rng.normal(0, 1.0, (N, L, 4, Fh, Fw))
    paf[:, :, (3, 6)] = rng.uniform(0.1, 0.8, (N, L, 2, Fh, Fw))
    cfg = CFConfig(232, CF_COCO17, N, Fh, Fw, 0, stride=4, pif_thr=0.5, paf_thr=0.5, seed_thr=0.8, grow_thr=0.05, rev_tol=3.0,
                   min_parts=2)
    got, ora = run_both(cfg, dict(pif=pif, paf=paf), limbs=[(0, 1), (1, 2)], cap=1000, acap=1000, pcap=400)
    assert_same(got, ora)
    assert got["pif_counts"].max() > 700
    maps, status = m.hp_cf_field(torch.from_numpy(pif).to(DEV), 4, 0.5, cap=1024)
    assert int(status.cpu()[0]) == 0
    for k in range(K):
        assert np.array_equal(bits(maps[0, k].cpu().numpy()), bits(oracle.cf_field(pif[0, k], 4, 0.5))), k


def test_a_crowd_at_full_hd():
    # 135 x 240 cells, 40 large persons: lists of 500 cells per part (8700 seeds to sort), 550 associations per limb
    cfg = CFConfig(250, CF_COCO17, 2, 135, 240, 40, stride=8, scale_lo=150.0, scale_hi=420.0, dropout=0.1, clutter=150)
    got, ora = run_both(cfg, pcap=90)
    assert_same(got, ora)
    assert max(got["pif_counts"].max(), 0) > 400 and min(len(p[1]) for p in ora["poses"]) >= 35


def test_benchmark_configuration():
    # the batch, the capacities and hence the launch shapes that bench.py times
    got, ora = run_both(CF_CONFIGS[2], cap=128, acap=256, pcap=32)
    assert_same(got, ora)
    assert min(len(p[1]) for p in ora["poses"]) >= 8


@pytest.mark.parametrize("over", [dict(pif_thr=0.0, paf_thr=0.0), dict(seed_thr=0.0, min_parts=1), dict(grow_thr=0.0),
                                  dict(rev_tol=0.0), dict(rev_tol=1e6), dict(min_parts=17), dict(seed_thr=2.5),
                                  dict(grow_thr=0.6), dict(pif_thr=0.5, paf_thr=0.5)],
                         ids=lambda o: "-".join("%s%g" % kv for kv in o.items()))
def test_parameter_corners(over):
    cfg = CF_CONFIGS[1]
    cap = acap = None
    if over.get("pif_thr") == 0.0:          # every cell whose vectors stay on the map is active: a small grid
        cfg = CFConfig(230, CF_COCO17, 1, 10, 12, 2, scale_lo=50.0, scale_hi=80.0, clutter=5)
        cap = acap = 120
    got, ora = run_both(cfg, cap=cap, acap=acap, **over)
    assert_same(got, ora)


def test_dense_random_fields():
    # no planted structure: hundreds of active cells per part, overlapping windows everywhere, equal values
    rng = np.random.default_rng(11)
    N, K, L, Fh, Fw = 2, 6, 7, 14, 18
    limbs = [(0, 1), (1, 2), (2, 3), (3, 4), (4, 5), (5, 0), (1, 4)]
    pif = np.empty((N, K, 5, Fh, Fw), np.float32)
    pif[:, :, 0] = rng.integers(0, 8, (N, K, Fh, Fw)) / 8
    pif[:, :, 1:3] = rng.integers(-4, 5, (N, K, 2, Fh, Fw)) / 4       # vectors on a quarter-cell lattice: many coincide
    pif[:, :, 3] = 1.0
    pif[:, :, 4] = rng.integers(1, 12, (N, K, Fh, Fw)) / 8
    paf = np.empty((N, L, 7, Fh, Fw), np.float32)
    paf[:, :, 0] = rng.integers(0, 8, (N, L, Fh, Fw)) / 8
    paf[:, :, (1, 2, 4, 5)] = rng.integers(-8, 9, (N, L, 4, Fh, Fw)) / 4
    paf[:, :, (3, 6)] = rng.integers(1, 8, (N, L, 2, Fh, Fw)) / 8
    cfg = CFConfig(231, CF_COCO17, N, Fh, Fw, 0, stride=8, pif_thr=0.3, paf_thr=0.3, seed_thr=0.5, grow_thr=0.01, rev_tol=6.0,
                   min_parts=2)
    got, ora = run_both(cfg, dict(pif=pif, paf=paf), limbs=limbs, pcap=680)   # 6 x 680 joints: the most the persons kernel holds
    assert_same(got, ora)
    assert max(len(c) for c, _ in ora["pif"][0]) > 100 and sum(len(p[1]) for p in ora["poses"]) > 20


def test_cyclic_and_reordered_limb_tables():
    cfg = CF_CONFIGS[1]
    d = generate_cf(cfg)
    sk = cfg.skeleton
    order = np.random.default_rng(2).permutation(sk.n_limbs)
    limbs = [(int(sk.limb_a[i]), int(sk.limb_b[i])) for i in order]
    got, ora = run_both(cfg, dict(pif=d["pif"], paf=np.ascontiguousarray(d["paf"][:, order])), limbs=limbs)
    assert_same(got, ora)
    flipped = [(b, a) for a, b in limbs]                                # every limb stored the other way round
    paf = np.ascontiguousarray(d["paf"][:, order][:, :, (0, 4, 5, 6, 1, 2, 3)])
    got2, ora2 = run_both(cfg, dict(pif=d["pif"], paf=paf), limbs=flipped)
    assert_same(got2, ora2)


def test_person_capacity_overflow_is_reported():
    cfg = CF_CONFIGS[1]
    got, ora = run_both(cfg, pcap=2)
    assert any(ora["overflow"])
    assert_same(got, ora, expect_status=4)
    assert list(got["pose_counts"]) == [len(p[1]) for p in ora["poses"]]


def test_list_capacity_overflow_is_reported():
    cfg = CF_CONFIGS[1]
    got, ora = run_both(cfg, cap=5, acap=1000)
    assert got["status"] & 1
    K = cfg.skeleton.n_parts
    assert all(got["pif_counts"][n][k] == len(ora["pif"][n][k][0]) for n in range(cfg.batch) for k in range(K))
    got, ora = run_both(cfg, acap=3)
    assert got["status"] & 2
    L = cfg.skeleton.n_limbs
    assert all(got["paf_counts"][n][l] == len(ora["paf"][n][l][0]) for n in range(cfg.batch) for l in range(L))


def test_candidate_lists_beyond_the_staged_size():
    # lists of more than 1024 candidates are written to the workspace as they are found, shorter ones are held in
    # LDS first: both forms give the same lists and persons
    cfg = CF_CONFIGS[1]
    got, ora = run_both(cfg, acap=1500)
    assert_same(got, ora)
    got, ora = run_both(cfg, acap=1024)
    assert_same(got, ora)
    got, ora = run_both(CF_CONFIGS[2], cap=256, acap=1025, pcap=32)
    assert_same(got, ora)


def test_images_are_independent_and_calls_repeat():
    m = hp()
    cfg = CF_CONFIGS[2]
    d = generate_cf(cfg)
    whole, ora = run_both(cfg, d)
    assert_same(whole, ora)
    one, _ = run_both(CFConfig(cfg.index, cfg.skeleton, 1, cfg.Fh, cfg.Fw, cfg.n_people),
                      dict(pif=d["pif"][5:6], paf=d["paf"][5:6]))
    assert np.array_equal(bits(one["poses"][0][0]), bits(whole["poses"][5][0]))
    again, _ = run_both(cfg, d)
    for n in range(cfg.batch):
        assert np.array_equal(bits(again["poses"][n][0]), bits(whole["poses"][n][0]))


@pytest.mark.parametrize("ci", [0, 1, 2])
def test_field_matches_oracle(ci):
    m = hp()
    cfg = CF_CONFIGS[ci]
    d = generate_cf(cfg)
    maps, status = m.hp_cf_field(torch.from_numpy(d["pif"]).to(DEV), cfg.stride, cfg.pif_thr, cap=128)
    torch.cuda.synchronize()
    assert int(status.cpu()[0]) == 0
    got = maps.cpu().numpy()
    for n in range(min(cfg.batch, 3)):
        for k in range(cfg.skeleton.n_parts):
            want = oracle.cf_field(d["pif"][n, k], cfg.stride, cfg.pif_thr)
            assert np.array_equal(bits(got[n, k]), bits(want)), (n, k)


def test_field_with_ragged_tiles_and_wide_windows():
    m = hp()
    rng = np.random.default_rng(6)
    N, K, Fh, Fw, s = 2, 3, 11, 19, 5          # 55 x 95 pixels: neither a multiple of the tile
    pif = np.zeros((N, K, 5, Fh, Fw), np.float32)
    pif[:, :, 0] = rng.random((N, K, Fh, Fw)) * (rng.random((N, K, Fh, Fw)) < 0.2)
    pif[:, :, 1:3] = rng.normal(0, 2.0, (N, K, 2, Fh, Fw))
    pif[:, :, 4] = rng.uniform(0.05, 3.0, (N, K, Fh, Fw))      # windows from 3 to 24 pixels
    maps, status = m.hp_cf_field(torch.from_numpy(pif).to(DEV), s, 0.05, cap=256)
    torch.cuda.synchronize()
    assert int(status.cpu()[0]) == 0
    got = maps.cpu().numpy()
    for n in range(N):
        for k in range(K):
            assert np.array_equal(bits(got[n, k]), bits(oracle.cf_field(pif[n, k], s, 0.05))), (n, k)


def test_exponential_matches_oracle_through_single_cells():
    # one isolated cell per part with a wide window: every map pixel is c * E(t) for a different t
    m = hp()
    K, Fh, Fw, s = 8, 8, 8, 8
    pif = np.zeros((1, K, 5, Fh, Fw), np.float32)
    rng = np.random.default_rng(8)
    for k in range(K):
        pif[0, k, :, 3, 4] = (1.0, rng.uniform(-0.5, 0.5), rng.uniform(-0.5, 0.5), 1.0, rng.uniform(0.2, 1.0))
    maps, _ = m.hp_cf_field(torch.from_numpy(pif).to(DEV), s, 0.05, cap=4)
    got = maps.cpu().numpy()
    for k in range(K):
        assert np.array_equal(bits(got[0, k]), bits(oracle.cf_field(pif[0, k], s, 0.05)))
        assert np.count_nonzero(got[0, k]) >= 49
