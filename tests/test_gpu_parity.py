"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from synth import CONFIGS, BENCH_CAPS, COCO18, BODY25, SynthConfig, generate, DEFAULT_PARAMS
from parity import assert_lists_equal, assert_poses_equal, run_oracle, caps_for, close

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def hp():
    import paper_2108_11826_amd as m
    return m


def prm_of(p=DEFAULT_PARAMS):
    return hp().Params(p.peak_thr, p.paf_thr, p.n_samples, p.min_valid_ratio, p.min_parts, p.scale)


def skel_of(sk):
    return hp().Skeleton(sk.n_parts, sk.limb_a, sk.limb_b)


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


SMALL = [
    SynthConfig(10, COCO18, 2, 5, 7, 1, scale_lo=20, scale_hi=40, noise_sd=0.05),
    SynthConfig(11, COCO18, 1, 1, 9, 1, scale_lo=20, scale_hi=40, noise_sd=0.05),
    SynthConfig(12, COCO18, 1, 9, 1, 1, scale_lo=20, scale_hi=40, noise_sd=0.05),
    SynthConfig(13, COCO18, 3, 33, 47, 6, noise_sd=0.02, dropout=0.1, n_spurious=10),
    SynthConfig(14, BODY25, 2, 31, 65, 5, noise_sd=0.02, dtype="float16"),
    SynthConfig(15, COCO18, 1, 2, 2, 1, scale_lo=10, scale_hi=12, noise_sd=0.05),
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: f"syn{c.index}")
def test_resize_bit_exact(cfg):
    b = generate(cfg)
    for lo in (b.cm, b.paf):
        got = hp().hp_resize(to_dev(lo)).cpu().numpy()
        want = oracle.resize(lo, 8)
        assert got.shape == want.shape
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def run_staged(b, ora, caps=None):
    """hp_resize -> hp_find_peaks -> hp_score_limbs -> hp_assemble."""
    m = hp()
    cfg = b.config
    sk = cfg.skeleton
    cap, ccap, pcap = caps or caps_for(ora)
    N = b.cm.shape[0]
    buf = m.Buffers(N, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, cap, ccap, pcap, DEV)
    skel, prm = skel_of(sk), prm_of()
    cm_hi = m.hp_resize(to_dev(b.cm))
    paf_hi = m.hp_resize(to_dev(b.paf))
    st = []
    m.hp_find_peaks(cm_hi, sk.n_parts, DEFAULT_PARAMS.peak_thr, buf)
    st.append(buf.host_status())
    m.hp_score_limbs(paf_hi, skel, prm, buf)
    st.append(buf.host_status())
    m.hp_assemble(skel, prm, buf)
    st.append(buf.host_status())
    return buf, st


def run_fused(b, ora, materialise, caps=None):
    m = hp()
    cfg = b.config
    sk = cfg.skeleton
    cap, ccap, pcap = caps or caps_for(ora)
    N = b.cm.shape[0]
    buf = m.Buffers(N, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, cap, ccap, pcap, DEV)
    cm, paf = to_dev(b.cm), to_dev(b.paf)
    cm_hi = paf_hi = None
    if materialise:
        cm_hi = torch.empty((N, sk.n_parts + 1, cfg.H, cfg.W), dtype=torch.float32, device=DEV)
        paf_hi = torch.empty((N, 2 * sk.n_limbs, cfg.H, cfg.W), dtype=torch.float32, device=DEV)
    m.hp_postprocess(cm, paf, skel_of(sk), prm_of(), buf, cm_hi, paf_hi)
    return buf, cm_hi, paf_hi


def check_all(buf, ora):
    assert buf.host_status() == 0
    assert_lists_equal("peaks", buf.host_peaks()[0], ora["peaks"])
    assert_lists_equal("candidates", buf.host_cands()[0], ora["candidates"])
    assert_lists_equal("connections", buf.host_conns()[0], ora["conns"])
    assert_poses_equal(buf.host_poses()[0], ora["poses"])


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: f"syn{c.index}")
def test_staged_calls_match_oracle(cfg):
    b = generate(cfg)
    ora = run_oracle(b, DEFAULT_PARAMS)
    buf, st = run_staged(b, ora)
    assert st == [0, 0, 0]
    check_all(buf, ora)


@pytest.mark.parametrize("ci", [0, 1, 2, 3, 4])
def test_staged_calls_full_configs(ci):
    """hp_resize -> hp_find_peaks -> hp_score_limbs -> hp_assemble on the five workloads at full size, with the
    capacities the benchmark times: the strip peak search on the materialised maps, the general scorer gathering from
    them, both matching kernels (lists of workloads 3 and 4 sort outside LDS) and the assembly, every list against the
    oracle."""
    print(f"staged route, config {ci}", flush=True)
    b = generate(CONFIGS[ci])
    ora = run_oracle(b, DEFAULT_PARAMS)
    buf, st = run_staged(b, ora, caps=BENCH_CAPS[ci])
    assert st == [0, 0, 0]
    check_all(buf, ora)


@pytest.mark.parametrize("materialise", [False, True], ids=["fused", "materialised"])
@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: f"syn{c.index}")
def test_postprocess_small(cfg, materialise):
    b = generate(cfg)
    ora = run_oracle(b, DEFAULT_PARAMS)
    buf, cm_hi, paf_hi = run_fused(b, ora, materialise)
    check_all(buf, ora)
    if materialise:
        for got, lo in ((cm_hi, b.cm), (paf_hi, b.paf)):
            want = oracle.resize(lo, 8)
            assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("materialise", [False, True], ids=["fused", "materialised"])
@pytest.mark.parametrize("ci", [0, 1, 2, 3, 4])
def test_postprocess_full_configs(ci, materialise):
    """The five workloads at full size, in the launch configuration the benchmark times."""
    cfg = CONFIGS[ci]
    print(f"config {ci} materialise={materialise}", flush=True)
    b = generate(cfg)
    ora = run_oracle(b, DEFAULT_PARAMS)
    buf, cm_hi, paf_hi = run_fused(b, ora, materialise, caps=BENCH_CAPS[ci])
    check_all(buf, ora)
    if materialise:
        # the maps are large: compare a sample of whole planes bit for bit
        rng = np.random.default_rng(ci)
        for got, lo in ((cm_hi, b.cm), (paf_hi, b.paf)):
            for _ in range(3):
                n, c = int(rng.integers(lo.shape[0])), int(rng.integers(lo.shape[1]))
                want = oracle.resize(lo[n, c], 8)
                assert np.array_equal(got[n, c].cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_results_are_deterministic():
    b = generate(CONFIGS[2])
    ora = run_oracle(b, DEFAULT_PARAMS)
    outs = []
    for _ in range(3):
        buf, _, _ = run_fused(b, ora, False)
        outs.append((buf.host_peaks(), buf.host_cands(), buf.host_conns(), buf.host_poses()))
    for o in outs[1:]:
        assert_lists_equal("peaks", o[0][0], outs[0][0][0])
        assert_lists_equal("candidates", o[1][0], outs[0][1][0])
        assert_lists_equal("connections", o[2][0], outs[0][2][0])
        assert_poses_equal(o[3][0], outs[0][3][0])


def test_empty_maps_give_empty_results():
    cfg = SynthConfig(20, COCO18, 2, 12, 17, 0, noise_sd=0.0)
    b = generate(cfg)
    assert not b.cm[:, :-1].any()
    ora = run_oracle(b, DEFAULT_PARAMS)
    for mat in (False, True):
        buf, _, _ = run_fused(b, ora, mat, caps=(16, 16, 16))
        check_all(buf, ora)
        assert buf.host_peaks()[1].sum() == 0 and buf.host_poses()[1].sum() == 0


def test_overflow_is_reported_not_hidden():
    m = hp()
    b = generate(CONFIGS[1])
    ora = run_oracle(b, DEFAULT_PARAMS)
    true_counts = np.array([[len(p[0]) for p in im] for im in ora["peaks"]])
    buf, _, _ = run_fused(b, ora, False, caps=(8, 1024, 64))
    assert buf.host_status() & m.STATUS_PEAK_OVERFLOW
    assert np.array_equal(buf.host_peaks()[1], true_counts)          # counts report the requirement
    # candidate overflow: peaks fit, candidate lists do not
    buf, _, _ = run_fused(b, ora, False, caps=(64, 2, 64))
    assert buf.host_status() == m.STATUS_CAND_OVERFLOW
    assert np.array_equal(buf.host_cands()[1], np.array([[len(c[0]) for c in im] for im in ora["candidates"]]))
    # pose overflow
    buf, _, _ = run_fused(b, ora, False, caps=(64, 1024, 2))
    assert buf.host_status() == m.STATUS_POSE_OVERFLOW
    assert buf.host_poses()[1][0] == len(ora["poses"][0][1])
    assert_lists_equal("connections", buf.host_conns()[0], ora["conns"])


def is_ordered_sublist(got, want):
    """got / want: (a, b, score) lists; every entry of got occurs in want, in want's order, at most once."""
    rows = {(int(a), int(b), np.float32(s).view(np.uint32).item()): k for k, (a, b, s) in enumerate(zip(*want))}
    pos = [rows.get((int(a), int(b), np.float32(s).view(np.uint32).item()), -1) for a, b, s in zip(*got)]
    return all(p >= 0 for p in pos) and all(p < q for p, q in zip(pos, pos[1:]))


@pytest.mark.parametrize("general", [False, True], ids=["one_launch", "general"])
def test_what_an_overflowed_list_holds(general):
    """A list that needed more than its capacity: the count is the requirement, the status bit is set, and the
    `cap` entries that are stored are entries of the true list in canonical order (which ones is not specified).
    Through the one-launch limb kernel and through the general kernels (candidate capacity beyond 1024 / peak
    capacity beyond 256 select those)."""
    m = hp()
    b = generate(CONFIGS[1])
    ora = run_oracle(b, DEFAULT_PARAMS)
    # peaks: capacity 8 where the workload has about 20 per part
    cap = 8
    buf, _, _ = run_fused(b, ora, False, caps=(cap, 2048 if general else 1024, 64))
    assert buf.host_status() & m.STATUS_PEAK_OVERFLOW
    lists, counts = buf.host_peaks()
    over = 0
    for c, want in enumerate(ora["peaks"][0]):
        assert counts[0, c] == len(want[0])
        assert len(lists[0][c][0]) == min(cap, len(want[0]))
        assert is_ordered_sublist(lists[0][c], want), f"part {c}"
        over += len(want[0]) > cap
    assert over > 0
    # candidates: the peaks fit, candidate capacity 2 where limbs have up to ten
    ccap = 2
    buf, _, _ = run_fused(b, ora, False, caps=(300 if general else 64, ccap, 64))
    assert buf.host_status() == m.STATUS_CAND_OVERFLOW
    assert_lists_equal("peaks", buf.host_peaks()[0], ora["peaks"])
    lists, counts = buf.host_cands()
    over = 0
    for l, want in enumerate(ora["candidates"][0]):
        assert counts[0, l] == len(want[0])
        assert len(lists[0][l][0]) == min(ccap, len(want[0]))
        assert is_ordered_sublist(lists[0][l], want), f"limb {l}"
        over += len(want[0]) > ccap
    assert over > 0


def test_staged_calls_report_overflow_too():
    """hp_find_peaks, hp_score_limbs and hp_assemble each overwrite the status word in their first kernel and
    report lists beyond their capacity; hp_assemble repeats the candidate overflow it is handed."""
    m = hp()
    b = generate(CONFIGS[1])
    cfg = b.config
    sk = cfg.skeleton
    ora = run_oracle(b, DEFAULT_PARAMS)
    skel, prm = skel_of(sk), prm_of()
    cm_hi, paf_hi = m.hp_resize(to_dev(b.cm)), m.hp_resize(to_dev(b.paf))
    # peaks do not fit
    buf = m.Buffers(1, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, 8, 256, 64, DEV)
    buf.status.fill_(0x70)
    m.hp_find_peaks(cm_hi, sk.n_parts, DEFAULT_PARAMS.peak_thr, buf)
    assert buf.host_status() == m.STATUS_PEAK_OVERFLOW
    assert np.array_equal(buf.host_peaks()[1], np.array([[len(p[0]) for p in im] for im in ora["peaks"]]))
    # peaks fit, candidates do not
    buf = m.Buffers(1, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, 64, 2, 64, DEV)
    buf.status.fill_(0x70)
    m.hp_find_peaks(cm_hi, sk.n_parts, DEFAULT_PARAMS.peak_thr, buf)
    assert buf.host_status() == 0
    buf.status.fill_(0x70)
    m.hp_score_limbs(paf_hi, skel, prm, buf)
    assert buf.host_status() == m.STATUS_CAND_OVERFLOW
    assert np.array_equal(buf.host_cands()[1], np.array([[len(c[0]) for c in im] for im in ora["candidates"]]))
    buf.status.fill_(0x70)
    m.hp_assemble(skel, prm, buf)
    assert buf.host_status() & m.STATUS_CAND_OVERFLOW and not buf.host_status() & 0x70
    # everything fits, persons do not
    buf = m.Buffers(1, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, 64, 256, 2, DEV)
    m.hp_find_peaks(cm_hi, sk.n_parts, DEFAULT_PARAMS.peak_thr, buf)
    m.hp_score_limbs(paf_hi, skel, prm, buf)
    buf.status.fill_(0x70)
    m.hp_assemble(skel, prm, buf)
    assert buf.host_status() == m.STATUS_POSE_OVERFLOW
    assert buf.host_poses()[1][0] == len(ora["poses"][0][1])


def test_large_lists_sort_outside_lds():
    """More peaks / candidates than the in-LDS sort holds: pure noise with a permissive PAF rule."""
    from synth import Params
    cfg = SynthConfig(21, COCO18, 1, 40, 64, 0, noise_sd=0.2)
    b = generate(cfg)
    p = Params(peak_thr=0.05, paf_thr=-1.0, n_samples=4, min_valid_ratio=0.5, min_parts=3)
    sk = cfg.skeleton
    # two limbs are enough to reach several thousand candidates each
    la, lb = sk.limb_a[:2], sk.limb_b[:2]
    paf = b.paf[:, :4]
    ora = oracle.postprocess(b.cm, paf, la, lb, p, threads=8)
    npk = max(len(x[0]) for x in ora["peaks"][0])
    ncand = max(len(x[0]) for x in ora["candidates"][0])
    assert npk > 300 and ncand > 5000
    m = hp()
    buf = m.Buffers(1, sk.n_parts, 2, cfg.h, cfg.w, 1024, 1 << 17, 4096, DEV)
    m.hp_postprocess(to_dev(b.cm), to_dev(paf), m.Skeleton(sk.n_parts, la, lb),
                     m.Params(p.peak_thr, p.paf_thr, p.n_samples, p.min_valid_ratio, p.min_parts, 8), buf)
    check_all(buf, ora)


@pytest.mark.parametrize("dtype", ["float32", "float16"])
@pytest.mark.parametrize("w", [1, 2, 3])
def test_narrow_maps(w, dtype):
    """Lo-res maps one, two and three columns wide (8, 16, 24 hi-res columns): the bilinear gather of the scorers has a
    form of its own for a single column, and the last column is the one place where its paired loads are shifted.
    Both capacities: the one-launch limb kernel and the general scorer."""
    from synth import Params
    rng = np.random.default_rng(700 + w)
    K, L, h = 3, 2, 40
    cm = (0.2 * rng.random((2, K + 1, h, w))).astype(dtype)           # the last channel is background
    paf = rng.normal(0.0, 0.5, (2, 2 * L, h, w)).astype(dtype)
    la, lb = [0, 1], [1, 2]
    p = Params(peak_thr=0.05, paf_thr=-0.5, n_samples=7, min_valid_ratio=0.6, min_parts=2)
    ora = oracle.postprocess(cm, paf, la, lb, p, threads=4)
    assert min(len(x[0]) for im in ora["candidates"] for x in im) > 20
    m = hp()
    for caps in ((256, 1 << 14, 256), (512, 1 << 15, 512)):
        buf = m.Buffers(2, K, L, h, w, *caps, DEV)
        m.hp_postprocess(to_dev(cm), to_dev(paf), m.Skeleton(K, la, lb),
                         m.Params(p.peak_thr, p.paf_thr, p.n_samples, p.min_valid_ratio, p.min_parts, 8), buf)
        check_all(buf, ora)


def test_assembly_with_tables_beyond_lds():
    """An image with more connections than the in-LDS person tables hold: the fold runs on the
    workspace tables instead and must give the same persons."""
    from synth import Params
    cfg = SynthConfig(22, COCO18, 2, 28, 36, 0, noise_sd=0.2)
    b = generate(cfg)
    p = Params(peak_thr=0.05, paf_thr=-1.0, n_samples=4, min_valid_ratio=0.5, min_parts=3)
    sk = cfg.skeleton
    ora = oracle.postprocess(b.cm, b.paf, sk.limb_a, sk.limb_b, p, threads=8)
    assert min(sum(len(x[0]) for x in im) for im in ora["conns"]) > 2000
    m = hp()
    buf = m.Buffers(2, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, 512, 1 << 15, 1024, DEV)
    m.hp_postprocess(to_dev(b.cm), to_dev(b.paf), skel_of(sk),
                     m.Params(p.peak_thr, p.paf_thr, p.n_samples, p.min_valid_ratio, p.min_parts, 8), buf)
    check_all(buf, ora)


def test_parts_used_by_no_limb_are_still_listed():
    """A skeleton whose limb table leaves parts out: their peak lists must still come back
    (small capacities: the one-launch limb kernel publishes them; large: the general kernels)."""
    cfg = SMALL[3]
    b = generate(cfg)
    sk = cfg.skeleton
    la, lb = sk.limb_a[5:9], sk.limb_b[5:9]
    paf = np.ascontiguousarray(b.paf[:, 10:18])
    ora = oracle.postprocess(b.cm, paf, la, lb, DEFAULT_PARAMS, threads=4)
    m = hp()
    for caps in ((64, 256, 64), (512, 4096, 64)):
        buf = m.Buffers(b.cm.shape[0], sk.n_parts, 4, cfg.h, cfg.w, *caps, DEV)
        m.hp_postprocess(to_dev(b.cm), to_dev(paf), m.Skeleton(sk.n_parts, la, lb), prm_of(), buf)
        check_all(buf, ora)


@pytest.mark.parametrize("shape", [(37, 53), (9, 7), (1, 1), (3, 250), (40, 248), (41, 252), (16, 496), (64, 500), (5, 4)],
                         ids=lambda s: f"{s[0]}x{s[1]}")
def test_find_peaks_on_arbitrary_maps(shape):
    """hp_find_peaks on given hi-res maps of any size: widths that are whole 16-byte groups take the
    strip kernel (one, two and three strips across, ragged last strip, rows not a multiple of the
    strip height), others the general one.  Values are quantised so that ties and plateaus abound."""
    m = hp()
    H, W = shape
    rng = np.random.default_rng(H * 1000 + W)
    N, K = 2, 3
    maps = (rng.integers(0, 12, size=(N, K + 1, H, W)) / 16.0).astype(np.float32)
    maps[0, 0, :, :] = 0.5                       # one plateau over a whole plane
    maps[1, 1, H - 1, W - 1] = 2.0               # a peak in the last corner
    maps[1, 2, 0, 0] = 2.0                       # and in the first
    want = [[oracle.find_peaks(maps[n, c], 0.05) for c in range(K)] for n in range(N)]
    cap = max(16, max(len(p[0]) for im in want for p in im) + 4)
    buf = m.Buffers(N, K, 1, max(1, H // 8), max(1, W // 8), cap, 16, 16, DEV)
    m.hp_find_peaks(to_dev(maps), K, 0.05, buf)
    assert buf.host_status() == 0
    assert_lists_equal("peaks", buf.host_peaks()[0], want)


@pytest.mark.parametrize("which", ["just_above", "equal"])
def test_scorer_at_the_validity_threshold(which):
    """The general scorer screens pairs with an approximate unit vector plus an error margin before
    it scores them exactly; pairs whose samples sit exactly on, or one float above, the validity
    threshold are where a screen that dropped too much would show.  Constant PAF (1/16, 0): every
    sample of a pair projects to ux / 16 exactly, and all pairs along (3k, 4k) share ux = fl(0.6)."""
    m = hp()
    h, w = 40, 60
    H, W = 8 * h, 8 * w
    K, L = 2, 1
    rng = np.random.default_rng(7)
    xa = rng.integers(0, W - 200, size=300)
    ya = rng.integers(0, H - 260, size=300)
    order = np.lexsort((xa, ya))
    xa, ya = xa[order].astype(np.int32), ya[order].astype(np.int32)
    ks = rng.integers(1, 60, size=300)
    xb, yb = xa + 3 * ks, ya + 4 * ks                      # B_i - A_i = k (3, 4), and many near-misses with other A
    order = np.lexsort((xb, yb))
    xb, yb = xb[order].astype(np.int32), yb[order].astype(np.int32)
    paf_lo = np.zeros((1, 2, h, w), np.float32)
    paf_lo[0, 0] = 0.0625
    d = np.float32(np.float32(3.0) / np.float32(5.0)) * np.float32(0.0625)
    thr = float(d) if which == "equal" else float(np.nextafter(d, np.float32(-1)))
    p = DEFAULT_PARAMS
    want = oracle.score_limb(paf_lo[0, 0], paf_lo[0, 1], 8, xa, ya, xb, yb, p.n_samples, thr, p.min_valid_ratio)
    on_axis = sum(1 for i, j in zip(want[0], want[1]) if (xb[j] - xa[i]) * 4 == (yb[j] - ya[i]) * 3)
    assert (on_axis > 100) if which == "just_above" else (on_axis == 0)
    cap = 512
    buf = m.Buffers(1, K, L, h, w, cap, 1 << 16, 16, DEV)
    buf.pcount.copy_(torch.tensor([[len(xa), len(xb)]], dtype=torch.int32))
    for t, v in ((buf.px, (xa, xb)), (buf.py, (ya, yb))):
        host = np.zeros((1, K, cap), np.int32)
        host[0, 0, :len(v[0])] = v[0]
        host[0, 1, :len(v[1])] = v[1]
        t.copy_(torch.from_numpy(host))
    paf_hi = m.hp_resize(to_dev(paf_lo))
    assert np.all(paf_hi[0, 0].cpu().numpy() == np.float32(0.0625))
    m.hp_score_limbs(paf_hi, m.Skeleton(K, [0], [1]), m.Params(p.peak_thr, thr, p.n_samples, p.min_valid_ratio, p.min_parts, 8), buf)
    assert buf.host_status() == 0
    assert_lists_equal("candidates", buf.host_cands()[0], [[want]])


PARAM_CASES = [
    dict(n_samples=2, min_valid_ratio=0.8),          # end points only
    dict(n_samples=3, min_valid_ratio=0.8),          # one interior sample: the one the screen looks at
    dict(n_samples=10, min_valid_ratio=1.0),         # no invalid sample allowed
    dict(n_samples=10, min_valid_ratio=0.0),         # nothing is ever rejected for invalid samples
    dict(n_samples=10, min_valid_ratio=0.55),        # more invalid samples allowed than the screen examines
    dict(n_samples=64, min_valid_ratio=0.8),         # HP_MAX_SAMPLES
    dict(n_samples=7, min_valid_ratio=0.8, paf_thr=-0.5, peak_thr=0.02),
    dict(n_samples=10, min_valid_ratio=0.8, min_parts=1),
    dict(n_samples=10, min_valid_ratio=0.8, min_parts=19),
]
# with a validity threshold of -0.5 nearly every pair of positive mean is a candidate (6 000 per limb here): more than
# the one-launch limb kernel is built for (1024), so that corner runs through the general kernels only
PARAM_LEGS = [(kw, path) for kw in PARAM_CASES for path in ("one_launch", "short_lists", "general")
              if path != "one_launch" or kw.get("paf_thr", 0.05) >= 0.0]


@pytest.mark.parametrize("kw,path", PARAM_LEGS,
                         ids=lambda v: v if isinstance(v, str) else "-".join(f"{a}{b}" for a, b in v.items()))
def test_postprocess_parameter_corners(kw, path):
    """Sample counts and validity ratios at their corners, through the one-launch limb kernel (small capacities),
    through the scorer for short lists (few peaks, many candidates allowed) and through the tiled scorer with its
    screen (large capacities)."""
    from synth import Params
    cfg = SynthConfig(30, COCO18, 2, 24, 31, 5, noise_sd=0.03, dropout=0.1, n_spurious=6)
    b = generate(cfg)
    p = Params(**{**dict(peak_thr=0.05, paf_thr=0.05, n_samples=10, min_valid_ratio=0.8, min_parts=3), **kw})
    sk = cfg.skeleton
    ora = oracle.postprocess(b.cm, b.paf, sk.limb_a, sk.limb_b, p, threads=8)
    pk = max(len(x[0]) for im in ora["peaks"] for x in im)
    cc = max(len(x[0]) for im in ora["candidates"] for x in im)
    pp = max(len(x[1]) for x in ora["poses"])
    m = hp()
    caps = {"general": (512, max(4096, cc + 8), max(64, pp + 8)),
            "short_lists": (max(16, pk + 8), max(2048, cc + 8), max(16, pp + 8)),
            "one_launch": (max(16, pk + 8), cc + 8, max(16, pp + 8))}[path]
    assert path == "general" or caps[0] <= 256
    assert path != "one_launch" or caps[1] <= 1024, "this leg is meant for the one-launch limb kernel"
    buf = m.Buffers(cfg.batch, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, *caps, DEV)
    prm = m.Params(p.peak_thr, p.paf_thr, p.n_samples, p.min_valid_ratio, p.min_parts, 8)
    m.hp_postprocess(to_dev(b.cm), to_dev(b.paf), skel_of(sk), prm, buf)
    check_all(buf, ora)


def _random_configs():
    """A spread of small workloads drawn from a fixed seed: sizes, people, noise, storage type,
    skeleton, truncation and clustering all vary together."""
    rng = np.random.default_rng(424242)
    out = []
    for k in range(14):
        sk = BODY25 if rng.random() < 0.35 else COCO18
        h, w = int(rng.integers(3, 40)), int(rng.integers(3, 56))
        out.append(SynthConfig(100 + k, sk, int(rng.integers(1, 5)), h, w, int(rng.integers(0, 9)),
                               scale_lo=20.0, scale_hi=float(rng.integers(40, 160)),
                               noise_sd=float(rng.choice([0.0, 0.01, 0.03, 0.06])),
                               dropout=float(rng.choice([0.0, 0.15, 0.3])), n_spurious=int(rng.integers(0, 12)),
                               truncation=bool(rng.random() < 0.4), clustered=bool(rng.random() < 0.3),
                               dtype="float16" if rng.random() < 0.4 else "float32"))
    return out


@pytest.mark.parametrize("form", ["fused", "materialised", "staged"])
@pytest.mark.parametrize("cfg", _random_configs(), ids=lambda c: f"rnd{c.index}-{c.skeleton.name}-{c.batch}x{c.h}x{c.w}-{c.dtype}")
def test_random_small_workloads(cfg, form):
    b = generate(cfg)
    ora = run_oracle(b, DEFAULT_PARAMS)
    caps = caps_for(ora)
    if cfg.index % 2:                    # every other one through the general kernels
        caps = (max(caps[0], 300), max(caps[1], 2048), caps[2])
    if form == "staged":
        buf, st = run_staged(b, ora, caps)
        assert st == [0, 0, 0]
    else:
        buf, _, _ = run_fused(b, ora, form == "materialised", caps)
    check_all(buf, ora)


def test_maximum_capacities():
    """The largest capacities the library accepts (16384 peaks per part, 2^20 candidates per limb):
    the launch shapes derived from them must be valid, whatever little the lists hold."""
    cfg = SynthConfig(40, COCO18, 1, 12, 15, 2, noise_sd=0.02)
    b = generate(cfg)
    sk = cfg.skeleton
    la, lb = sk.limb_a[:3], sk.limb_b[:3]
    paf = np.ascontiguousarray(b.paf[:, :6])
    ora = oracle.postprocess(b.cm, paf, la, lb, DEFAULT_PARAMS, threads=4)
    m = hp()
    buf = m.Buffers(1, sk.n_parts, 3, cfg.h, cfg.w, 16384, 1 << 20, 4096, DEV)
    skel = m.Skeleton(sk.n_parts, la, lb)
    m.hp_postprocess(to_dev(b.cm), to_dev(paf), skel, prm_of(), buf)
    check_all(buf, ora)
    # and the staged calls with the same buffers
    m.hp_find_peaks(m.hp_resize(to_dev(b.cm)), sk.n_parts, DEFAULT_PARAMS.peak_thr, buf)
    m.hp_score_limbs(m.hp_resize(to_dev(paf)), skel, prm_of(), buf)
    m.hp_assemble(skel, prm_of(), buf)
    check_all(buf, ora)
