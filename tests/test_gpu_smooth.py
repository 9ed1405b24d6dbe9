"""GPU parity of the optional smoothing step (hp_smooth) against its oracle: every float bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from synth import CONFIGS, BENCH_CAPS, generate, gaussian_taps, DEFAULT_PARAMS

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def hp():
    import paper_2108_11826_amd as m
    return m


CASES = [
    dict(N=2, C_mem=3, C=2, H=37, W=53, taps=gaussian_taps(3.0, 8)),
    dict(N=1, C_mem=1, C=1, H=1, W=1, taps=gaussian_taps(3.0, 8)),
    dict(N=1, C_mem=2, C=2, H=130, W=67, taps=np.array([0.25, -0.5, 2.0, 0.125, 0.5], np.float32)),
    dict(N=1, C_mem=1, C=1, H=64, W=64, taps=gaussian_taps(9.0, 32)),          # the longest tap vector
    dict(N=3, C_mem=4, C=3, H=200, W=131, taps=gaussian_taps(4.0, 12)),
    dict(N=1, C_mem=2, C=1, H=65, W=129, taps=np.array([1.0], np.float32)),
    dict(N=2, C_mem=2, C=2, H=3, W=300, taps=np.array([0.25, 0.5, 0.25], np.float32)),
    dict(N=1, C_mem=1, C=1, H=300, W=2, taps=gaussian_taps(2.0, 5)),
    # rows of whole 16-byte groups with 5, 9, 13 or 17 taps take the kernel that walks down strips:
    # one and several strips, ragged last strip, a map narrower than the halo, one row, bands that end mid-pass
    dict(N=2, C_mem=3, C=2, H=45, W=64, taps=gaussian_taps(1.0, 2)),
    dict(N=1, C_mem=2, C=2, H=100, W=260, taps=gaussian_taps(2.0, 4)),
    dict(N=1, C_mem=1, C=1, H=33, W=4, taps=gaussian_taps(2.5, 6)),
    dict(N=1, C_mem=1, C=1, H=1, W=512, taps=gaussian_taps(2.5, 6)),
    dict(N=1, C_mem=2, C=2, H=300, W=1028, taps=np.linspace(-1.0, 2.0, 9).astype(np.float32)),
    dict(N=3, C_mem=20, C=19, H=17, W=8, taps=gaussian_taps(1.0, 2)),
    dict(N=1, C_mem=5, C=4, H=2048, W=2048 * 4, taps=gaussian_taps(3.0, 8)),         # 67 M pixels: 17 taps, marching
    # strips overlap by the taps' reach rounded up to 16-byte pieces: widths on both sides of one strip's and two
    # strips' output columns, for every tap count the kernel is built for (17 taps: 240 columns a strip; 5: 248)
    dict(N=1, C_mem=1, C=1, H=40, W=240, taps=gaussian_taps(3.0, 8)),
    dict(N=1, C_mem=1, C=1, H=40, W=244, taps=gaussian_taps(3.0, 8)),
    dict(N=1, C_mem=2, C=2, H=23, W=484, taps=gaussian_taps(3.0, 8)),
    dict(N=2, C_mem=2, C=2, H=19, W=656, taps=gaussian_taps(3.0, 8)),
    dict(N=1, C_mem=1, C=1, H=18, W=248, taps=gaussian_taps(1.0, 2)),
    dict(N=1, C_mem=1, C=1, H=18, W=252, taps=gaussian_taps(1.0, 2)),
    dict(N=1, C_mem=1, C=1, H=50, W=500, taps=gaussian_taps(2.5, 6)),
    dict(N=1, C_mem=1, C=1, H=9, W=12, taps=np.linspace(0.5, -0.25, 17).astype(np.float32)),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "%dx%dx%dx%d-t%d" % (c["N"], c["C"], c["H"], c["W"], len(c["taps"])))
def test_smooth_bit_exact(case):
    m = hp()
    rng = np.random.default_rng(len(case["taps"]) + case["H"])
    maps = (rng.random((case["N"], case["C_mem"], case["H"], case["W"]), dtype=np.float32) - 0.25).astype(np.float32)
    out = torch.full(maps.shape, -7.0, dtype=torch.float32, device=DEV)
    m.hp_smooth(torch.from_numpy(maps).to(DEV), torch.from_numpy(case["taps"]).to(DEV), channels=case["C"], out=out)
    got = out.cpu().numpy()
    want = oracle.smooth(maps[:, :case["C"]], case["taps"])
    assert np.array_equal(got[:, :case["C"]].view(np.uint32), want.view(np.uint32))
    assert np.all(got[:, case["C"]:] == -7.0)                # channels beyond C are left alone


def test_smoothed_peaks_of_a_full_workload():
    # configs[2]: upsample, smooth the 18 part channels (sigma 3, 17 taps), find peaks; the oracle does the same
    m = hp()
    cfg = CONFIGS[2]
    sk = cfg.skeleton
    b = generate(cfg)
    taps = gaussian_taps(3.0, 8)
    cm_hi = m.hp_resize(torch.from_numpy(b.cm).to(DEV))
    sm = m.hp_smooth(cm_hi, torch.from_numpy(taps).to(DEV), channels=sk.n_parts)
    cap, ccap, pcap = BENCH_CAPS[2]
    buf = m.Buffers(cfg.batch, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, cap, ccap, pcap, DEV)
    m.hp_find_peaks(sm, sk.n_parts, DEFAULT_PARAMS.peak_thr, buf)
    assert buf.host_status() == 0
    peaks, _ = buf.host_peaks()
    got = sm.cpu().numpy()
    for n in (0, cfg.batch - 1):
        want = oracle.smooth(oracle.resize(b.cm[n, :sk.n_parts], 8), taps)
        assert np.array_equal(got[n, :sk.n_parts].view(np.uint32), want.view(np.uint32))
        for c in range(sk.n_parts):
            ox, oy, os_ = oracle.find_peaks(want[c], DEFAULT_PARAMS.peak_thr)
            gx, gy, gs = peaks[n][c]
            assert np.array_equal(gx, ox) and np.array_equal(gy, oy)
            assert np.array_equal(np.asarray(gs).view(np.uint32), np.asarray(os_).view(np.uint32))
        # smoothing removes the noise peaks: fewer peaks than on the raw maps
    raw = sum(len(oracle.find_peaks(oracle.resize(b.cm[0, c], 8), DEFAULT_PARAMS.peak_thr)[0]) for c in range(sk.n_parts))
    smooth = sum(len(peaks[0][c][0]) for c in range(sk.n_parts))
    assert 0 < smooth <= raw


@pytest.mark.parametrize("smoothed", [False, True], ids=["raw", "smoothed"])
def test_refined_peak_positions(smoothed):
    # the staged route with the optional steps: upsample, (smooth,) find peaks, refine; every float against the oracle
    m = hp()
    cfg = CONFIGS[1]
    sk = cfg.skeleton
    b = generate(cfg)
    taps = gaussian_taps(3.0, 8)
    maps = m.hp_resize(torch.from_numpy(b.cm).to(DEV))
    if smoothed:
        maps = m.hp_smooth(maps, torch.from_numpy(taps).to(DEV), channels=sk.n_parts)
    cap, ccap, pcap = BENCH_CAPS[1]
    buf = m.Buffers(cfg.batch, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, cap, ccap, pcap, DEV)
    m.hp_find_peaks(maps, sk.n_parts, DEFAULT_PARAMS.peak_thr, buf)
    xf, yf = m.hp_refine_peaks(maps, sk.n_parts, buf)
    xf, yf = xf.cpu().numpy(), yf.cpu().numpy()
    peaks, _ = buf.host_peaks()
    moved = 0
    for c in range(sk.n_parts):
        plane = oracle.resize(b.cm[0, c], 8)
        if smoothed:
            plane = oracle.smooth(plane, taps)
        ox, oy, _ = oracle.find_peaks(plane, DEFAULT_PARAMS.peak_thr)
        assert np.array_equal(peaks[0][c][0], ox) and np.array_equal(peaks[0][c][1], oy)
        wx, wy = oracle.refine_peaks(plane, ox, oy)
        k = len(ox)
        assert np.array_equal(xf[0, c, :k].view(np.uint32), wx.view(np.uint32))
        assert np.array_equal(yf[0, c, :k].view(np.uint32), wy.view(np.uint32))
        assert np.all(xf[0, c, k:] == 0) and np.all(yf[0, c, k:] == 0)      # entries beyond the count are untouched
        moved += int(np.count_nonzero(wx != ox) + np.count_nonzero(wy != oy))
    assert moved > 0
