"""hp_postprocess_static (the entry point that allocates nothing: its workspace is a fixed array in the
library's device image) against hp_postprocess, through the C ABI: every output bit for bit, on calls
that follow each other on one GPU with different sizes, so that the second finds the first's leftovers
in the array."""

import numpy as np
import pytest
import torch

from synth import CONFIGS, BENCH_CAPS, COCO18, BODY25, SynthConfig, generate, DEFAULT_PARAMS as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def hp():
    import paper_2108_11826_amd as m
    return m


def outputs(buf):
    """Every output tensor of a call, trimmed to what the counts say is defined."""
    torch.cuda.synchronize()
    return (buf.host_status(), buf.host_peaks(), buf.host_cands(), buf.host_conns(), buf.host_poses())


def same(a, b):
    if isinstance(a, (tuple, list)):
        return len(a) == len(b) and all(same(x, y) for x, y in zip(a, b))
    if isinstance(a, np.ndarray):
        if a.dtype == np.float32:
            return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))
        return np.array_equal(a, b)
    return a == b


def both(cfg, caps, materialise=False):
    m = hp()
    sk = cfg.skeleton
    b = generate(cfg)
    N = b.cm.shape[0]
    cm, paf = torch.from_numpy(b.cm).to(DEV), torch.from_numpy(b.paf).to(DEV)
    skel = m.Skeleton(sk.n_parts, sk.limb_a, sk.limb_b)
    prm = m.Params(P.peak_thr, P.paf_thr, P.n_samples, P.min_valid_ratio, P.min_parts, P.scale)
    his = [None, None]
    if materialise:
        his = [torch.empty((N, c, cfg.H, cfg.W), dtype=torch.float32, device=DEV) for c in (sk.n_parts + 1, 2 * sk.n_limbs)]
    ref_buf = m.Buffers(N, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, *caps, DEV)
    m.hp_postprocess(cm, paf, skel, prm, ref_buf, *his)
    ref = outputs(ref_buf)
    ref_hi = [t.clone() for t in his] if materialise else None
    got_buf = m.Buffers(N, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, *caps, DEV)
    if materialise:
        for t in his:
            t.zero_()
    m.hp_postprocess_static(cm, paf, skel, prm, got_buf, *his)
    got = outputs(got_buf)
    assert ref[0] == 0 and ref[4][1].sum() > 0            # the reference call found persons
    assert same(got, ref), f"workload {cfg.index}"
    if materialise:
        assert all(torch.equal(a, b) for a, b in zip(his, ref_hi))


def test_two_calls_in_a_row_the_second_smaller():
    print("static workspace: workload 2 (batch 8, 46x82) then workload 0 (batch 1, 46x46)", flush=True)
    both(CONFIGS[2], BENCH_CAPS[2])
    both(CONFIGS[0], BENCH_CAPS[0])


def test_sizes_follow_each_other_in_any_order():
    """Layouts of different calls overlap in the array: list counters of one call lie where another staged its lists."""
    print("static workspace: mixed sizes, general kernels and fp16", flush=True)
    small = SynthConfig(13, COCO18, 3, 33, 47, 6, noise_sd=0.02, dropout=0.1, n_spurious=10)
    half = SynthConfig(14, BODY25, 2, 31, 65, 5, noise_sd=0.02, dtype="float16")
    both(small, (64, 256, 32))
    both(CONFIGS[2], BENCH_CAPS[2], materialise=True)
    both(half, (300, 2048, 32))                  # capacities beyond the one-launch limb kernel: the general kernels
    both(CONFIGS[1], BENCH_CAPS[1])
    both(small, (32, 64, 16))


def test_sizes_beyond_the_array_are_rejected():
    m = hp()
    from paper_2108_11826_amd import binding as B
    cfg = CONFIGS[3]
    sk = cfg.skeleton
    caps = BENCH_CAPS[3]
    assert m.hp_workspace_bytes(cfg.batch, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, 8, *caps) > 8 << 20
    cm = torch.zeros((cfg.batch, sk.n_parts + 1, cfg.h, cfg.w), device=DEV)
    paf = torch.zeros((cfg.batch, 2 * sk.n_limbs, cfg.h, cfg.w), device=DEV)
    buf = m.Buffers(cfg.batch, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, *caps, DEV)
    buf.pose_count.fill_(-7)
    with pytest.raises(B.HPError) as e:
        m.hp_postprocess_static(cm, paf, m.Skeleton(sk.n_parts, sk.limb_a, sk.limb_b), m.Params(), buf)
    assert e.value.code == -3
    torch.cuda.synchronize()
    assert int(buf.pose_count[0]) == -7                  # nothing was enqueued
