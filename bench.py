"""Benchmark: post-processed frames/s of hp_postprocess on synthetic CM/PAF tensors, with the
roofline of the dominant HBM-bound kernel and the CPU oracle timed beside it.

A step is one hp_postprocess call (upsampling, peak NMS, compaction, limb scoring, matching,
assembly) over one batch that is already resident in HBM.  `value` is measured on the form
that keeps the upsampled maps in registers, with the steps issued round-robin on a few HIP
streams (each with its own output buffers and workspace) so that consecutive batches overlap,
as the operators of the paper's streaming dataflow do (Section 2.2.1); the one-stream rate is
reported beside it.  The same number of steps is then timed on the form that materialises the
hi-res maps (its upsampling kernel is the HBM-bound one the roofline object describes), and
once more with per-kernel event stamps for the kernel times.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# plain (non-packed) fp32 lane operations: 256 CUs x 4 SIMDs x 16 lanes/clk x 2.4 GHz
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=2, help="index into the synthetic workloads (2 = 656x368 batch 8)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU work spent on the oracle baseline (0 = skip)")
    ap.add_argument("--streams", type=int, default=3, help="HIP streams the timed steps are spread over")
    ap.add_argument("--no-streaming", action="store_true", help="skip the streaming-front measurement")
    ap.add_argument("--streaming-sweep", action="store_true",
                    help="print one JSON line per (batch slot, offered load) point of the streaming front and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain device copies of a known size (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (images are independent; "
              "a batch would be split across GPUs with no communication). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2108_11826_amd as hp
    from synth import CONFIGS, BENCH_CAPS, generate, DEFAULT_PARAMS as P

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    cfg = CONFIGS[args.config]
    sk = cfg.skeleton
    N, K, L, h, w = cfg.batch, sk.n_parts, sk.n_limbs, cfg.h, cfg.w
    batch = generate(cfg)
    cm, paf = torch.from_numpy(batch.cm).to(dev), torch.from_numpy(batch.paf).to(dev)
    skel = hp.Skeleton(K, sk.limb_a, sk.limb_b)
    prm = hp.Params(P.peak_thr, P.paf_thr, P.n_samples, P.min_valid_ratio, P.min_parts, P.scale)
    cap, ccap, pcap = BENCH_CAPS[args.config]
    buf = hp.Buffers(N, K, L, h, w, cap, ccap, pcap, dev)
    cm_hi = torch.empty((N, K + 1, cfg.H, cfg.W), dtype=torch.float32, device=dev)
    paf_hi = torch.empty((N, 2 * L, cfg.H, cfg.W), dtype=torch.float32, device=dev)

    def streaming_point(max_batch, depth, n_lanes, offered_fps, n_frames, copy):
        """Frames handed one at a time to the streaming front (hp_batcher_*) at a fixed rate (0 = as fast as they are
        taken): achieved rate, mean batch size (per batch) and the delay from a frame's arrival to its result."""
        lanes = hp.BatcherLanes(n_lanes, max_batch, K, L, h, w, cap, ccap, pcap, cm.dtype, dev)
        reps = (max_batch + N - 1) // N
        for l in range(n_lanes):
            lanes.cm[l].copy_(cm.repeat(reps, 1, 1, 1)[:max_batch])
            lanes.paf[l].copy_(paf.repeat(reps, 1, 1, 1)[:max_batch])
        torch.cuda.synchronize()
        bt = hp.hp_batcher_create(skel, prm, lanes, depth)
        gap = int(round(1e9 / offered_fps)) if offered_fps else 0
        src = (cm, paf) if copy else (None, None)
        hp.hp_batcher_drive(bt, min(200, n_frames), gap, *src)
        lat, size, elapsed = hp.hp_batcher_drive(bt, n_frames, gap, *src)
        hp.hp_batcher_destroy(bt)
        return {"max_batch": max_batch, "batches_in_flight": depth, "lanes": n_lanes,
                "frames": "copied into the slot (one launch per frame)" if copy else "already in the slot",
                "offered_fps": offered_fps if offered_fps else "unlimited", "fps": round(n_frames / elapsed * 1e9, 1),
                "mean_batch": round(float(np.mean(1.0 / size)) ** -1, 2),
                "latency_us_p50": round(float(np.percentile(lat, 50)) / 1e3, 1),
                "latency_us_p99": round(float(np.percentile(lat, 99)) / 1e3, 1)}

    if args.streaming_sweep:
        for copy in (True, False):
            for mb, depth, n_lanes in ((1, 2, 3), (N, 1, 3), (N, 2, 4), (N, 3, 5), (4 * N, 2, 4)):
                for load in (10_000, 50_000, 100_000, 200_000, 400_000, 0):
                    print(json.dumps(streaming_point(mb, depth, n_lanes, load, 4000, copy)), flush=True)
        return

    call_fused = hp.PostprocessCall(cm, paf, skel, prm, buf)
    call_mat = hp.PostprocessCall(cm, paf, skel, prm, buf, cm_hi, paf_hi)

    def step(materialise):
        (call_mat if materialise else call_fused)()

    def timed(materialise):
        for _ in range(args.warmup):
            step(materialise)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(materialise)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # several batches in flight: every stream owns its outputs and workspace, the inputs are shared
    n_streams = max(1, args.streams)
    lanes = [(torch.cuda.Stream(), hp.Buffers(N, K, L, h, w, cap, ccap, pcap, dev)) for _ in range(n_streams)]
    torch.cuda.synchronize()
    calls = [hp.PostprocessCall(cm, paf, skel, prm, bf, stream=st) for st, bf in lanes]

    def timed_streams():
        def run(k):
            for i in range(k):
                calls[i % n_streams]()
        run(max(args.warmup, 2 * n_streams))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(args.steps)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # correctness gate (outside the timed regions): the timed launch configuration against the oracle
    import oracle
    ora = oracle.postprocess(batch.cm, batch.paf, sk.limb_a, sk.limb_b, P, threads=min(16, len(os.sched_getaffinity(0))))
    parity = True
    for materialise in (False, True):
        step(materialise)
        torch.cuda.synchronize()
        poses, _ = buf.host_poses()
        peaks, _ = buf.host_peaks()
        ok = buf.host_status() == 0
        for n in range(N):
            ok = ok and np.array_equal(poses[n][0], ora["poses"][n][0]) and np.array_equal(poses[n][2], ora["poses"][n][2])
            for c in range(K):
                ok = ok and all(np.array_equal(peaks[n][c][q], ora["peaks"][n][c][q]) for q in range(3))
        parity = parity and bool(ok)

    if args.calibrate_copy:
        # a plain copy of exactly 256 MiB in and 256 MiB out, for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    t_fused = timed(False)
    t_multi = timed_streams()
    for st, bf in lanes:                      # every lane must hold the oracle's persons too
        poses, _ = bf.host_poses()
        ok = bf.host_status() == 0 and all(np.array_equal(poses[n][0], ora["poses"][n][0]) and
                                           np.array_equal(poses[n][2], ora["poses"][n][2]) for n in range(N))
        parity = parity and bool(ok)
    t_mat = timed(True)

    # per-kernel times: the same steps again with every launch stamped by a pair of events
    hp.hp_profile_begin(2 * args.steps * 8)
    for _ in range(args.steps):
        step(False)
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    prof = hp.hp_profile_end()
    kern_us = {k: 1e3 * ms / n for k, (ms, n) in prof.items()}

    # the staged calls (hp_resize -> hp_find_peaks -> hp_score_limbs -> hp_assemble) on the materialised
    # maps: their peak search reads the hi-res confidence maps from HBM, the general scorer gathers PAFs
    staged_steps = max(3, min(args.steps, 50))

    def staged():
        hp.hp_find_peaks(cm_hi, K, P.peak_thr, buf)
        hp.hp_score_limbs(paf_hi, skel, prm, buf)
        hp.hp_assemble(skel, prm, buf)

    step(True)
    staged()
    torch.cuda.synchronize()
    poses, _ = buf.host_poses()
    ok = buf.host_status() == 0 and all(np.array_equal(poses[n][0], ora["poses"][n][0]) and
                                        np.array_equal(poses[n][2], ora["poses"][n][2]) for n in range(N))
    parity = parity and bool(ok)
    hp.hp_profile_begin(staged_steps * 8)
    for _ in range(staged_steps):
        staged()
    torch.cuda.synchronize()
    staged_us = {k: 1e3 * ms / n for k, (ms, n) in hp.hp_profile_end().items()}

    # what a plain fill of the same number of bytes reaches on this GPU (the practical ceiling of a
    # write-dominated kernel), timed with events on the same stream
    fill_t = torch.empty(((cm_hi.numel() + paf_hi.numel()),), dtype=torch.float32, device=dev)
    for _ in range(3):
        fill_t.fill_(1.0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fills = 20
    e0.record()
    for _ in range(fills):
        fill_t.fill_(1.0)
    e1.record()
    torch.cuda.synchronize()
    fill_us = 1e3 * e0.elapsed_time(e1) / fills
    fill_gbs = fill_t.numel() * 4 / (fill_us * 1e-6) / 1e9
    del fill_t

    n_pairs = sum(len(ora["peaks"][n][a][0]) * len(ora["peaks"][n][b][0]) for n in range(N) for a, b in sk.limbs)
    esz = batch.cm.dtype.itemsize
    lo_bytes = (batch.cm.size + batch.paf.size) * esz
    hi_bytes = (cm_hi.numel() + paf_hi.numel()) * 4
    k1_bytes = lo_bytes + hi_bytes
    k1_us = kern_us["resize_write"]
    achieved = k1_bytes / (k1_us * 1e-6) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_resize_write_cfg{args.config}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")
    roofline = {"kernel": "k_resize_write (x8 upsampling of all CM+PAF channels into materialised hi-res maps; "
                          "dominant kernel of the materialising form)",
                "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "bytes_per_launch": k1_bytes, "us_per_launch": round(k1_us, 2),
                "plain_fill_same_bytes": {"us": round(fill_us, 2), "GB/s": round(fill_gbs, 1),
                                          "frac_of_fill": round(achieved / fill_gbs, 4)}}
    # staged peak search: reads K of the K+1 hi-res confidence maps once, writes peaks only
    nms_bytes = N * K * cfg.H * cfg.W * 4
    nms_ach = nms_bytes / (staged_us["nms_hi"] * 1e-6) / 1e9
    roofline_nms_hi = {"kernel": "k_nms_hi_strip (hp_find_peaks: 3x3 thresholded NMS on the materialised hi-res CMs)",
                       "bound": "hbm", "achieved": round(nms_ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(nms_ach / HBM_PEAK_GBS, 4), "bytes_per_launch": nms_bytes,
                       "us_per_launch": round(staged_us["nms_hi"], 2)}
    # fused form: nothing but the lo-res CM is read; the bound is the plain ALUs
    cm_px = N * K * cfg.H * cfg.W
    fused_us = kern_us["resize_nms"]
    fused_ach = 12.0 * cm_px / (fused_us * 1e-6) / 1e12
    roofline_fused = {"kernel": "k_resize_nms (maps kept in registers; dominant kernel of the timed step)",
                      "bound": "alu", "achieved": round(fused_ach, 2), "peak": round(ALU_PEAK_TLANEOPS, 1),
                      "unit": "Tlane-op/s", "frac": round(fused_ach / ALU_PEAK_TLANEOPS, 4),
                      "ops_per_launch": 12 * cm_px, "us_per_launch": round(fused_us, 2),
                      "note": "ops are those of the dense definition (12 lane-ops per hi-res CM pixel); the kernel "
                              "skips tiles whose nine source nodes cannot reach the threshold, so it executes fewer",
                      "hbm_bytes_per_launch": batch.cm[:, :K].size * esz}
    score_bytes = 80.0 * n_pairs
    lo_name = "limb_small" if "limb_small" in kern_us else "score_lo"
    roofline_scoring = {"kernel": "k_score<float, true> (hp_score_limbs: limb scoring with PAFs gathered from the "
                                  "materialised maps; 80 useful bytes per pair, 4-byte gathers)",
                        "bound": "hbm",
                        "achieved": round(score_bytes / (staged_us["score_hi"] * 1e-6) / 1e9, 2),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(score_bytes / (staged_us["score_hi"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 6),
                        "bytes_per_launch": score_bytes, "pairs_per_launch": n_pairs,
                        "us_per_launch": round(staged_us["score_hi"], 2),
                        "us_per_launch_lo_res_form": round(kern_us[lo_name], 2),
                        "lo_res_form_kernel": lo_name}

    # the operator before the network (decoded frames -> resized channel-first tensor), at the frame size of
    # the paper's benchmark video and the input size of this workload's network, on a batch large enough to
    # be bandwidth-bound
    pre_frames = 64
    pre_src = torch.randint(0, 256, (pre_frames, 360, 640, 3), dtype=torch.uint8, device=dev)
    pre_dst = torch.empty((pre_frames, 3, cfg.H, cfg.W), dtype=torch.float32, device=dev)
    for _ in range(3):
        hp.hp_preprocess(pre_src, cfg.H, cfg.W, 1 / 255.0, 0.0, True, out=pre_dst)
    torch.cuda.synchronize()
    hp.hp_profile_begin(64)
    for _ in range(20):
        hp.hp_preprocess(pre_src, cfg.H, cfg.W, 1 / 255.0, 0.0, True, out=pre_dst)
    torch.cuda.synchronize()
    ms, nl = hp.hp_profile_end()["preprocess"]
    pre_us = 1e3 * ms / nl
    pre_bytes = pre_src.numel() + pre_dst.numel() * 4
    pre_ok = bool(np.array_equal(pre_dst[pre_frames - 1].cpu().numpy(),
                                 oracle.preprocess(pre_src[pre_frames - 1:].cpu().numpy(), cfg.H, cfg.W, 1 / 255.0, 0.0, True)[0]))
    parity = parity and pre_ok
    preprocess = {"kernel": "k_preprocess (hp_preprocess: 640x360 8-bit interleaved frames -> %dx%d fp32 channel-first)" % (cfg.W, cfg.H),
                  "frames_per_launch": pre_frames, "us_per_launch": round(pre_us, 2),
                  "frames_per_s": round(pre_frames / (pre_us * 1e-6), 1),
                  "roofline": {"bound": "hbm", "achieved": round(pre_bytes / (pre_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": round(pre_bytes / (pre_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                               "bytes_per_launch": pre_bytes},
                  "parity_with_oracle": pre_ok}
    del pre_src, pre_dst

    # the optional smoothing of the upsampled confidence maps (a 17-tap sampled Gaussian, sigma 3) on this workload's maps
    from synth import gaussian_taps
    taps_np = gaussian_taps(3.0, 8)
    taps_dev = torch.from_numpy(taps_np).to(dev)
    hp.hp_resize(cm, cm_hi)
    sm_dst = torch.empty_like(cm_hi)
    for _ in range(3):
        hp.hp_smooth(cm_hi, taps_dev, channels=K, out=sm_dst)
    torch.cuda.synchronize()
    hp.hp_profile_begin(64)
    for _ in range(20):
        hp.hp_smooth(cm_hi, taps_dev, channels=K, out=sm_dst)
    torch.cuda.synchronize()
    ms, nl = hp.hp_profile_end()["smooth"]
    sm_us = 1e3 * ms / nl
    sm_px = N * K * cfg.H * cfg.W
    sm_ok = bool(np.array_equal(sm_dst[N - 1, K - 1].cpu().numpy(),
                                oracle.smooth(oracle.resize(batch.cm[N - 1, K - 1], 8), taps_np)))
    parity = parity and sm_ok
    sm_fma = sm_px * len(taps_np) * (1 + (64 + len(taps_np) - 1) / 64)
    smooth = {"kernel": "k_smooth (hp_smooth: separable %d-tap smoothing of the %d part maps per image, %dx%d)" % (len(taps_np), K, cfg.W, cfg.H),
              "us_per_launch": round(sm_us, 2),
              "roofline": {"bound": "hbm", "achieved": round(8 * sm_px / (sm_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": round(8 * sm_px / (sm_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "bytes_per_launch": 8 * sm_px},
              "alu": {"achieved": round(sm_fma / (sm_us * 1e-6) / 1e12, 2), "peak": round(ALU_PEAK_TLANEOPS, 1), "unit": "Tfma/s",
                      "frac": round(sm_fma / (sm_us * 1e-6) / 1e12 / ALU_PEAK_TLANEOPS, 4)},
              "parity_with_oracle": sm_ok}
    del sm_dst

    # the operator after post-processing (poses drawn on the original frames), on the same 64 frames of the benchmark
    # video's size, with the poses of this workload's batch repeated
    reps = pre_frames // N
    vbuf = hp.Buffers(reps * N, K, L, h, w, cap, ccap, pcap, dev)
    hp.hp_postprocess(cm.repeat(reps, 1, 1, 1), paf.repeat(reps, 1, 1, 1), skel, prm, vbuf)
    vis_src = torch.randint(0, 256, (reps * N, 360, 640, 3), dtype=torch.uint8, device=dev)
    vis_dst = torch.empty_like(vis_src)
    vrng = np.random.default_rng(7)
    limb_rgb, part_rgb = vrng.integers(0, 256, (L, 3), dtype=np.uint8), vrng.integers(0, 256, (K, 3), dtype=np.uint8)
    for _ in range(3):
        hp.hp_draw_poses(vis_src, cfg.H, cfg.W, skel, vbuf, limb_rgb, part_rgb, 4, 4, out=vis_dst)
    torch.cuda.synchronize()
    hp.hp_profile_begin(64)
    for _ in range(20):
        hp.hp_draw_poses(vis_src, cfg.H, cfg.W, skel, vbuf, limb_rgb, part_rgb, 4, 4, out=vis_dst)
    torch.cuda.synchronize()
    pr = hp.hp_profile_end()
    list_us, tiles_us = 1e3 * pr["draw_list"][0] / pr["draw_list"][1], 1e3 * pr["draw"][0] / pr["draw"][1]
    vis_bytes = 2 * vis_src.numel()
    vpeaks, _ = vbuf.host_peaks()
    vposes, _ = vbuf.host_poses()
    vpx, vpy = np.zeros((1, K, cap), np.int32), np.zeros((1, K, cap), np.int32)
    for c in range(K):
        vpx[0, c, :len(vpeaks[N - 1][c][0])], vpy[0, c, :len(vpeaks[N - 1][c][1])] = vpeaks[N - 1][c][0], vpeaks[N - 1][c][1]
    vis_ok = bool(np.array_equal(vis_dst[N - 1].cpu().numpy(),
                                 oracle.draw_poses(vis_src[N - 1:N].cpu().numpy(), cfg.H, cfg.W, sk.limb_a, sk.limb_b, vpx, vpy,
                                                   [vposes[N - 1][0]], limb_rgb, part_rgb, 4, 4)[0]))
    parity = parity and vis_ok
    visualise = {"kernel": "k_draw_list + k_draw_tiles (hp_draw_poses: the batch's poses drawn on 640x360 8-bit frames, "
                           "thickness 4, radius 4)",
                 "frames_per_launch": reps * N, "persons_per_frame": round(float(vbuf.pose_count.float().mean()), 1),
                 "us_per_call": round(list_us + tiles_us, 2), "us_list": round(list_us, 2), "us_tiles": round(tiles_us, 2),
                 "frames_per_s": round(reps * N / ((list_us + tiles_us) * 1e-6), 1),
                 "roofline": {"kernel": "k_draw_tiles", "bound": "hbm", "achieved": round(vis_bytes / (tiles_us * 1e-6) / 1e9, 1),
                              "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": round(vis_bytes / (tiles_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                              "bytes_per_launch": vis_bytes},
                 "parity_with_oracle": vis_ok}
    del vis_src, vis_dst, vbuf

    # the second algorithm class: pose-proposal post-processing on a synthetic batch (12 x 12 grid, 19 parts, 9 x 9 neighbourhood)
    from synth import PPConfig, PP_COCO19, generate_pp
    pp_cfg = PPConfig(101, PP_COCO19, 8, 12, 12, 4, dropout=0.1)
    pp_in = generate_pp(pp_cfg)
    pp_sk = pp_cfg.skeleton
    pp_t = [torch.from_numpy(np.ascontiguousarray(pp_in[k])).to(dev) for k in ("resp", "conf", "box", "edge")]
    pp_buf = hp.PPBuffers(pp_cfg.batch, pp_sk.n_parts, 64, 32, dev)
    pp_skel = hp.Skeleton(pp_sk.n_parts, pp_sk.limb_a, pp_sk.limb_b)
    pp_call = lambda: hp.hp_pp_decode(*pp_t, pp_skel, pp_buf, pp_cfg.img_w, pp_cfg.img_h, pp_cfg.det_thr, pp_cfg.nms_thr,
                                      pp_cfg.edge_thr, pp_cfg.min_parts)
    for _ in range(3):
        pp_call()
    torch.cuda.synchronize()
    hp.hp_profile_begin(256)
    for _ in range(20):
        pp_call()
    torch.cuda.synchronize()
    pr = hp.hp_profile_end()
    t0 = time.perf_counter()
    for _ in range(200):
        pp_call()
    torch.cuda.synchronize()
    pp_us = (time.perf_counter() - t0) / 200 * 1e6
    pp_got = pp_buf.host()
    pp_ora = oracle.pp_decode(pp_in["resp"], pp_in["conf"], pp_in["box"], pp_in["edge"], pp_sk.limb_a, pp_sk.limb_b, pp_cfg.img_w,
                              pp_cfg.img_h, pp_cfg.det_thr, pp_cfg.nms_thr, pp_cfg.edge_thr, pp_cfg.min_parts)
    pp_ok = pp_got["status"] == 0 and all(
        np.array_equal(pp_got["poses"][n][0], pp_ora["poses"][n][0]) and np.array_equal(pp_got["poses"][n][2], pp_ora["poses"][n][2])
        and all(np.array_equal(pp_got["dets"][n][k][0], pp_ora["dets"][n][k][0]) for k in range(pp_sk.n_parts))
        for n in range(pp_cfg.batch))
    parity = parity and bool(pp_ok)
    pose_proposal = {"what": "hp_pp_decode: batch %d, %dx%d grid, %d parts, %dx%d neighbourhood, %d planted persons per image"
                             % (pp_cfg.batch, pp_cfg.Gh, pp_cfg.Gw, pp_sk.n_parts, pp_cfg.Nh, pp_cfg.Nw, pp_cfg.n_people),
                     "us_per_call": round(pp_us, 2), "frames_per_s": round(pp_cfg.batch / (pp_us * 1e-6), 1),
                     "kernel_us": {k: round(1e3 * ms / nl, 2) for k, (ms, nl) in sorted(pr.items())},
                     "bound": "latency (a few KB per image: one wavefront walks the limb tree of an image)",
                     "parity_with_oracle": bool(pp_ok)}

    # the third algorithm class: composite-field decoding on a synthetic batch (46 x 82 grid, stride 8, 17 parts, 19 limbs)
    from synth import CF_CONFIGS, generate_cf
    cf_cfg = CF_CONFIGS[2]
    cf_in = generate_cf(cf_cfg)
    cf_sk = cf_cfg.skeleton
    cf_pif, cf_paf = (torch.from_numpy(cf_in[k]).to(dev) for k in ("pif", "paf"))
    cf_buf = hp.CFBuffers(cf_cfg.batch, cf_sk.n_parts, cf_sk.n_limbs, 128, 256, 32, dev)
    cf_skel = hp.Skeleton(cf_sk.n_parts, cf_sk.limb_a, cf_sk.limb_b)
    cf_prm = (cf_cfg.stride, cf_cfg.pif_thr, cf_cfg.paf_thr, cf_cfg.seed_thr, cf_cfg.grow_thr, cf_cfg.rev_tol, cf_cfg.min_parts)
    cf_call = lambda: hp.hp_cf_decode(cf_pif, cf_paf, cf_skel, cf_buf, *cf_prm)
    for _ in range(3):
        cf_call()
    torch.cuda.synchronize()
    hp.hp_profile_begin(256)
    for _ in range(20):
        cf_call()
    torch.cuda.synchronize()
    pr = hp.hp_profile_end()
    t0 = time.perf_counter()
    for _ in range(100):
        cf_call()
    torch.cuda.synchronize()
    cf_us = (time.perf_counter() - t0) / 100 * 1e6
    # the same call with three batches in flight on separate streams (own outputs and workspace each), as for the headline
    cf_lanes = [(torch.cuda.Stream(), hp.CFBuffers(cf_cfg.batch, cf_sk.n_parts, cf_sk.n_limbs, 128, 256, 32, dev)) for _ in range(3)]
    torch.cuda.synchronize()

    def cf_round(reps):
        for i in range(reps):
            st, b = cf_lanes[i % 3]
            with torch.cuda.stream(st):
                hp.hp_cf_decode(cf_pif, cf_paf, cf_skel, b, *cf_prm)
        torch.cuda.synchronize()

    cf_round(6)
    t0 = time.perf_counter()
    cf_round(150)
    cf_us3 = (time.perf_counter() - t0) / 150 * 1e6
    cf_same_lanes = all(torch.equal(b.xyv, cf_buf.xyv) and torch.equal(b.pose_count, cf_buf.pose_count) for _, b in cf_lanes)
    del cf_lanes
    cf_got = cf_buf.host()
    cf_ora = oracle.cf_decode(cf_in["pif"], cf_in["paf"], cf_sk.limb_a, cf_sk.limb_b, *cf_prm, pcap=32)
    same = lambda a, b: np.array_equal(np.ascontiguousarray(a).view(np.uint32), np.ascontiguousarray(b).view(np.uint32))
    cf_ok = cf_got["status"] == 0 and all(
        np.array_equal(cf_got["poses"][n][1], cf_ora["poses"][n][1]) and same(cf_got["poses"][n][0], cf_ora["poses"][n][0])
        and same(cf_got["poses"][n][2], cf_ora["poses"][n][2])
        and all(same(cf_got["pif"][n][k][1], cf_ora["pif"][n][k][1]) for k in range(cf_sk.n_parts))
        for n in range(cf_cfg.batch))
    cf_ok = bool(cf_ok) and bool(cf_same_lanes)
    parity = parity and cf_ok
    hp.hp_profile_begin(64)
    for _ in range(5):
        cf_maps, _ = hp.hp_cf_field(cf_pif, cf_cfg.stride, cf_cfg.pif_thr, cap=128)
    torch.cuda.synchronize()
    prf = hp.hp_profile_end()
    cf_field_us = 1e3 * prf["cf_field"][0] / prf["cf_field"][1]
    cf_field_bytes = cf_maps.numel() * 4
    del cf_maps
    composite_fields = {"what": "hp_cf_decode: batch %d, %dx%d grid, stride %d, %d parts, %d limbs, %d planted persons per image"
                                % (cf_cfg.batch, cf_cfg.Fh, cf_cfg.Fw, cf_cfg.stride, cf_sk.n_parts, cf_sk.n_limbs, cf_cfg.n_people),
                        "us_per_call": round(cf_us, 2), "frames_per_s": round(cf_cfg.batch / (cf_us * 1e-6), 1),
                        "frames_per_s_three_streams": round(cf_cfg.batch / (cf_us3 * 1e-6), 1),
                        "kernel_us": {k: round(1e3 * ms / nl, 2) for k, (ms, nl) in sorted(pr.items())},
                        "bound": "latency (persons of an image grow one after the other, a round of growth at a time; the fine "
                                 "confidence maps are never written: their values are summed where they are needed)",
                        "field": {"what": "hp_cf_field: the fine maps of the same batch written out (fp32, %d MB)"
                                          % (cf_field_bytes // 2**20),
                                  "kernel": "k_cf_field", "us": round(cf_field_us, 2), "bound": "hbm",
                                  "achieved": round(cf_field_bytes / (cf_field_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS,
                                  "unit": "GB/s", "frac": round(cf_field_bytes / (cf_field_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
                        "parity_with_oracle": bool(cf_ok)}

    # the streaming front: frames arrive one at a time, the batch slot grows only while batches are running
    streaming = None if args.no_streaming else {
        "what": "hp_batcher_* (dynamic batch slot in front of hp_postprocess, Section 2.2.2): frames of this workload handed "
                "in one at a time by the library's load generator; latency = scheduled arrival -> result seen on the host",
        "dynamic_batching": [streaming_point(N, 2, 4, load, 2000, True) for load in (10_000, 100_000, 200_000, 0)],
        "no_batching": [streaming_point(1, 2, 3, load, 2000, True) for load in (10_000, 0)],
    }

    cpu = None
    if args.cpu_seconds > 0:
        T = min(16, len(os.sched_getaffinity(0)))
        t0 = time.perf_counter()
        oracle.postprocess(batch.cm, batch.paf, sk.limb_a, sk.limb_b, P, threads=T)
        one = time.perf_counter() - t0
        reps = max(1, int(args.cpu_seconds / max(one * T, 1e-3)))      # cpu_seconds of CPU work in total
        t0 = time.perf_counter()
        for _ in range(reps):
            oracle.postprocess(batch.cm, batch.paf, sk.limb_a, sk.limb_b, P, threads=T)
        dt = time.perf_counter() - t0
        t1 = time.perf_counter()
        oracle.postprocess(batch.cm, batch.paf, sk.limb_a, sk.limb_b, P, threads=1)
        dt1 = time.perf_counter() - t1
        cpu = {"value": round(N * reps / dt, 2), "unit": "frames/s", "cores": T, "kind": "oracle",
               "sample": f"the same batch of {N} frames of workload {args.config}, {reps} repetitions, "
                         f"(image, part) and (image, limb) calls farmed over {T} threads",
               "single_thread_value": round(N / dt1, 2)}

    value = N * args.steps / t_multi
    out = {
        "metric": "post-processed frames/s at 656x368 batch 8; achieved HBM GB/s vs peak",
        "value": round(value, 1), "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * t_multi / args.steps, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if esz == 4 else "f16 storage, f32 arithmetic", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}]: {sk.name}, batch {N}, input {cfg.W}x{cfg.H} "
                               f"(CM {K + 1}x{h}x{w}, PAF {2 * L}x{h}x{w}, x8 upsampling), {cfg.n_people} planted "
                               f"people per image", "form": "fused (hi-res maps never written)",
                   "streams_in_flight": n_streams,
                   "capacities": {"peaks": cap, "candidates": ccap, "persons": pcap}},
        "parity_with_oracle": parity,
        "value_one_stream": round(N * args.steps / t_fused, 1),
        "ms_per_step_one_stream": round(1e3 * t_fused / args.steps, 5),
        "value_materialised": round(N * args.steps / t_mat, 1),
        "ms_per_step_materialised": round(1e3 * t_mat / args.steps, 5),
        "kernel_us": {k: round(v, 2) for k, v in sorted(kern_us.items())},
        "kernel_us_note": "each launch carries a pair of HIP events stamped with the kernel's begin and end "
                          "(extended launch call); profiles/ holds the rocprofv3 durations of the same command",
        "staged_kernel_us": {k: round(v, 2) for k, v in sorted(staged_us.items())},
        "roofline": roofline, "roofline_fused": roofline_fused, "roofline_nms_hi": roofline_nms_hi,
        "roofline_scoring": roofline_scoring,
        "preprocess": preprocess,
        "pose_proposal": pose_proposal,
        "composite_fields": composite_fields,
        "smooth": smooth,
        "visualise": visualise,
        "streaming": streaming,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
