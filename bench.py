"""Benchmark: post-processed frames/s of hp_postprocess on synthetic CM/PAF tensors, the HBM roofline of the
staged upsampling kernel, and the CPU oracle timed beside it.

A step is one pass of the whole operator (upsampling, peak NMS, compaction, limb scoring, matching, assembly)
over one batch that is already resident in HBM.

How rates are timed.  Whatever --steps says, a rate comes from WINDOWS windows (default 10) of
max(100, --steps) calls each, every window bracketed by HIP events recorded on the streams the calls
run on (start: one event all streams wait for; end: one event per stream, the latest counts); the line
reports the median window (`value`, `ms_per_step`) and the best one.  --steps / --warmup are echoed.

Which number belongs to which form of the operator:
  value, ms_per_step      hp_postprocess, fused form (the upsampled maps stay in registers), calls issued
                          round-robin on a few HIP streams with their own outputs and workspaces, as the
                          operators of the paper's streaming dataflow overlap (Section 2.2.1);
  *_one_stream            the same calls on one stream (the latency of one batch);
  *_materialised          hp_postprocess with the hi-res maps written out as hp_resize would;
  *_staged                the four staged calls hp_resize (CM, PAF) -> hp_find_peaks -> hp_score_limbs ->
                          hp_assemble, each reading what the previous one wrote to HBM;
  roofline                the staged upsampling kernel k_resize_write (HBM-bound; "form" says so), with the
                          composites of the resize + NMS + scoring kernels of the materialising and the staged
                          route; roofline_fused belongs to the kernel `value` times and counts the work it
                          executes, not the dense definition.
HBM traffic (`traffic`) is measured by this run itself: before the GPU is touched, two short child runs of
this script under `rocprofv3 --pmc` (FETCH_SIZE, then WRITE_SIZE) count the bytes of the staged kernels and of
a plain copy of known size that scales the counters.  When rocprofv3 is missing or a child fails, traffic is null.
"""
import argparse
import csv
import json
import os
import shutil
import statistics
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# plain (non-packed) fp32 lane operations: 256 CUs x 4 SIMDs x 16 lanes/clk x 2.4 GHz
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
COPY_BYTES = 256 << 20          # the calibration copy: this many bytes read and as many written


# ---------------------------------------------------------------------------------------------------------------
# HBM byte counters: child runs under rocprofv3 (started before this process touches the GPU)

def pmc_child(config):
    """The work whose HBM bytes are counted: a few launches of the materialising hp_postprocess, of the staged
    calls, and of the calibration copy.  Runs under `rocprofv3 --pmc <counter>`; prints nothing of interest."""
    import torch
    import paper_2108_11826_amd as hp
    from synth import CONFIGS, BENCH_CAPS, generate, DEFAULT_PARAMS as P
    dev = "cuda:0"
    cfg = CONFIGS[config]
    sk = cfg.skeleton
    N, K, L = cfg.batch, sk.n_parts, sk.n_limbs
    b = generate(cfg)
    cm, paf = torch.from_numpy(b.cm).to(dev), torch.from_numpy(b.paf).to(dev)
    skel = hp.Skeleton(K, sk.limb_a, sk.limb_b)
    prm = hp.Params(P.peak_thr, P.paf_thr, P.n_samples, P.min_valid_ratio, P.min_parts, P.scale)
    buf = hp.Buffers(N, K, L, cfg.h, cfg.w, *BENCH_CAPS[config], dev)
    cm_hi = torch.empty((N, K + 1, cfg.H, cfg.W), dtype=torch.float32, device=dev)
    paf_hi = torch.empty((N, 2 * L, cfg.H, cfg.W), dtype=torch.float32, device=dev)
    src = torch.zeros(COPY_BYTES // 4, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    for _ in range(4):
        hp.hp_postprocess(cm, paf, skel, prm, buf, cm_hi, paf_hi)
        hp.hp_find_peaks(cm_hi, K, P.peak_thr, buf)
        hp.hp_score_limbs(paf_hi, skel, prm, buf)
        hp.hp_assemble(skel, prm, buf)
        hp.hp_postprocess(cm, paf, skel, prm, buf)
        hp.hp_bench_copy(dst, src)
    torch.cuda.synchronize()


def measure_traffic(config):
    """{kernel tag: HBM bytes per launch} from two child runs, or (None, reason)."""
    exe = shutil.which("rocprofv3")
    if exe is None:
        return None, "rocprofv3 not found"
    means = {}
    tmp = tempfile.mkdtemp(prefix="hp_pmc_", dir="/tmp")
    try:
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            out = os.path.join(tmp, counter)
            cmd = ["timeout", "-s", "KILL", "120", exe, "--pmc", counter, "--output-format", "csv", "-d", out, "-o", "c",
                   "--", "python3", os.path.abspath(__file__), "--pmc-child", "--config", str(config)]
            r = subprocess.run(cmd, cwd="/tmp", env={**os.environ, "TMPDIR": "/tmp"}, stdout=subprocess.PIPE,
                               stderr=subprocess.STDOUT, text=True)
            if r.returncode != 0:
                return None, f"rocprofv3 --pmc {counter} ended with {r.returncode}: {r.stdout[-300:]}"
            rows = []
            for dirpath, _, files in os.walk(out):
                for f in files:
                    if f.endswith("counter_collection.csv"):
                        with open(os.path.join(dirpath, f)) as fh:
                            rows += list(csv.DictReader(fh))
            acc = {}
            for row in rows:
                if row.get("Counter_Name") == counter:
                    acc.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
            if not acc:
                return None, f"no {counter} rows"
            means[counter] = {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}
    finally:
        shutil.rmtree(tmp, ignore_errors=True)

    def kib(counter, tag):
        # "k_score" means the scorer of hp_score_limbs, which gathers from the materialised maps: k_score<float, true>
        hit = [v for k, v in means[counter].items() if tag in k and (tag != "k_score" or "true>" in k)]
        return hit[0][0] if hit else None

    copy_f, copy_w = kib("FETCH_SIZE", "k_copy16"), kib("WRITE_SIZE", "k_copy16")
    if not copy_f or not copy_w:
        return None, "calibration copy not found in the counters"
    # the counters are in KiB per dispatch; the copy of COPY_BYTES each way says what one unit is worth
    f_scale, w_scale = COPY_BYTES / copy_f, COPY_BYTES / copy_w
    out = {"scale": {"fetch_bytes_per_unit": round(f_scale, 2), "write_bytes_per_unit": round(w_scale, 2),
                     "note": "plain copy of 256 MiB by hp_bench_copy: counter units per dispatch -> bytes"}}
    for tag in ("k_resize_write", "k_nms_hi_strip", "k_score", "k_resize_nms", "k_limb_small", "k_assemble"):
        f, w = kib("FETCH_SIZE", tag), kib("WRITE_SIZE", tag)
        if f is not None and w is not None:
            out[tag] = {"fetched": int(f * f_scale), "written": int(w * w_scale), "total": int(f * f_scale + w * w_scale)}
    return out, None


# ---------------------------------------------------------------------------------------------------------------

def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--windows", type=int, default=10, help="timed windows per rate (each of max(100, --steps) calls)")
    ap.add_argument("--config", type=int, default=2, help="index into the synthetic workloads (2 = 656x368 batch 8)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU work spent on the oracle baseline (0 = skip)")
    ap.add_argument("--streams", type=int, default=4, help="HIP streams the timed steps are spread over")
    ap.add_argument("--no-streaming", action="store_true", help="skip the streaming-front measurement")
    ap.add_argument("--no-traffic", action="store_true", help="skip the rocprofv3 child runs that count HBM bytes")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other workloads (a kernel profile of one workload wants them out)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the operators around the hot path (pre-processing, smoothing, drawing, the other two "
                         "algorithm classes, the streaming front) and the other workloads")
    ap.add_argument("--streaming-sweep", action="store_true",
                    help="print one JSON line per (batch slot, offered load) point of the streaming front and exit")
    ap.add_argument("--pmc-child", action="store_true", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (images are independent; "
              "a batch would be split across GPUs with no communication). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if args.pmc_child:
        pmc_child(args.config)
        return

    # HBM byte counters first: the children run before this process initialises the GPU
    traffic, traffic_note = (None, "skipped (--no-traffic)")
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ):
        traffic_note = "skipped: this run is itself being profiled"
        traffic_s = 0.0
    elif not args.no_traffic and not args.streaming_sweep:
        t0 = time.perf_counter()
        try:
            traffic, traffic_note = measure_traffic(args.config)
        except Exception as e:          # measurement tooling must never take the benchmark down
            traffic, traffic_note = None, f"{type(e).__name__}: {e}"
        traffic_s = time.perf_counter() - t0
    else:
        traffic_s = 0.0

    import numpy as np
    import torch
    import paper_2108_11826_amd as hp
    import oracle
    from synth import CONFIGS, BENCH_CAPS, generate, DEFAULT_PARAMS as P

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    T = min(16, len(os.sched_getaffinity(0)))
    prm = hp.Params(P.peak_thr, P.paf_thr, P.n_samples, P.min_valid_ratio, P.min_parts, P.scale)
    window_calls = max(100, args.steps)
    n_windows = max(3, args.windows)
    n_streams = max(1, args.streams)
    # Every kernel of this run goes to one of n_streams streams made here, never to the default stream: a process has
    # four hardware queues on this machine and the default stream would hold one of them from its first launch on, so
    # that a fourth lane would share a queue with another lane (400 k frames/s instead of 660 k).  The first of the
    # streams is torch's current stream from here on and carries everything that is not spread over the lanes.
    lane_streams = [torch.cuda.Stream() for _ in range(n_streams)]
    torch.cuda.set_stream(lane_streams[0])

    def timed_windows(calls, streams, calls_per_window=window_calls, windows=n_windows, warm=None):
        """Median / min / max milliseconds per call over `windows` windows of `calls_per_window` calls, the calls
        taken round-robin from `calls` (calls[i] enqueues on streams[i]); HIP events on those streams."""
        warm = max(args.warmup, 2 * len(calls)) if warm is None else warm
        for i in range(warm):
            calls[i % len(calls)]()
        # the window opens on the first of the streams and the others wait for that event: the default stream stays
        # out of it (a process has four hardware queues here; a fifth stream would share one with a lane)
        first = streams[0]
        per_call = []
        for _ in range(windows):
            torch.cuda.synchronize()
            start = torch.cuda.Event(enable_timing=True)
            start.record(first)
            for st in streams[1:]:
                st.wait_event(start)
            for i in range(calls_per_window):
                calls[i % len(calls)]()
            ends = []
            for st in streams:
                e = torch.cuda.Event(enable_timing=True)
                e.record(st)
                ends.append(e)
            torch.cuda.synchronize()
            per_call.append(max(start.elapsed_time(e) for e in ends) / calls_per_window)
        return {"median_ms": statistics.median(per_call), "min_ms": min(per_call), "max_ms": max(per_call),
                "windows": windows, "calls_per_window": calls_per_window}

    def poses_match(buf, ora, N, K, peaks_too=True):
        poses, _ = buf.host_poses()
        ok = buf.host_status() == 0
        for n in range(N):
            ok = ok and np.array_equal(poses[n][0], ora["poses"][n][0]) and np.array_equal(poses[n][2], ora["poses"][n][2])
        if peaks_too:
            peaks, _ = buf.host_peaks()
            for n in range(N):
                for c in range(K):
                    ok = ok and all(np.array_equal(peaks[n][c][q], ora["peaks"][n][c][q]) for q in range(3))
        return bool(ok)

    def lanes_for(N, K, L, h, w, caps, cm, paf, skel):
        lanes = [(st, hp.Buffers(N, K, L, h, w, *caps, dev)) for st in lane_streams]
        torch.cuda.synchronize()
        return lanes, [hp.PostprocessCall(cm, paf, skel, prm, bf, stream=st) for st, bf in lanes]

    # ---- the workload of the metric --------------------------------------------------------------------------
    cfg = CONFIGS[args.config]
    sk = cfg.skeleton
    N, K, L, h, w = cfg.batch, sk.n_parts, sk.n_limbs, cfg.h, cfg.w
    batch = generate(cfg)
    cm, paf = torch.from_numpy(batch.cm).to(dev), torch.from_numpy(batch.paf).to(dev)
    skel = hp.Skeleton(K, sk.limb_a, sk.limb_b)
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

    main_stream = lane_streams[0]
    call_fused = hp.PostprocessCall(cm, paf, skel, prm, buf)
    call_mat = hp.PostprocessCall(cm, paf, skel, prm, buf, cm_hi, paf_hi)

    def staged_route():
        hp.hp_resize(cm, cm_hi)
        hp.hp_resize(paf, paf_hi)
        hp.hp_find_peaks(cm_hi, K, P.peak_thr, buf)
        hp.hp_score_limbs(paf_hi, skel, prm, buf)
        hp.hp_assemble(skel, prm, buf)

    # correctness gate (outside the timed regions): every timed form against the oracle
    ora = oracle.postprocess(batch.cm, batch.paf, sk.limb_a, sk.limb_b, P, threads=T)
    parity = True
    for form in (call_fused, call_mat, staged_route):
        buf.pose_count.fill_(-1)
        form()
        torch.cuda.synchronize()
        parity = parity and poses_match(buf, ora, N, K)

    lanes, calls = lanes_for(N, K, L, h, w, (cap, ccap, pcap), cm, paf, skel)
    t_multi = timed_windows(calls, [st for st, _ in lanes])
    for _, bf in lanes:                        # every lane must hold the oracle's persons too
        parity = parity and poses_match(bf, ora, N, K, peaks_too=False)
    t_one = timed_windows([call_fused], [main_stream])
    t_mat = timed_windows([call_mat], [main_stream])
    t_staged = timed_windows([staged_route], [main_stream], windows=max(3, n_windows // 2))

    # per-kernel times: the same calls with every launch stamped by a pair of events
    prof_steps = min(window_calls, 200)
    hp.hp_profile_begin(prof_steps * 16)
    for _ in range(prof_steps):
        call_fused()
    for _ in range(prof_steps):
        call_mat()
    torch.cuda.synchronize()
    kern_us = {k: 1e3 * ms / n for k, (ms, n) in hp.hp_profile_end().items()}
    staged_steps = min(window_calls, 100)
    hp.hp_profile_begin(staged_steps * 16)
    for _ in range(staged_steps):
        staged_route()
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
    k1_bytes = lo_bytes + hi_bytes                        # lo CM+PAF read once, hi CM+PAF written once
    score_bytes = 80.0 * n_pairs                          # 10 samples x 2 channels x 4 B per pair
    gbs = lambda nbytes, us: nbytes / (us * 1e-6) / 1e9
    tr = lambda tag: (traffic or {}).get(tag, {}).get("total")

    k1_us = kern_us["resize_write"]                       # one launch writes CM and PAF (materialising form)
    staged_w_us = staged_us["resize_write"]               # mean of the two hp_resize launches of the staged route
    k1_staged_us = 2 * staged_w_us + staged_us["nms_hi"]
    roofline = {
        "kernel": "k_resize_write (x8 bilinear upsampling of all CM and PAF channels into materialised hi-res maps)",
        "form": "staged / materialising: this kernel is not part of the fused step that `value` times "
                "(see roofline_fused for that one)",
        "bound": "hbm", "achieved": round(gbs(k1_bytes, k1_us), 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(gbs(k1_bytes, k1_us) / HBM_PEAK_GBS, 4), "traffic": tr("k_resize_write"),
        "traffic_note": "HBM bytes per launch from this run's own rocprofv3 --pmc children (FETCH_SIZE + WRITE_SIZE, "
                        "scaled by a plain copy of 256 MiB)" if tr("k_resize_write") else traffic_note,
        "bytes_per_launch": k1_bytes, "us_per_launch": round(k1_us, 2),
        "plain_fill_same_bytes": {"us": round(fill_us, 2), "GB/s": round(fill_gbs, 1),
                                  "frac_of_fill": round(gbs(k1_bytes, k1_us) / fill_gbs, 4)},
        "composites": {
            "note": "algorithmic bytes of resize + NMS = lo-res read once + hi-res written once (a fused kernel need "
                    "not re-read the maps); scoring adds 80 useful bytes per candidate pair; durations are sums of "
                    "kernel durations",
            "resize_nms_materialising": {
                "kernels": "k_resize_write + k_resize_nms", "us": round(k1_us + kern_us["resize_nms"], 2),
                "frac": round(gbs(k1_bytes, k1_us + kern_us["resize_nms"]) / HBM_PEAK_GBS, 4)},
            "resize_nms_scoring_materialising": {
                "kernels": "k_resize_write + k_resize_nms + " + ("k_limb_small" if "limb_small" in kern_us else "k_sort_peaks + k_score + k_match"),
                "us": round(k1_us + kern_us["resize_nms"] + kern_us.get("limb_small", kern_us.get("score_lo", 0.0)), 2),
                "frac": round(gbs(k1_bytes + score_bytes, k1_us + kern_us["resize_nms"] +
                                  kern_us.get("limb_small", kern_us.get("score_lo", 0.0))) / HBM_PEAK_GBS, 4)},
            "resize_nms_staged": {
                "kernels": "k_resize_write (CM) + k_resize_write (PAF) + k_nms_hi_strip", "us": round(k1_staged_us, 2),
                "frac": round(gbs(k1_bytes, k1_staged_us) / HBM_PEAK_GBS, 4)},
            "resize_nms_scoring_staged": {
                "kernels": "the same + k_score (gathering from the materialised PAFs)",
                "us": round(k1_staged_us + staged_us["score_hi"], 2),
                "frac": round(gbs(k1_bytes + score_bytes, k1_staged_us + staged_us["score_hi"]) / HBM_PEAK_GBS, 4)}}}

    # staged peak search: reads K of the K+1 hi-res confidence maps once, writes peaks only
    nms_bytes = N * K * cfg.H * cfg.W * 4
    roofline_nms_hi = {"kernel": "k_nms_hi_strip (hp_find_peaks: 3x3 thresholded NMS on the materialised hi-res CMs)",
                       "form": "staged", "bound": "hbm", "achieved": round(gbs(nms_bytes, staged_us["nms_hi"]), 1),
                       "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(gbs(nms_bytes, staged_us["nms_hi"]) / HBM_PEAK_GBS, 4),
                       "traffic": tr("k_nms_hi_strip"), "bytes_per_launch": nms_bytes,
                       "us_per_launch": round(staged_us["nms_hi"], 2)}

    # fused form: nothing but the lo-res CM is read.  Work executed: phase 1 looks at every lo-res node of the K
    # searched channels (9 loads, 9 max, 1 multiply, 1 compare: 11 lane-ops), phase 2 upsamples and tests the two
    # 8x4 tiles of the nodes whose 3x3 neighbourhood can reach the threshold: per tile 42 (horizontal pass) + 130
    # (vertical pass) + 80 (row maxima) + 32 x 7 (tests) = 476 lane-ops of the definition.  The surviving nodes are
    # counted here from the input with the kernel's rule.
    cmk = torch.from_numpy(np.ascontiguousarray(batch.cm[:, :K])).to(dev).float()
    mx9 = torch.nn.functional.max_pool2d(torch.nn.functional.pad(cmk, (1, 1, 1, 1), mode="replicate"), 3, 1)
    alive = int((~(mx9 * np.float32(1.000001) < np.float32(P.peak_thr))).sum()) if P.peak_thr > 0 else int(cmk.numel())
    nodes = int(cmk.numel())
    fused_ops = 11 * nodes + 476 * 2 * alive
    dense_ops = 12 * N * K * cfg.H * cfg.W
    fused_us = kern_us["resize_nms"]
    roofline_fused = {"kernel": "k_resize_nms (peak search on upsampled values kept in registers; first kernel of the timed step)",
                      "form": "fused", "bound": "alu", "achieved": round(fused_ops / (fused_us * 1e-6) / 1e12, 2),
                      "peak": round(ALU_PEAK_TLANEOPS, 1), "unit": "Tlane-op/s",
                      "frac": round(fused_ops / (fused_us * 1e-6) / 1e12 / ALU_PEAK_TLANEOPS, 4),
                      "ops_per_launch": fused_ops, "us_per_launch": round(fused_us, 2),
                      "nodes": nodes, "nodes_whose_tiles_are_searched": alive,
                      "note": "executed work: 11 lane-ops per lo-res node + 476 per searched 8x4 tile; the kernel is "
                              "latency-bound (two dependent rounds of loads and a workgroup-wide compaction), not ALU-bound; "
                              "the dense definition would be %d lane-ops" % dense_ops,
                      "hbm_bytes_per_launch": batch.cm[:, :K].size * esz, "traffic": tr("k_resize_nms")}
    del cmk, mx9
    lo_name = "limb_small" if "limb_small" in kern_us else "score_lo"
    roofline_scoring = {"kernel": "k_score<float, true> (hp_score_limbs: limb scoring with PAFs gathered from the "
                                  "materialised maps; 80 useful bytes per pair, 4-byte gathers)",
                        "form": "staged", "bound": "hbm",
                        "achieved": round(gbs(score_bytes, staged_us["score_hi"]), 2),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(gbs(score_bytes, staged_us["score_hi"]) / HBM_PEAK_GBS, 6),
                        "traffic": tr("k_score"), "bytes_per_launch": score_bytes, "pairs_per_launch": n_pairs,
                        "us_per_launch": round(staged_us["score_hi"], 2),
                        "note": "gather-bound, not stream-bound: every 4-byte sample pulls a whole sector",
                        "us_per_launch_lo_res_form": round(kern_us[lo_name], 2),
                        "lo_res_form_kernel": lo_name}

    # ---- the other four workloads: fused form, same streams and window scheme (shorter), parity with the oracle ----
    other_configs = None
    if not args.no_extras and not args.no_other_configs:
        other_configs = {}
        for ci in range(len(CONFIGS)):
            if ci == args.config:
                continue
            c2 = CONFIGS[ci]
            s2 = c2.skeleton
            b2 = generate(c2)
            cm2, paf2 = torch.from_numpy(b2.cm).to(dev), torch.from_numpy(b2.paf).to(dev)
            skel2 = hp.Skeleton(s2.n_parts, s2.limb_a, s2.limb_b)
            o2 = oracle.postprocess(b2.cm, b2.paf, s2.limb_a, s2.limb_b, P, threads=T)
            lanes2, calls2 = lanes_for(c2.batch, s2.n_parts, s2.n_limbs, c2.h, c2.w, BENCH_CAPS[ci], cm2, paf2, skel2)
            t2 = timed_windows(calls2, [st for st, _ in lanes2], calls_per_window=60, windows=5, warm=6)
            ok2 = all(poses_match(bf, o2, c2.batch, s2.n_parts) for _, bf in lanes2)
            t2one = timed_windows([calls2[0]], [lanes2[0][0]], calls_per_window=30, windows=3, warm=3)
            parity = parity and ok2
            other_configs[f"configs[{ci}]"] = {
                "workload": f"{s2.name}, batch {c2.batch}, input {c2.W}x{c2.H}, {b2.cm.dtype}",
                "value": round(c2.batch / (t2["median_ms"] * 1e-3), 1), "unit": "frames/s",
                "value_best_window": round(c2.batch / (t2["min_ms"] * 1e-3), 1),
                "ms_per_step": round(t2["median_ms"], 5), "ms_per_step_one_stream": round(t2one["median_ms"], 5),
                "windows": t2["windows"], "calls_per_window": t2["calls_per_window"],
                "capacities": dict(zip(("peaks", "candidates", "persons"), BENCH_CAPS[ci])),
                "parity_with_oracle": ok2}
            del lanes2, calls2, cm2, paf2

    extras = {}
    if not args.no_extras:
        extras, ok = widened_operators(hp, oracle, np, torch, dev, cfg, batch, cm, paf, cm_hi, skel, prm, P, N, K, L, h, w,
                                       (cap, ccap, pcap), lane_streams)
        parity = parity and ok
        if not args.no_streaming:
            extras["streaming"] = {
                "what": "hp_batcher_* (dynamic batch slot in front of hp_postprocess, Section 2.2.2): frames of this workload "
                        "handed in one at a time by the library's load generator; latency = scheduled arrival -> result seen "
                        "on the host",
                "dynamic_batching": [streaming_point(N, 2, 4, load, 2000, True) for load in (10_000, 100_000, 200_000, 0)],
                "no_batching": [streaming_point(1, 2, 3, load, 2000, True) for load in (10_000, 0)]}

    cpu = None
    if args.cpu_seconds > 0:
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

    fps = lambda t, key="median_ms": round(N / (t[key] * 1e-3), 1)
    out = {
        "metric": "post-processed frames/s at 656x368 batch 8; achieved HBM GB/s vs peak",
        "value": fps(t_multi), "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t_multi["median_ms"], 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if esz == 4 else "f16 storage, f32 arithmetic", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}]: {sk.name}, batch {N}, input {cfg.W}x{cfg.H} "
                               f"(CM {K + 1}x{h}x{w}, PAF {2 * L}x{h}x{w}, x8 upsampling), {cfg.n_people} planted "
                               f"people per image", "form": "fused (hi-res maps never written)",
                   "streams_in_flight": n_streams,
                   "capacities": {"peaks": cap, "candidates": ccap, "persons": pcap}},
        "timing": {"method": "HIP events on the streams of the calls; median over windows",
                   "windows": t_multi["windows"], "calls_per_window": t_multi["calls_per_window"],
                   "ms_per_step_median": round(t_multi["median_ms"], 5), "ms_per_step_min": round(t_multi["min_ms"], 5),
                   "ms_per_step_max": round(t_multi["max_ms"], 5), "value_best_window": fps(t_multi, "min_ms"),
                   "note": "--steps and --warmup are echoed; every rate of this line is timed over its own windows of "
                           "max(100, --steps) calls, whatever --steps is"},
        "parity_with_oracle": parity,
        "value_one_stream": fps(t_one), "ms_per_step_one_stream": round(t_one["median_ms"], 5),
        "ms_per_step_one_stream_min": round(t_one["min_ms"], 5),
        "value_materialised": fps(t_mat), "ms_per_step_materialised": round(t_mat["median_ms"], 5),
        "value_staged": fps(t_staged), "ms_per_step_staged": round(t_staged["median_ms"], 5),
        "ms_per_step_staged_min": round(t_staged["min_ms"], 5),
        "staged_route": "hp_resize (CM) -> hp_resize (PAF) -> hp_find_peaks -> hp_score_limbs -> hp_assemble, one stream",
        "kernel_us": {k: round(v, 2) for k, v in sorted(kern_us.items())},
        "kernel_us_note": "each launch carries a pair of HIP events stamped with the kernel's begin and end "
                          "(extended launch call); profiles/ holds the rocprofv3 durations of the same command",
        "staged_kernel_us": {k: round(v, 2) for k, v in sorted(staged_us.items())},
        "roofline": roofline, "roofline_fused": roofline_fused, "roofline_nms_hi": roofline_nms_hi,
        "roofline_scoring": roofline_scoring,
        "hbm_traffic": traffic if traffic else {"note": traffic_note},
        "hbm_traffic_seconds": round(traffic_s, 1),
        "other_configs": other_configs,
        **extras,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def widened_operators(hp, oracle, np, torch, dev, cfg, batch, cm, paf, cm_hi, skel, prm, P, N, K, L, h, w, caps, lane_streams):
    """The operators around the hot path, each timed per kernel and checked against its oracle: pre-processing,
    smoothing, drawing, the pose-proposal and the composite-field family.  Returns ({name: object}, all parity ok)."""
    cap, ccap, pcap = caps
    sk = cfg.skeleton
    parity = True

    def kernel_us(call, reps, max_launches=256):
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        hp.hp_profile_begin(max_launches)
        for _ in range(reps):
            call()
        torch.cuda.synchronize()
        return {k: 1e3 * ms / n for k, (ms, n) in hp.hp_profile_end().items()}

    # the operator before the network (decoded frames -> resized channel-first tensor), at the frame size of
    # the paper's benchmark video and the input size of this workload's network, on a batch large enough to
    # be bandwidth-bound
    pre_frames = 64
    pre_src = torch.randint(0, 256, (pre_frames, 360, 640, 3), dtype=torch.uint8, device=dev)
    pre_dst = torch.empty((pre_frames, 3, cfg.H, cfg.W), dtype=torch.float32, device=dev)
    pre_us = kernel_us(lambda: hp.hp_preprocess(pre_src, cfg.H, cfg.W, 1 / 255.0, 0.0, True, out=pre_dst), 20)["preprocess"]
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
    sm_us = kernel_us(lambda: hp.hp_smooth(cm_hi, taps_dev, channels=K, out=sm_dst), 20)["smooth"]
    sm_px = N * K * cfg.H * cfg.W
    sm_ok = bool(np.array_equal(sm_dst[N - 1, K - 1].cpu().numpy(),
                                oracle.smooth(oracle.resize(batch.cm[N - 1, K - 1], 8), taps_np)))
    parity = parity and sm_ok
    sm_fma = sm_px * len(taps_np) * 2
    smooth = {"kernel": "k_smooth_march (hp_smooth: separable %d-tap smoothing of the %d part maps per image, %dx%d)" % (len(taps_np), K, cfg.W, cfg.H),
              "us_per_launch": round(sm_us, 2),
              "roofline": {"bound": "hbm", "achieved": round(8 * sm_px / (sm_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": round(8 * sm_px / (sm_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "bytes_per_launch": 8 * sm_px},
              "alu": {"achieved": round(sm_fma / (sm_us * 1e-6) / 1e12, 2), "peak": round(ALU_PEAK_TLANEOPS, 1), "unit": "Tfma/s",
                      "frac": round(sm_fma / (sm_us * 1e-6) / 1e12 / ALU_PEAK_TLANEOPS, 4),
                      "note": "fused multiply-adds of the definition: 2 x taps per pixel"},
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
    pr = kernel_us(lambda: hp.hp_draw_poses(vis_src, cfg.H, cfg.W, skel, vbuf, limb_rgb, part_rgb, 4, 4, out=vis_dst), 20)
    list_us, tiles_us = pr["draw_list"], pr["draw"]
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

    def wall_us(call, reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            call()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e6

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
    pr = kernel_us(pp_call, 20)
    pp_us = wall_us(pp_call, 200)
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
                     "kernel_us": {k: round(v, 2) for k, v in sorted(pr.items())},
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
    pr = kernel_us(cf_call, 20)
    cf_us = wall_us(cf_call, 100)
    # the same call with three batches in flight on separate streams (own outputs and workspace each), as for the headline
    cf_lanes = [(st, hp.CFBuffers(cf_cfg.batch, cf_sk.n_parts, cf_sk.n_limbs, 128, 256, 32, dev)) for st in lane_streams[:3]]
    torch.cuda.synchronize()

    def cf_round(reps):
        for i in range(reps):
            st, b = cf_lanes[i % len(cf_lanes)]
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
    cf_maps = [None]

    def cf_field_call():
        cf_maps[0], _ = hp.hp_cf_field(cf_pif, cf_cfg.stride, cf_cfg.pif_thr, cap=128)

    cf_field_us = kernel_us(cf_field_call, 5, 64)["cf_field"]
    cf_field_bytes = cf_maps[0].numel() * 4
    cf_maps[0] = None
    composite_fields = {"what": "hp_cf_decode: batch %d, %dx%d grid, stride %d, %d parts, %d limbs, %d planted persons per image"
                                % (cf_cfg.batch, cf_cfg.Fh, cf_cfg.Fw, cf_cfg.stride, cf_sk.n_parts, cf_sk.n_limbs, cf_cfg.n_people),
                        "us_per_call": round(cf_us, 2), "frames_per_s": round(cf_cfg.batch / (cf_us * 1e-6), 1),
                        "frames_per_s_three_streams": round(cf_cfg.batch / (cf_us3 * 1e-6), 1),
                        "kernel_us": {k: round(v, 2) for k, v in sorted(pr.items())},
                        "bound": "latency (persons of an image grow one after the other, a round of growth at a time; the fine "
                                 "confidence maps are never written: their values are summed where they are needed)",
                        "field": {"what": "hp_cf_field: the fine maps of the same batch written out (fp32, %d MB)"
                                          % (cf_field_bytes // 2**20),
                                  "kernel": "k_cf_field", "us": round(cf_field_us, 2), "bound": "hbm",
                                  "achieved": round(cf_field_bytes / (cf_field_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS,
                                  "unit": "GB/s", "frac": round(cf_field_bytes / (cf_field_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
                        "parity_with_oracle": bool(cf_ok)}
    return {"preprocess": preprocess, "pose_proposal": pose_proposal, "composite_fields": composite_fields,
            "smooth": smooth, "visualise": visualise}, parity


if __name__ == "__main__":
    main()
