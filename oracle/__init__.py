"""CPU oracle for bottom-up pose post-processing: TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over `hp_oracle.c` (the plain C statement of the
post-processing operator of the paper's Section 2.2.1) plus the loops that
chain its steps over images, parts and limbs.  Only tests, the smoke check and
the benchmark's `cpu_baseline` leg may import this package; it shares no code
with the HIP library.

Parity pins: see the header of `hp_oracle.c` (assembly is pinned by planted
skeleton recovery and invariants only; parity with the paper's own engine is
unpinned).
"""
import ctypes
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hp_oracle.c")
_SRC_PRE = os.path.join(_HERE, "hp_pre_oracle.c")
_SRC_DRAW = os.path.join(_HERE, "hp_draw_oracle.c")
_SRC_SMOOTH = os.path.join(_HERE, "hp_smooth_oracle.c")
_SRC_REFINE = os.path.join(_HERE, "hp_refine_oracle.c")
_SRC_PP = os.path.join(_HERE, "hp_pp_oracle.c")
_SRC_CF = os.path.join(_HERE, "hp_cf_oracle.c")


def _cpu_has_fma():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("flags"):
                    return " fma " in line + " "
    except OSError:
        pass
    return False


def build(force=False):
    """Compile the oracle twice: with hardware FMA and without (libm fmaf)."""
    out = []
    for tag, extra in (("fma", ["-mfma"]), ("generic", [])):
        so = os.path.join(_HERE, f"libhp_oracle_{tag}.so")
        newest = max(os.path.getmtime(f) for f in (_SRC, _SRC_PRE, _SRC_DRAW, _SRC_SMOOTH, _SRC_REFINE, _SRC_PP, _SRC_CF))
        if force or not os.path.exists(so) or os.path.getmtime(so) < newest:
            cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
                   "-shared", "-Wall", "-Wextra", *extra, _SRC, _SRC_PRE, _SRC_DRAW, _SRC_SMOOTH, _SRC_REFINE, _SRC_PP, _SRC_CF, "-o", so, "-lm"]
            subprocess.check_call(cmd)
        out.append(so)
    build_cf_libm(force)
    return out


def build_cf_libm(force=False):
    """The composite-field oracle alone, compiled with the C library's exponential in place of rule C0's fixed
    arithmetic (-DHPC_LIBM_EXP): a checker of the oracle, used by tests/test_oracle_cf.py only."""
    so = os.path.join(_HERE, "libhp_oracle_cf_libmexp.so")
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(_SRC_CF):
        subprocess.check_call(["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall",
                               "-Wextra", "-DHPC_LIBM_EXP", _SRC_CF, "-o", so, "-lm"])
    return so


_lib = None
_lib_cf_libm = None
_lock = threading.Lock()


def _declare_cf(L):
    i32p, f32p, ci, cf = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float), ctypes.c_int, ctypes.c_float
    L.hpc_expneg.restype = cf
    L.hpc_expneg.argtypes = [cf]
    L.hpc_field.restype = None
    L.hpc_field.argtypes = [f32p, ci, ci, ci, cf, f32p]
    L.hpc_decode.restype = ci
    L.hpc_decode.argtypes = [f32p, f32p, ci, ci, i32p, i32p, ci, ci, ci, cf, cf, cf, cf, cf, ci, ci,
                             i32p, f32p, i32p, i32p, f32p, f32p, i32p, f32p, i32p, f32p, i32p]


def lib_cf_libm():
    global _lib_cf_libm
    with _lock:
        if _lib_cf_libm is None:
            L = ctypes.CDLL(build_cf_libm())
            _declare_cf(L)
            _lib_cf_libm = L
    return _lib_cf_libm


def lib():
    global _lib
    if _lib is not None:
        return _lib
    with _lock:
        if _lib is not None:
            return _lib
        fma_so, gen_so = build()
        L = ctypes.CDLL(fma_so if _cpu_has_fma() else gen_so)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        ci = ctypes.c_int
        cf = ctypes.c_float
        L.hpo_up.restype = cf
        L.hpo_up.argtypes = [f32p, ci, ci, ci, ci, ci]
        L.hpo_resize.restype = None
        L.hpo_resize.argtypes = [f32p, ci, ci, ci, ci, f32p]
        L.hpo_find_peaks.restype = ci
        L.hpo_find_peaks.argtypes = [f32p, ci, ci, cf, ci, i32p, i32p, f32p]
        L.hpo_need.restype = ci
        L.hpo_need.argtypes = [cf, ci]
        L.hpo_score_limb.restype = ci
        L.hpo_score_limb.argtypes = [f32p, f32p, ci, ci, ci, ci, i32p, i32p, ci, i32p, i32p,
                                     ci, cf, ci, ci, i32p, i32p, f32p]
        L.hpo_match_limb.restype = ci
        L.hpo_match_limb.argtypes = [ci, i32p, i32p, f32p, ci, ci, i32p, i32p, f32p]
        L.hpo_assemble.restype = ci
        L.hpo_assemble.argtypes = [ci, ci, i32p, i32p, f32p, ci, i32p, i32p, i32p, f32p,
                                   ci, ci, ci, i32p, i32p, f32p]
        u8p = ctypes.POINTER(ctypes.c_uint8)
        L.hpq_preprocess.restype = None
        L.hpq_preprocess.argtypes = [u8p, ci, ci, ci, ci, ci, ci, ci, f32p, f32p, f32p]
        L.hpp_iou.restype = cf
        L.hpp_iou.argtypes = [f32p, f32p]
        L.hpp_detect.restype = ci
        L.hpp_detect.argtypes = [f32p, f32p, f32p, ci, ci, cf, cf, cf, cf, ci, i32p, f32p, f32p]
        L.hpp_parse.restype = ci
        L.hpp_parse.argtypes = [ci, ci, i32p, i32p, i32p, f32p, i32p, ci, f32p, ci, ci, ci, ci, cf, ci, ci, i32p, i32p, f32p]
        L.hpf_refine.restype = None
        L.hpf_refine.argtypes = [f32p, ci, ci, ci, i32p, i32p, f32p, f32p]
        L.hps_smooth.restype = ci
        L.hps_smooth.argtypes = [f32p, f32p, ci, ci, ci, f32p, ci]
        L.hpv_in_capsule.restype = ci
        L.hpv_in_capsule.argtypes = [ci] * 7
        L.hpv_in_disc.restype = ci
        L.hpv_in_disc.argtypes = [ci] * 5
        L.hpv_draw.restype = None
        L.hpv_draw.argtypes = [u8p, u8p, ci, ci, ci, ci, ci, ci, ci, i32p, i32p, i32p, i32p, ci, i32p, ci, u8p, u8p, ci, ci]
        _declare_cf(L)
        _lib = L
    return _lib


def _f32(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i32(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _as_f32(a):
    """Exact widening of fp16/fp32 storage to contiguous fp32."""
    return np.ascontiguousarray(np.asarray(a).astype(np.float32))


def up(lo_plane, s, Y, X):
    lo_plane = _as_f32(lo_plane)
    h, w = lo_plane.shape
    return float(lib().hpo_up(_f32(lo_plane), h, w, s, int(Y), int(X)))


def resize(lo, s=8):
    """[..., h, w] -> fp32 [..., s*h, s*w]."""
    lo = _as_f32(lo)
    h, w = lo.shape[-2:]
    planes = int(np.prod(lo.shape[:-2], dtype=np.int64))
    hi = np.empty(lo.shape[:-2] + (s * h, s * w), dtype=np.float32)
    lib().hpo_resize(_f32(lo), planes, h, w, s, _f32(hi))
    return hi


def preprocess(images, Hd, Wd, alpha, beta, reverse_channels=False):
    """uint8 [N, Hs, Ws, C] -> fp32 [N, C, Hd, Wd] (pre-processing operator, hp_pre_oracle.c)."""
    im = np.ascontiguousarray(images, dtype=np.uint8)
    N, Hs, Ws, C = im.shape
    al = np.ascontiguousarray(np.broadcast_to(np.asarray(alpha, np.float32), (C,)))
    be = np.ascontiguousarray(np.broadcast_to(np.asarray(beta, np.float32), (C,)))
    out = np.empty((N, C, Hd, Wd), np.float32)
    lib().hpq_preprocess(im.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), N, Hs, Ws, C, int(Hd), int(Wd),
                         1 if reverse_channels else 0, _f32(al), _f32(be), _f32(out))
    return out


def pp_iou(a, b):
    a, b = np.ascontiguousarray(a, np.float32), np.ascontiguousarray(b, np.float32)
    return float(lib().hpp_iou(_f32(a), _f32(b)))


def pp_detect(resp, conf, box, img_w, img_h, det_thr, nms_thr):
    """Pose-proposal detections of one (image, part): resp, conf [Gh, Gw], box [4, Gh, Gw] ->
    (cell int32[], score fp32[], corners fp32[n, 4]) in the order kept (hp_pp_oracle.c, D1-D3)."""
    r, c, b = (np.ascontiguousarray(v, np.float32) for v in (resp, conf, box))
    Gh, Gw = r.shape
    cap = Gh * Gw
    cell, score, corners = np.zeros(cap, np.int32), np.zeros(cap, np.float32), np.zeros((cap, 4), np.float32)
    n = lib().hpp_detect(_f32(r), _f32(c), _f32(b), Gh, Gw, float(img_w), float(img_h), float(det_thr), float(nms_thr), cap,
                         _i32(cell), _f32(score), _f32(corners))
    return cell[:n].copy(), score[:n].copy(), corners[:n].copy()


def pp_decode(resp, conf, box, edge, limb_a, limb_b, img_w, img_h, det_thr, nms_thr, edge_thr, min_parts):
    """Whole pose-proposal post-processing of a batch (D1-D5): resp, conf [N, K, Gh, Gw]; box [N, K, 4, Gh, Gw];
    edge [N, L, Nh, Nw, Gh, Gw].  Returns {"dets": [n][k] -> (cell, score, corners), "poses": [n] -> (slots, nparts, score)}."""
    resp, conf, box, edge = (np.ascontiguousarray(v, np.float32) for v in (resp, conf, box, edge))
    N, K, Gh, Gw = resp.shape
    L, Nh, Nw = edge.shape[1:4]
    la, lb = np.ascontiguousarray(limb_a, np.int32), np.ascontiguousarray(limb_b, np.int32)
    cap = Gh * Gw
    dets, poses = [], []
    for n in range(N):
        per_part = [pp_detect(resp[n, k], conf[n, k], box[n, k], img_w, img_h, det_thr, nms_thr) for k in range(K)]
        dets.append(per_part)
        cell, score = np.zeros((K, cap), np.int32), np.zeros((K, cap), np.float32)
        count = np.zeros(K, np.int32)
        for k in range(K):
            m = len(per_part[k][0])
            cell[k, :m], score[k, :m], count[k] = per_part[k][0], per_part[k][1], m
        pcap = max(1, int(count[la[0]]))
        slots, nparts, pscore = np.zeros((pcap, K), np.int32), np.zeros(pcap, np.int32), np.zeros(pcap, np.float32)
        e = np.ascontiguousarray(edge[n])
        m = lib().hpp_parse(K, L, _i32(la), _i32(lb), _i32(cell), _f32(score), _i32(count), cap, _f32(e), Gh, Gw, Nh, Nw,
                            float(edge_thr), int(min_parts), pcap, _i32(slots), _i32(nparts), _f32(pscore))
        poses.append((slots[:m].copy(), nparts[:m].copy(), pscore[:m].copy()))
    return {"dets": dets, "poses": poses}


def cf_expneg(t):
    """E(t) of the composite-field decoder (hp_cf_oracle.c, C0), elementwise on an fp32 array."""
    t = np.ascontiguousarray(t, np.float32)
    f = lib().hpc_expneg
    return np.array([f(float(v)) for v in t.ravel()], np.float32).reshape(t.shape)


def cf_field(pif_k, stride, pif_thr):
    """Fine confidence map [Fh * stride, Fw * stride] of one part's intensity field [5, Fh, Fw] (C1-C2)."""
    p = np.ascontiguousarray(pif_k, np.float32)
    _, Fh, Fw = p.shape
    out = np.empty((Fh * stride, Fw * stride), np.float32)
    lib().hpc_field(_f32(p), Fh, Fw, int(stride), float(pif_thr), _f32(out))
    return out


def cf_decode(pif, paf, limb_a, limb_b, stride, pif_thr, paf_thr, seed_thr, grow_thr, rev_tol, min_parts, pcap=64,
              libm_exp=False):
    """Composite-field decoding of a batch (C1-C8): pif [N, K, 5, Fh, Fw], paf [N, L, 7, Fh, Fw].
    Returns {"pif": [n][k] -> (cell, value), "paf": [n][l] -> (cell, F1, F2), "poses": [n] -> (xyv [m, K, 3], nparts,
    score), "overflow": [n]}."""
    pif, paf = np.ascontiguousarray(pif, np.float32), np.ascontiguousarray(paf, np.float32)
    N, K, _, Fh, Fw = pif.shape
    L = paf.shape[1]
    la, lb = np.ascontiguousarray(limb_a, np.int32), np.ascontiguousarray(limb_b, np.int32)
    cells = Fh * Fw
    out = {"pif": [], "paf": [], "poses": [], "overflow": []}
    dec = (lib_cf_libm() if libm_exp else lib()).hpc_decode      # libm_exp: the test-only build, see build_cf_libm

    def one(n):
        pc, pv, pn = np.zeros((K, cells), np.int32), np.zeros((K, cells), np.float32), np.zeros(K, np.int32)
        ac, f1, f2, an = (np.zeros((L, cells), np.int32), np.zeros((L, cells), np.float32),
                          np.zeros((L, cells), np.float32), np.zeros(L, np.int32))
        xyv, npt, sc = np.zeros((pcap, K, 3), np.float32), np.zeros(pcap, np.int32), np.zeros(pcap, np.float32)
        ovf = np.zeros(1, np.int32)
        a, b = np.ascontiguousarray(pif[n]), np.ascontiguousarray(paf[n])
        m = dec(_f32(a), _f32(b), K, L, _i32(la), _i32(lb), Fh, Fw, int(stride), float(pif_thr),
                             float(paf_thr), float(seed_thr), float(grow_thr), float(rev_tol), int(min_parts), int(pcap),
                             _i32(pc), _f32(pv), _i32(pn), _i32(ac), _f32(f1), _f32(f2), _i32(an), _f32(xyv), _i32(npt),
                             _f32(sc), _i32(ovf))
        return ([(pc[k, :pn[k]].copy(), pv[k, :pn[k]].copy()) for k in range(K)],
                [(ac[l, :an[l]].copy(), f1[l, :an[l]].copy(), f2[l, :an[l]].copy()) for l in range(L)],
                (xyv[:m].copy(), npt[:m].copy(), sc[:m].copy()), int(ovf[0]))

    for n in range(N):
        p, a, ps, o = one(n)
        out["pif"].append(p)
        out["paf"].append(a)
        out["poses"].append(ps)
        out["overflow"].append(o)
    return out


def refine_peaks(plane_hi, px, py):
    """Sub-pixel positions (xf, yf) of the peaks (px, py) of one fp32 plane (hp_refine_oracle.c)."""
    u = np.ascontiguousarray(plane_hi, np.float32)
    x, y = np.ascontiguousarray(px, np.int32), np.ascontiguousarray(py, np.int32)
    xf, yf = np.empty(len(x), np.float32), np.empty(len(x), np.float32)
    lib().hpf_refine(_f32(u), u.shape[0], u.shape[1], len(x), _i32(x), _i32(y), _f32(xf), _f32(yf))
    return xf, yf


def smooth(maps, taps):
    """Separable correlation of fp32 maps [..., H, W] with an odd-length tap vector, edges repeated (hp_smooth_oracle.c)."""
    m = np.ascontiguousarray(maps, np.float32)
    t = np.ascontiguousarray(taps, np.float32)
    assert t.ndim == 1 and len(t) % 2 == 1
    H, W = m.shape[-2:]
    out = np.empty_like(m)
    rc = lib().hps_smooth(_f32(m), _f32(out), int(np.prod(m.shape[:-2], dtype=np.int64)), H, W, _f32(t), len(t))
    assert rc == 0
    return out


def in_capsule(px, py, ax, ay, bx, by, thickness):
    return bool(lib().hpv_in_capsule(int(px), int(py), int(ax), int(ay), int(bx), int(by), int(thickness)))


def in_disc(px, py, cx, cy, radius):
    return bool(lib().hpv_in_disc(int(px), int(py), int(cx), int(cy), int(radius)))


def draw_poses(frames, H, W, limb_a, limb_b, peak_x, peak_y, slots, limb_rgb, part_rgb, thickness, radius):
    """Visualisation operator (hp_draw_oracle.c): frames uint8 [N, Hf, Wf, C] -> frames with the poses drawn.

    peak_x / peak_y: int32 [N, K, cap] on a W x H map; slots: per image an int32 [n_persons, K] array of peak
    ranks (-1 = part missing); limb_rgb [L, 3], part_rgb [K, 3] uint8."""
    fr = np.ascontiguousarray(frames, np.uint8)
    N, Hf, Wf, C = fr.shape
    la, lb = np.ascontiguousarray(limb_a, np.int32), np.ascontiguousarray(limb_b, np.int32)
    x, y = np.ascontiguousarray(peak_x, np.int32), np.ascontiguousarray(peak_y, np.int32)
    K, cap = x.shape[1], x.shape[2]
    lrgb, prgb = np.ascontiguousarray(limb_rgb, np.uint8), np.ascontiguousarray(part_rgb, np.uint8)
    assert lrgb.shape == (len(la), 3) and prgb.shape == (K, 3)
    out = np.empty_like(fr)
    u8 = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
    for n in range(N):
        sl = np.ascontiguousarray(slots[n], np.int32).reshape(-1, K)
        lib().hpv_draw(u8(fr[n]), u8(out[n]), Hf, Wf, C, int(H), int(W), K, len(la), _i32(la), _i32(lb), _i32(x[n]),
                       _i32(y[n]), cap, _i32(sl), len(sl), u8(lrgb), u8(prgb), int(thickness), int(radius))
    return out


def find_peaks(plane_hi, thr):
    """Peaks of one fp32 hi-res plane: (x int32[], y int32[], score fp32[]) in raster order."""
    u = np.ascontiguousarray(plane_hi, dtype=np.float32)
    H, W = u.shape
    cap = 256
    while True:
        px = np.empty(cap, np.int32)
        py = np.empty(cap, np.int32)
        ps = np.empty(cap, np.float32)
        n = lib().hpo_find_peaks(_f32(u), H, W, float(thr), cap, _i32(px), _i32(py), _f32(ps))
        if n <= cap:
            return px[:n].copy(), py[:n].copy(), ps[:n].copy()
        cap = n


def need(min_valid_ratio, S):
    return int(lib().hpo_need(float(min_valid_ratio), int(S)))


def score_limb(pafx_lo, pafy_lo, s, xA, yA, xB, yB, n_samples, paf_thr, min_valid_ratio):
    """Accepted candidates (i int32[], j int32[], score fp32[]) of one limb, (i, j) order."""
    pafx_lo = _as_f32(pafx_lo)
    pafy_lo = _as_f32(pafy_lo)
    h, w = pafx_lo.shape
    xA = np.ascontiguousarray(xA, np.int32)
    yA = np.ascontiguousarray(yA, np.int32)
    xB = np.ascontiguousarray(xB, np.int32)
    yB = np.ascontiguousarray(yB, np.int32)
    nd = need(min_valid_ratio, n_samples)
    ccap = max(1024, 4 * max(len(xA), len(xB)))
    while True:
        ci = np.empty(ccap, np.int32)
        cj = np.empty(ccap, np.int32)
        cs = np.empty(ccap, np.float32)
        n = lib().hpo_score_limb(_f32(pafx_lo), _f32(pafy_lo), h, w, s,
                                 len(xA), _i32(xA), _i32(yA), len(xB), _i32(xB), _i32(yB),
                                 int(n_samples), float(paf_thr), nd, ccap, _i32(ci), _i32(cj), _f32(cs))
        if n <= ccap:
            return ci[:n].copy(), cj[:n].copy(), cs[:n].copy()
        ccap = n


def match_limb(ci, cj, cs, nA, nB):
    """Greedy matching: connections (i, j, score) in acceptance order."""
    ci = np.ascontiguousarray(ci, np.int32)
    cj = np.ascontiguousarray(cj, np.int32)
    cs = np.ascontiguousarray(cs, np.float32)
    m = max(min(nA, nB), 1)
    mi = np.empty(m, np.int32)
    mj = np.empty(m, np.int32)
    ms = np.empty(m, np.float32)
    n = lib().hpo_match_limb(len(ci), _i32(ci), _i32(cj), _f32(cs), int(nA), int(nB),
                             _i32(mi), _i32(mj), _f32(ms))
    return mi[:n].copy(), mj[:n].copy(), ms[:n].copy()


def assemble(limb_a, limb_b, K, peak_scores, conns, min_parts):
    """Persons of one image.

    peak_scores: list over parts of fp32 arrays; conns: list over limbs of
    (mi, mj, ms).  Returns (slots int32 [P, K], nparts int32 [P], score fp32 [P]).
    """
    limb_a = np.ascontiguousarray(limb_a, np.int32)
    limb_b = np.ascontiguousarray(limb_b, np.int32)
    L = len(limb_a)
    pcount = np.array([len(p) for p in peak_scores], np.int32)
    pstride = max(int(pcount.max()) if K else 0, 1)
    pscore = np.zeros((K, pstride), np.float32)
    for c in range(K):
        pscore[c, :pcount[c]] = peak_scores[c]
    mcount = np.array([len(c[0]) for c in conns], np.int32)
    mstride = max(int(mcount.max()) if L else 0, 1)
    mi = np.zeros((L, mstride), np.int32)
    mj = np.zeros((L, mstride), np.int32)
    ms = np.zeros((L, mstride), np.float32)
    for l in range(L):
        mi[l, :mcount[l]], mj[l, :mcount[l]], ms[l, :mcount[l]] = conns[l]
    pcap = int(mcount.sum()) + 1
    slots = np.empty((pcap, K), np.int32)
    nparts = np.empty(pcap, np.int32)
    score = np.empty(pcap, np.float32)
    n = lib().hpo_assemble(K, L, _i32(limb_a), _i32(limb_b), _f32(pscore), pstride,
                           _i32(mcount), _i32(mi), _i32(mj), _f32(ms), mstride,
                           int(min_parts), pcap, _i32(slots), _i32(nparts), _f32(score))
    assert n <= pcap
    return slots[:n].copy(), nparts[:n].copy(), score[:n].copy()


def postprocess(cm_lo, paf_lo, limb_a, limb_b, params, threads=1, stages="all"):
    """The whole operator on a batch.

    cm_lo [N, K+1, h, w], paf_lo [N, 2L, h, w] (fp16 or fp32).  The last CM
    channel is background and is not searched.  Returns a dict of ragged
    results:
      peaks[n][c]  = (x, y, score)      candidates[n][l] = (i, j, score)
      conns[n][l]  = (i, j, score)      poses[n] = (slots, nparts, score)
    `threads` farms the independent (image, part) and (image, limb) calls over
    a thread pool (the C calls release the GIL); results do not depend on it.
    """
    cm_lo = _as_f32(cm_lo)
    paf_lo = _as_f32(paf_lo)
    N, C_cm, h, w = cm_lo.shape
    K = C_cm - 1
    L = len(limb_a)
    s = params.scale
    assert paf_lo.shape == (N, 2 * L, h, w)

    def run(fn, items):
        if threads <= 1:
            return [fn(it) for it in items]
        with ThreadPoolExecutor(threads) as ex:
            return list(ex.map(fn, items))

    def peaks_of(nc):
        n, c = nc
        return find_peaks(resize(cm_lo[n, c], s), params.peak_thr)

    flat = run(peaks_of, [(n, c) for n in range(N) for c in range(K)])
    peaks = [[flat[n * K + c] for c in range(K)] for n in range(N)]
    out = {"peaks": peaks}
    if stages == "peaks":
        return out

    def limb_of(nl):
        n, l = nl
        a, b = int(limb_a[l]), int(limb_b[l])
        xA, yA, _ = peaks[n][a]
        xB, yB, _ = peaks[n][b]
        cand = score_limb(paf_lo[n, 2 * l], paf_lo[n, 2 * l + 1], s, xA, yA, xB, yB,
                          params.n_samples, params.paf_thr, params.min_valid_ratio)
        conn = match_limb(*cand, len(xA), len(xB))
        return cand, conn

    flat = run(limb_of, [(n, l) for n in range(N) for l in range(L)])
    out["candidates"] = [[flat[n * L + l][0] for l in range(L)] for n in range(N)]
    out["conns"] = [[flat[n * L + l][1] for l in range(L)] for n in range(N)]

    def person_of(n):
        return assemble(limb_a, limb_b, K, [p[2] for p in peaks[n]], out["conns"][n], params.min_parts)

    out["poses"] = run(person_of, list(range(N)))
    return out
