"""ctypes binding of libhp.so: argument marshalling only, every step runs in the library.

The functions carry the names of the C entry points (include/hp.h).  Tensors are torch
tensors on the GPU; the current torch stream is passed as the HIP stream.  There is no
fallback: if the library is missing, loading raises.
"""
import ctypes
import os
from ctypes import POINTER, Structure, c_float, c_int, c_int32, c_int64, c_size_t, c_uint64, c_void_p

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))

HP_F32, HP_F16 = 0, 1
STATUS_PEAK_OVERFLOW, STATUS_CAND_OVERFLOW, STATUS_POSE_OVERFLOW = 1, 2, 4

EXPORTS = ("hp_workspace_bytes", "hp_workspace_init", "hp_resize", "hp_find_peaks", "hp_score_limbs", "hp_assemble",
           "hp_postprocess", "hp_postprocess_static", "hp_preprocess", "hp_smooth", "hp_refine_peaks", "hp_pp_decode", "hp_cf_decode", "hp_cf_field", "hp_cf_workspace_bytes", "hp_draw_poses", "hp_draw_workspace_bytes", "hp_profile_begin", "hp_profile_end", "hp_kernel_name", "hp_strerror", "hp_version",
           "hp_batcher_create", "hp_batcher_destroy", "hp_batcher_acquire", "hp_batcher_commit", "hp_batcher_submit",
           "hp_batcher_flush", "hp_batcher_next", "hp_batcher_release", "hp_batch_simulate", "hp_batcher_drive",
           "hp_bench_copy")
HP_ERR_BUSY, HP_ERR_TIMEOUT, HP_ERR_STATE = -6, -7, -8
HP_K_COUNT = 22


class HPError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {hp_strerror(code)} ({code})")


class _Skeleton(Structure):
    _fields_ = [("n_parts", c_int32), ("n_limbs", c_int32),
                ("limb_a", POINTER(c_int32)), ("limb_b", POINTER(c_int32))]


class _Params(Structure):
    _fields_ = [("peak_thr", c_float), ("paf_thr", c_float), ("n_samples", c_int32),
                ("min_valid_ratio", c_float), ("min_parts", c_int32), ("scale", c_int32)]


class _Peaks(Structure):
    _fields_ = [("x", c_void_p), ("y", c_void_p), ("score", c_void_p), ("count", c_void_p), ("cap", c_int32)]


class _Pairs(Structure):
    _fields_ = [("i", c_void_p), ("j", c_void_p), ("score", c_void_p), ("count", c_void_p), ("cap", c_int32)]


class _Poses(Structure):
    _fields_ = [("slots", c_void_p), ("nparts", c_void_p), ("score", c_void_p), ("count", c_void_p),
                ("cap", c_int32)]


class _PPParams(Structure):
    _fields_ = [("det_thr", c_float), ("nms_thr", c_float), ("edge_thr", c_float), ("min_parts", c_int32),
                ("img_w", c_float), ("img_h", c_float)]


class _CFParams(Structure):
    _fields_ = [("pif_thr", c_float), ("paf_thr", c_float), ("seed_thr", c_float), ("grow_thr", c_float),
                ("rev_tol", c_float), ("min_parts", c_int32), ("stride", c_int32)]


class _CFLists(Structure):
    _fields_ = [("pif_cell", c_void_p), ("pif_val", c_void_p), ("pif_count", c_void_p), ("paf_cell", c_void_p),
                ("paf_f1", c_void_p), ("paf_f2", c_void_p), ("paf_count", c_void_p), ("cap", c_int32), ("acap", c_int32)]


class _CFPoses(Structure):
    _fields_ = [("xyv", c_void_p), ("nparts", c_void_p), ("score", c_void_p), ("count", c_void_p), ("cap", c_int32)]


class _PPDets(Structure):
    _fields_ = [("cell", c_void_p), ("score", c_void_p), ("box", c_void_p), ("count", c_void_p), ("cap", c_int32)]


class _Lane(Structure):
    _fields_ = [("cm_lo", c_void_p), ("paf_lo", c_void_p), ("peaks", _Peaks), ("cands", _Pairs), ("conns", _Pairs),
                ("poses", _Poses), ("workspace", c_void_p), ("ws_bytes", c_size_t), ("status", c_void_p),
                ("stream", c_void_p)]


class _BatcherConfig(Structure):
    _fields_ = [("max_batch", c_int32), ("depth", c_int32), ("n_lanes", c_int32)]


class _BatchInfo(Structure):
    _fields_ = [("lane", c_int32), ("n_frames", c_int32), ("rc", c_int32), ("reserved", c_int32),
                ("seq", c_uint64), ("start_ns", c_int64), ("done_ns", c_int64)]


def lib_path():
    return os.path.join(_PKG, "libhp.so")


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2108_11826_amd.build)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: build it with `python -m paper_2108_11826_amd.build`")
        L = ctypes.CDLL(path)
        L.hp_workspace_bytes.restype = c_size_t
        L.hp_workspace_bytes.argtypes = [c_int] * 9
        L.hp_workspace_init.restype = c_int
        L.hp_workspace_init.argtypes = [c_void_p, c_size_t, c_void_p]
        L.hp_resize.restype = c_int
        L.hp_resize.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p]
        L.hp_find_peaks.restype = c_int
        L.hp_find_peaks.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_int, c_float, POINTER(_Peaks),
                                    c_void_p, c_size_t, c_void_p, c_void_p]
        L.hp_score_limbs.restype = c_int
        L.hp_score_limbs.argtypes = [c_void_p, c_int, c_int, c_int, POINTER(_Skeleton), POINTER(_Params),
                                     POINTER(_Peaks), POINTER(_Pairs), c_void_p, c_size_t, c_void_p, c_void_p]
        L.hp_assemble.restype = c_int
        L.hp_assemble.argtypes = [POINTER(_Skeleton), POINTER(_Params), c_int, POINTER(_Peaks), POINTER(_Pairs),
                                  POINTER(_Pairs), POINTER(_Poses), c_void_p, c_size_t, c_void_p, c_void_p]
        L.hp_postprocess.restype = c_int
        L.hp_postprocess.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, POINTER(_Skeleton),
                                     POINTER(_Params), c_void_p, c_void_p, POINTER(_Peaks), POINTER(_Pairs),
                                     POINTER(_Pairs), POINTER(_Poses), c_void_p, c_size_t, c_void_p, c_void_p]
        L.hp_postprocess_static.restype = c_int
        L.hp_postprocess_static.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, POINTER(_Skeleton),
                                            POINTER(_Params), c_void_p, c_void_p, POINTER(_Peaks), POINTER(_Pairs),
                                            POINTER(_Pairs), POINTER(_Poses), c_void_p, c_void_p]
        L.hp_preprocess.restype = c_int
        L.hp_preprocess.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p, c_int, c_int, c_int,
                                    POINTER(c_float), POINTER(c_float), c_void_p]
        L.hp_pp_decode.restype = c_int
        L.hp_pp_decode.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, POINTER(_Skeleton),
                                   POINTER(_PPParams), POINTER(_PPDets), POINTER(_Poses), c_void_p, c_void_p]
        L.hp_refine_peaks.restype = c_int
        L.hp_refine_peaks.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_int, POINTER(_Peaks), c_void_p, c_void_p, c_void_p]
        L.hp_smooth.restype = c_int
        L.hp_smooth.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p, c_int, c_void_p]
        L.hp_draw_poses.restype = c_int
        L.hp_draw_poses.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, POINTER(_Skeleton),
                                    POINTER(_Peaks), POINTER(_Poses), POINTER(ctypes.c_uint8), POINTER(ctypes.c_uint8),
                                    c_int, c_int, c_void_p, c_size_t, c_void_p]
        L.hp_cf_workspace_bytes.restype = c_size_t
        L.hp_cf_workspace_bytes.argtypes = [c_int] * 5
        L.hp_cf_decode.restype = c_int
        L.hp_cf_decode.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, POINTER(_Skeleton), POINTER(_CFParams),
                                   POINTER(_CFLists), POINTER(_CFPoses), c_void_p, c_size_t, c_void_p, c_void_p]
        L.hp_cf_field.restype = c_int
        L.hp_cf_field.argtypes = [c_void_p, c_int, c_int, c_int, c_int, POINTER(_CFParams), c_void_p, c_void_p, c_void_p,
                                  c_int, c_void_p, c_void_p, c_size_t, c_void_p, c_void_p]
        L.hp_draw_workspace_bytes.restype = c_size_t
        L.hp_draw_workspace_bytes.argtypes = [c_int] * 6
        L.hp_batcher_create.restype = c_int
        L.hp_batcher_create.argtypes = [c_int, c_int, c_int, POINTER(_Skeleton), POINTER(_Params),
                                        POINTER(_BatcherConfig), POINTER(_Lane), POINTER(c_void_p)]
        L.hp_batcher_destroy.restype = c_int
        L.hp_batcher_destroy.argtypes = [c_void_p]
        L.hp_batcher_acquire.restype = c_int
        L.hp_batcher_acquire.argtypes = [c_void_p, c_int, POINTER(c_void_p), POINTER(c_void_p)]
        L.hp_batcher_commit.restype = c_int
        L.hp_batcher_commit.argtypes = [c_void_p, c_uint64, c_void_p, c_int]
        L.hp_batcher_submit.restype = c_int
        L.hp_batcher_submit.argtypes = [c_void_p, c_int, c_void_p, c_void_p, c_uint64, c_void_p, c_int]
        L.hp_batcher_flush.restype = c_int
        L.hp_batcher_flush.argtypes = [c_void_p]
        L.hp_batcher_next.restype = c_int
        L.hp_batcher_next.argtypes = [c_void_p, c_int, POINTER(_BatchInfo), POINTER(c_uint64), POINTER(c_int64)]
        L.hp_batcher_release.restype = c_int
        L.hp_batcher_release.argtypes = [c_void_p, c_int]
        L.hp_batch_simulate.restype = c_int
        L.hp_batch_simulate.argtypes = [c_int, POINTER(c_int64), POINTER(_BatcherConfig), c_int64, c_int64,
                                        POINTER(c_int64), POINTER(c_int32), POINTER(c_int64)]
        L.hp_batcher_drive.restype = c_int
        L.hp_batcher_drive.argtypes = [c_void_p, c_int, c_int64, c_int, c_void_p, c_void_p, c_int,
                                       POINTER(c_int64), POINTER(c_int32), POINTER(c_int64)]
        L.hp_bench_copy.restype = c_int
        L.hp_bench_copy.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
        L.hp_profile_begin.restype = c_int
        L.hp_profile_begin.argtypes = [c_int]
        L.hp_profile_end.restype = c_int
        L.hp_profile_end.argtypes = [POINTER(c_float), POINTER(c_int32)]
        L.hp_kernel_name.restype = ctypes.c_char_p
        L.hp_kernel_name.argtypes = [c_int]
        L.hp_strerror.restype = ctypes.c_char_p
        L.hp_strerror.argtypes = [c_int]
        L.hp_version.restype = c_int
        L.hp_version.argtypes = []
        _lib = L
    return _lib


def hp_strerror(code):
    return lib().hp_strerror(int(code)).decode()


def hp_version():
    return int(lib().hp_version())


def hp_bench_copy(dst, src):
    """Plain copy of one GPU tensor into another of the same size by a kernel of the library (counter calibration)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("sizes differ")
    _check(lib().hp_bench_copy(_dev(dst), _dev(src), c_size_t(nbytes), _stream()), "hp_bench_copy")


def hp_profile_begin(max_launches):
    _check(lib().hp_profile_begin(int(max_launches)), "hp_profile_begin")


def hp_profile_end():
    """{kernel name: (total ms, launches)} of the launches recorded since hp_profile_begin."""
    ms = (c_float * HP_K_COUNT)()
    n = (c_int32 * HP_K_COUNT)()
    _check(lib().hp_profile_end(ms, n), "hp_profile_end")
    return {lib().hp_kernel_name(k).decode(): (float(ms[k]), int(n[k])) for k in range(HP_K_COUNT) if n[k] > 0}


def hp_workspace_init(workspace):
    """Clears a workspace tensor (uint8, on the GPU) on the current stream."""
    _check(lib().hp_workspace_init(_dev(workspace, torch.uint8), c_size_t(workspace.numel()), _stream()),
           "hp_workspace_init")


def hp_workspace_bytes(N, K, L, h, w, scale, cap, ccap, pcap):
    return int(lib().hp_workspace_bytes(N, K, L, h, w, scale, cap, ccap, pcap))


class Skeleton:
    """Host-side skeleton descriptor (keeps the limb arrays alive)."""

    def __init__(self, n_parts, limb_a, limb_b):
        self.limb_a = np.ascontiguousarray(limb_a, np.int32)
        self.limb_b = np.ascontiguousarray(limb_b, np.int32)
        self.n_parts = int(n_parts)
        self.n_limbs = len(self.limb_a)
        self.c = _Skeleton(self.n_parts, self.n_limbs,
                           self.limb_a.ctypes.data_as(POINTER(c_int32)),
                           self.limb_b.ctypes.data_as(POINTER(c_int32)))


class Params:
    def __init__(self, peak_thr=0.05, paf_thr=0.05, n_samples=10, min_valid_ratio=0.8, min_parts=3, scale=8):
        self.c = _Params(peak_thr, paf_thr, n_samples, min_valid_ratio, min_parts, scale)
        self.peak_thr, self.scale = float(peak_thr), int(scale)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return HP_F32
    if t.dtype == torch.float16:
        return HP_F16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t, dtype=None):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError("expected a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


class Buffers:
    """Caller-owned output buffers and workspace for a given problem size, allocated once."""

    def __init__(self, N, K, L, h, w, cap, ccap, pcap, device="cuda:0", scale=8):
        self.N, self.K, self.L, self.h, self.w = N, K, L, h, w
        self.cap, self.ccap, self.pcap = cap, ccap, pcap
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.px, self.py = torch.empty((N, K, cap), **i32), torch.empty((N, K, cap), **i32)
        self.ps, self.pcount = torch.empty((N, K, cap), **f32), torch.empty((N, K), **i32)
        self.ci, self.cj = torch.empty((N, L, ccap), **i32), torch.empty((N, L, ccap), **i32)
        self.cs, self.ccount = torch.empty((N, L, ccap), **f32), torch.empty((N, L), **i32)
        self.mi, self.mj = torch.empty((N, L, cap), **i32), torch.empty((N, L, cap), **i32)
        self.ms, self.mcount = torch.empty((N, L, cap), **f32), torch.empty((N, L), **i32)
        self.slots = torch.empty((N, pcap, K), **i32)
        self.nparts, self.pscore = torch.empty((N, pcap), **i32), torch.empty((N, pcap), **f32)
        self.pose_count = torch.empty((N,), **i32)
        self.status = torch.zeros((1,), **i32)
        self.ws_bytes = hp_workspace_bytes(N, K, L, h, w, scale, cap, ccap, pcap)
        if self.ws_bytes == 0:
            raise HPError(-1, "hp_workspace_bytes")
        self.workspace = torch.empty((self.ws_bytes,), dtype=torch.uint8, device=device)
        with torch.cuda.device(self.workspace.device):
            _check(lib().hp_workspace_init(c_void_p(self.workspace.data_ptr()), c_size_t(self.ws_bytes), _stream()),
                   "hp_workspace_init")
        self.peaks = _Peaks(self.px.data_ptr(), self.py.data_ptr(), self.ps.data_ptr(), self.pcount.data_ptr(), cap)
        self.cands = _Pairs(self.ci.data_ptr(), self.cj.data_ptr(), self.cs.data_ptr(), self.ccount.data_ptr(), ccap)
        self.conns = _Pairs(self.mi.data_ptr(), self.mj.data_ptr(), self.ms.data_ptr(), self.mcount.data_ptr(), cap)
        self.poses = _Poses(self.slots.data_ptr(), self.nparts.data_ptr(), self.pscore.data_ptr(),
                            self.pose_count.data_ptr(), pcap)

    def ws(self):
        return c_void_p(self.workspace.data_ptr()), c_size_t(self.ws_bytes)

    # ---- host copies as ragged lists (for tests and reports) ---------------
    def host_status(self):
        return int(self.status.cpu()[0])

    def host_peaks(self):
        cnt = self.pcount.cpu().numpy()
        x, y, s = self.px.cpu().numpy(), self.py.cpu().numpy(), self.ps.cpu().numpy()
        return [[(x[n, c, :min(cnt[n, c], self.cap)].copy(), y[n, c, :min(cnt[n, c], self.cap)].copy(),
                  s[n, c, :min(cnt[n, c], self.cap)].copy()) for c in range(self.K)] for n in range(self.N)], cnt

    def _host_pairs(self, i, j, s, count, cap):
        cnt = count.cpu().numpy()
        i, j, s = i.cpu().numpy(), j.cpu().numpy(), s.cpu().numpy()
        return [[(i[n, l, :min(cnt[n, l], cap)].copy(), j[n, l, :min(cnt[n, l], cap)].copy(),
                  s[n, l, :min(cnt[n, l], cap)].copy()) for l in range(self.L)] for n in range(self.N)], cnt

    def host_cands(self):
        return self._host_pairs(self.ci, self.cj, self.cs, self.ccount, self.ccap)

    def host_conns(self):
        return self._host_pairs(self.mi, self.mj, self.ms, self.mcount, self.cap)

    def host_poses(self):
        cnt = self.pose_count.cpu().numpy()
        sl, npt, sc = self.slots.cpu().numpy(), self.nparts.cpu().numpy(), self.pscore.cpu().numpy()
        return [(sl[n, :min(cnt[n], self.pcap)].copy(), npt[n, :min(cnt[n], self.pcap)].copy(),
                 sc[n, :min(cnt[n], self.pcap)].copy()) for n in range(self.N)], cnt


def _check(rc, where):
    if rc != 0:
        raise HPError(rc, where)


def hp_resize(src_lo, dst_hi=None, scale=8):
    """src_lo [N, C, h, w] fp32/fp16 on the GPU -> dst_hi fp32 [N, C, 8h, 8w]."""
    N, C, h, w = src_lo.shape
    if dst_hi is None:
        dst_hi = torch.empty((N, C, scale * h, scale * w), dtype=torch.float32, device=src_lo.device)
    _check(lib().hp_resize(_dev(src_lo), _dtype_code(src_lo), N, C, h, w, scale, _dev(dst_hi, torch.float32),
                           _stream()), "hp_resize")
    return dst_hi


def hp_find_peaks(cm_hi, K, thr, buf):
    N, C_cm, H, W = cm_hi.shape
    wsp, wsb = buf.ws()
    _check(lib().hp_find_peaks(_dev(cm_hi, torch.float32), N, C_cm, K, H, W, thr, ctypes.byref(buf.peaks),
                               wsp, wsb, _dev(buf.status), _stream()), "hp_find_peaks")


def hp_score_limbs(paf_hi, skel, prm, buf):
    N, C, H, W = paf_hi.shape
    wsp, wsb = buf.ws()
    _check(lib().hp_score_limbs(_dev(paf_hi, torch.float32), N, H, W, ctypes.byref(skel.c), ctypes.byref(prm.c),
                                ctypes.byref(buf.peaks), ctypes.byref(buf.cands), wsp, wsb, _dev(buf.status),
                                _stream()), "hp_score_limbs")


def hp_assemble(skel, prm, buf):
    wsp, wsb = buf.ws()
    _check(lib().hp_assemble(ctypes.byref(skel.c), ctypes.byref(prm.c), buf.N, ctypes.byref(buf.peaks),
                             ctypes.byref(buf.cands), ctypes.byref(buf.conns), ctypes.byref(buf.poses),
                             wsp, wsb, _dev(buf.status), _stream()), "hp_assemble")


def hp_postprocess(cm_lo, paf_lo, skel, prm, buf, cm_hi=None, paf_hi=None):
    N, C_cm, h, w = cm_lo.shape
    if cm_lo.dtype != paf_lo.dtype:
        raise TypeError("cm_lo and paf_lo must share a dtype")
    wsp, wsb = buf.ws()
    _check(lib().hp_postprocess(_dev(cm_lo), _dev(paf_lo), _dtype_code(cm_lo), N, h, w,
                                ctypes.byref(skel.c), ctypes.byref(prm.c),
                                _dev(cm_hi, torch.float32) if cm_hi is not None else None,
                                _dev(paf_hi, torch.float32) if paf_hi is not None else None,
                                ctypes.byref(buf.peaks), ctypes.byref(buf.cands), ctypes.byref(buf.conns),
                                ctypes.byref(buf.poses), wsp, wsb, _dev(buf.status), _stream()),
           "hp_postprocess")


def hp_postprocess_static(cm_lo, paf_lo, skel, prm, buf, cm_hi=None, paf_hi=None):
    """hp_postprocess on the library's own fixed workspace (buf's outputs are used, its workspace is not)."""
    N, C_cm, h, w = cm_lo.shape
    if cm_lo.dtype != paf_lo.dtype:
        raise TypeError("cm_lo and paf_lo must share a dtype")
    _check(lib().hp_postprocess_static(_dev(cm_lo), _dev(paf_lo), _dtype_code(cm_lo), N, h, w,
                                       ctypes.byref(skel.c), ctypes.byref(prm.c),
                                       _dev(cm_hi, torch.float32) if cm_hi is not None else None,
                                       _dev(paf_hi, torch.float32) if paf_hi is not None else None,
                                       ctypes.byref(buf.peaks), ctypes.byref(buf.cands), ctypes.byref(buf.conns),
                                       ctypes.byref(buf.poses), _dev(buf.status), _stream()),
           "hp_postprocess_static")


def hp_preprocess(images, Hd, Wd, alpha, beta, reverse_channels=False, out=None, dtype=torch.float32):
    """images uint8 [N, Hs, Ws, C] on the GPU -> `dtype` [N, C, Hd, Wd] (resize + channel-first + scale/offset)."""
    N, Hs, Ws, C = images.shape
    if out is None:
        out = torch.empty((N, C, Hd, Wd), dtype=dtype, device=images.device)
    al = (c_float * C)(*np.broadcast_to(np.asarray(alpha, np.float32), (C,)).tolist())
    be = (c_float * C)(*np.broadcast_to(np.asarray(beta, np.float32), (C,)).tolist())
    _check(lib().hp_preprocess(_dev(images, torch.uint8), N, Hs, Ws, C, _dtype_code(out), _dev(out), int(Hd), int(Wd),
                               1 if reverse_channels else 0, al, be, _stream()), "hp_preprocess")
    return out


class PPBuffers:
    """Caller-owned outputs of hp_pp_decode: detection lists per (image, part) and persons per image."""

    def __init__(self, N, K, cap, pcap, device="cuda:0"):
        self.N, self.K, self.cap, self.pcap = N, K, cap, pcap
        i32, f32 = dict(dtype=torch.int32, device=device), dict(dtype=torch.float32, device=device)
        self.cell, self.score = torch.zeros((N, K, cap), **i32), torch.zeros((N, K, cap), **f32)
        self.box, self.count = torch.zeros((N, K, cap, 4), **f32), torch.zeros((N, K), **i32)
        self.slots, self.nparts = torch.zeros((N, pcap, K), **i32), torch.zeros((N, pcap), **i32)
        self.pscore, self.pose_count = torch.zeros((N, pcap), **f32), torch.zeros((N,), **i32)
        self.status = torch.zeros((1,), **i32)
        self.dets = _PPDets(self.cell.data_ptr(), self.score.data_ptr(), self.box.data_ptr(), self.count.data_ptr(), cap)
        self.poses = _Poses(self.slots.data_ptr(), self.nparts.data_ptr(), self.pscore.data_ptr(),
                            self.pose_count.data_ptr(), pcap)

    def host(self):
        """{"dets": [n][k] -> (cell, score, corners), "poses": [n] -> (slots, nparts, score), "status": int}."""
        cnt, pc = self.count.cpu().numpy(), self.pose_count.cpu().numpy()
        cell, score, box = self.cell.cpu().numpy(), self.score.cpu().numpy(), self.box.cpu().numpy()
        sl, npt, ps = self.slots.cpu().numpy(), self.nparts.cpu().numpy(), self.pscore.cpu().numpy()
        dets = [[(cell[n, k, :min(cnt[n, k], self.cap)].copy(), score[n, k, :min(cnt[n, k], self.cap)].copy(),
                  box[n, k, :min(cnt[n, k], self.cap)].copy()) for k in range(self.K)] for n in range(self.N)]
        poses = [(sl[n, :min(pc[n], self.pcap)].copy(), npt[n, :min(pc[n], self.pcap)].copy(),
                  ps[n, :min(pc[n], self.pcap)].copy()) for n in range(self.N)]
        return {"dets": dets, "poses": poses, "det_counts": cnt, "pose_counts": pc, "status": int(self.status.cpu()[0])}


def hp_pp_decode(resp, conf, box, edge, skel, buf, img_w, img_h, det_thr, nms_thr, edge_thr, min_parts):
    """Pose-proposal post-processing: resp, conf [N, K, Gh, Gw]; box [N, K, 4, Gh, Gw]; edge [N, L, Nh, Nw, Gh, Gw]
    (fp32 on the GPU) -> buf (a PPBuffers)."""
    N, K, Gh, Gw = resp.shape
    Nh, Nw = edge.shape[2], edge.shape[3]
    prm = _PPParams(det_thr, nms_thr, edge_thr, int(min_parts), img_w, img_h)
    _check(lib().hp_pp_decode(_dev(resp, torch.float32), _dev(conf, torch.float32), _dev(box, torch.float32),
                              _dev(edge, torch.float32), N, Gh, Gw, Nh, Nw, ctypes.byref(skel.c), ctypes.byref(prm),
                              ctypes.byref(buf.dets), ctypes.byref(buf.poses), _dev(buf.status), _stream()), "hp_pp_decode")


class CFBuffers:
    """Caller-owned outputs and workspace of hp_cf_decode: the active cells per (image, part) and (image, limb), and the
    persons per image."""

    def __init__(self, N, K, L, cap, acap, pcap, device="cuda:0"):
        self.N, self.K, self.L, self.cap, self.acap, self.pcap = N, K, L, cap, acap, pcap
        i32, f32 = dict(dtype=torch.int32, device=device), dict(dtype=torch.float32, device=device)
        self.pif_cell, self.pif_val = torch.zeros((N, K, cap), **i32), torch.zeros((N, K, cap), **f32)
        self.pif_count = torch.zeros((N, K), **i32)
        self.paf_cell, self.paf_count = torch.zeros((N, L, acap), **i32), torch.zeros((N, L), **i32)
        self.paf_f1, self.paf_f2 = torch.zeros((N, L, acap), **f32), torch.zeros((N, L, acap), **f32)
        self.xyv, self.nparts = torch.zeros((N, pcap, K, 3), **f32), torch.zeros((N, pcap), **i32)
        self.pscore, self.pose_count = torch.zeros((N, pcap), **f32), torch.zeros((N,), **i32)
        self.status = torch.zeros((1,), **i32)
        self.workspace = torch.empty((hp_cf_workspace_bytes(N, K, L, cap, acap),), dtype=torch.uint8, device=device)
        self.lists = _CFLists(self.pif_cell.data_ptr(), self.pif_val.data_ptr(), self.pif_count.data_ptr(),
                              self.paf_cell.data_ptr(), self.paf_f1.data_ptr(), self.paf_f2.data_ptr(),
                              self.paf_count.data_ptr(), cap, acap)
        self.poses = _CFPoses(self.xyv.data_ptr(), self.nparts.data_ptr(), self.pscore.data_ptr(),
                              self.pose_count.data_ptr(), pcap)

    def host(self):
        """{"pif": [n][k] -> (cell, value), "paf": [n][l] -> (cell, F1, F2), "poses": [n] -> (xyv, nparts, score), ...}."""
        pn, an, pc = self.pif_count.cpu().numpy(), self.paf_count.cpu().numpy(), self.pose_count.cpu().numpy()
        pcell, pval = self.pif_cell.cpu().numpy(), self.pif_val.cpu().numpy()
        acell, f1, f2 = self.paf_cell.cpu().numpy(), self.paf_f1.cpu().numpy(), self.paf_f2.cpu().numpy()
        xyv, npt, ps = self.xyv.cpu().numpy(), self.nparts.cpu().numpy(), self.pscore.cpu().numpy()
        pif = [[(pcell[n, k, :min(pn[n, k], self.cap)].copy(), pval[n, k, :min(pn[n, k], self.cap)].copy())
                for k in range(self.K)] for n in range(self.N)]
        paf = [[tuple(a[n, l, :min(an[n, l], self.acap)].copy() for a in (acell, f1, f2)) for l in range(self.L)]
               for n in range(self.N)]
        poses = [(xyv[n, :pc[n]].copy(), npt[n, :pc[n]].copy(), ps[n, :pc[n]].copy()) for n in range(self.N)]
        return {"pif": pif, "paf": paf, "poses": poses, "pif_counts": pn, "paf_counts": an, "pose_counts": pc,
                "status": int(self.status.cpu()[0])}


def hp_cf_workspace_bytes(N, K, L, cap, acap):
    return int(lib().hp_cf_workspace_bytes(int(N), int(K), int(L), int(cap), int(acap)))


def hp_cf_decode(pif, paf, skel, buf, stride, pif_thr, paf_thr, seed_thr, grow_thr, rev_tol, min_parts):
    """Composite-field decoding: pif [N, K, 5, Fh, Fw], paf [N, L, 7, Fh, Fw] (fp32 on the GPU) -> buf (a CFBuffers)."""
    N, K, _, Fh, Fw = pif.shape
    prm = _CFParams(pif_thr, paf_thr, seed_thr, grow_thr, rev_tol, int(min_parts), int(stride))
    _check(lib().hp_cf_decode(_dev(pif, torch.float32), _dev(paf, torch.float32), N, Fh, Fw, ctypes.byref(skel.c),
                              ctypes.byref(prm), ctypes.byref(buf.lists), ctypes.byref(buf.poses),
                              _dev(buf.workspace, torch.uint8), c_size_t(buf.workspace.numel()), _dev(buf.status), _stream()),
           "hp_cf_decode")


def hp_cf_field(pif, stride, pif_thr, cap=256, out=None):
    """The fine confidence maps [N, K, Fh * stride, Fw * stride] of intensity fields pif [N, K, 5, Fh, Fw] (fp32 on the
    GPU); returns (maps, status) with status a one-element int32 GPU tensor."""
    N, K, _, Fh, Fw = pif.shape
    dev = pif.device
    if out is None:
        out = torch.empty((N, K, Fh * stride, Fw * stride), dtype=torch.float32, device=dev)
    cell = torch.empty((N, K, cap), dtype=torch.int32, device=dev)
    val = torch.empty((N, K, cap), dtype=torch.float32, device=dev)
    count = torch.empty((N, K), dtype=torch.int32, device=dev)
    status = torch.zeros((1,), dtype=torch.int32, device=dev)
    ws = torch.empty((hp_cf_workspace_bytes(N, K, 0, cap, 0),), dtype=torch.uint8, device=dev)
    prm = _CFParams(pif_thr, 0.0, 0.0, 0.0, 0.0, 0, int(stride))
    _check(lib().hp_cf_field(_dev(pif, torch.float32), N, K, Fh, Fw, ctypes.byref(prm), _dev(cell), _dev(val), _dev(count),
                             int(cap), _dev(out, torch.float32), _dev(ws, torch.uint8), c_size_t(ws.numel()), _dev(status),
                             _stream()), "hp_cf_field")
    return out, status


def hp_refine_peaks(maps_hi, K, buf):
    """Sub-pixel positions of buf's peaks on maps_hi (fp32 [N, C_mem, H, W]): (xf, yf), fp32 [N, K, cap] on the GPU."""
    N, C_mem, H, W = maps_hi.shape
    xf = torch.zeros((N, K, buf.cap), dtype=torch.float32, device=maps_hi.device)
    yf = torch.zeros_like(xf)
    _check(lib().hp_refine_peaks(_dev(maps_hi, torch.float32), N, C_mem, int(K), H, W, ctypes.byref(buf.peaks),
                                 _dev(xf), _dev(yf), _stream()), "hp_refine_peaks")
    return xf, yf


def hp_smooth(maps_hi, taps, channels=None, out=None):
    """maps_hi fp32 [N, C_mem, H, W] on the GPU -> the first `channels` channels (default: all) smoothed with `taps`
    (a 1-D fp32 GPU tensor of odd length); other channels of `out` are left as they are."""
    N, C_mem, H, W = maps_hi.shape
    C = C_mem if channels is None else int(channels)
    if out is None:
        out = torch.empty_like(maps_hi)
    _check(lib().hp_smooth(_dev(maps_hi, torch.float32), _dev(out, torch.float32), N, C, C_mem, H, W,
                           _dev(taps, torch.float32), int(taps.numel()), _stream()), "hp_smooth")
    return out


def hp_draw_workspace_bytes(N, K, L, pcap, Hf, Wf):
    return int(lib().hp_draw_workspace_bytes(int(N), int(K), int(L), int(pcap), int(Hf), int(Wf)))


def hp_draw_poses(frames, H, W, skel, buf, limb_rgb, part_rgb, thickness=4, radius=4, out=None, workspace=None):
    """frames uint8 [N, Hf, Wf, C] on the GPU -> the frames with buf's poses drawn (out may be `frames` itself).

    `workspace` is a uint8 GPU tensor of hp_draw_workspace_bytes(N, K, L, pcap, Hf, Wf) bytes; without one, a tensor kept
    on `buf` is used (allocated at the first call)."""
    N, Hf, Wf, C = frames.shape
    if out is None:
        out = torch.empty_like(frames)
    if workspace is None:
        workspace = getattr(buf, "draw_workspace", None)
        need = hp_draw_workspace_bytes(N, skel.n_parts, skel.n_limbs, buf.pcap, Hf, Wf)
        if workspace is None or workspace.numel() < need:
            workspace = buf.draw_workspace = torch.empty((need,), dtype=torch.uint8, device=frames.device)
    lrgb = np.ascontiguousarray(limb_rgb, np.uint8)
    prgb = np.ascontiguousarray(part_rgb, np.uint8)
    if lrgb.shape != (skel.n_limbs, 3) or prgb.shape != (skel.n_parts, 3):
        raise ValueError("limb_rgb / part_rgb must be [n_limbs, 3] / [n_parts, 3]")
    u8 = lambda a: a.ctypes.data_as(POINTER(ctypes.c_uint8))
    _check(lib().hp_draw_poses(_dev(frames, torch.uint8), _dev(out, torch.uint8), N, Hf, Wf, C, int(H), int(W),
                               ctypes.byref(skel.c), ctypes.byref(buf.peaks), ctypes.byref(buf.poses), u8(lrgb), u8(prgb),
                               int(thickness), int(radius), _dev(workspace, torch.uint8), c_size_t(workspace.numel()),
                               _stream()), "hp_draw_poses")
    return out


class PostprocessCall:
    """hp_postprocess with its arguments marshalled once, for loops that repeat the same call.

    The tensors, descriptors and the stream are fixed at construction (the stream defaults to the
    current torch stream); calling the object enqueues one hp_postprocess on that stream.
    """

    def __init__(self, cm_lo, paf_lo, skel, prm, buf, cm_hi=None, paf_hi=None, stream=None):
        N, C_cm, h, w = cm_lo.shape
        if cm_lo.dtype != paf_lo.dtype:
            raise TypeError("cm_lo and paf_lo must share a dtype")
        self._keep = (cm_lo, paf_lo, skel, prm, buf, cm_hi, paf_hi, stream)
        wsp, wsb = buf.ws()
        st = stream if stream is not None else torch.cuda.current_stream()
        self._fn = lib().hp_postprocess
        self._args = (_dev(cm_lo), _dev(paf_lo), _dtype_code(cm_lo), N, h, w, ctypes.byref(skel.c),
                      ctypes.byref(prm.c),
                      _dev(cm_hi, torch.float32) if cm_hi is not None else None,
                      _dev(paf_hi, torch.float32) if paf_hi is not None else None,
                      ctypes.byref(buf.peaks), ctypes.byref(buf.cands), ctypes.byref(buf.conns),
                      ctypes.byref(buf.poses), wsp, wsb, _dev(buf.status), c_void_p(st.cuda_stream))

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != 0:
            raise HPError(rc, "hp_postprocess")


# ---- streaming front: the dynamic batch slot in front of hp_postprocess ------------------------

class BatcherLanes:
    """Caller-owned buffers of a batcher: per lane a stream, frame staging for max_batch frames and a Buffers."""

    def __init__(self, n_lanes, max_batch, K, L, h, w, cap, ccap, pcap, dtype=torch.float32, device="cuda:0"):
        self.n_lanes, self.max_batch = int(n_lanes), int(max_batch)
        self.dtype, self.h, self.w, self.K, self.L = dtype, h, w, K, L
        with torch.cuda.device(device):
            self.streams = [torch.cuda.Stream() for _ in range(self.n_lanes)]
            self.cm = [torch.zeros((max_batch, K + 1, h, w), dtype=dtype, device=device) for _ in range(self.n_lanes)]
            self.paf = [torch.zeros((max_batch, 2 * L, h, w), dtype=dtype, device=device) for _ in range(self.n_lanes)]
            self.buf = [Buffers(max_batch, K, L, h, w, cap, ccap, pcap, device) for _ in range(self.n_lanes)]
            torch.cuda.synchronize()
        self.c = (_Lane * self.n_lanes)()
        for l in range(self.n_lanes):
            b = self.buf[l]
            self.c[l] = _Lane(self.cm[l].data_ptr(), self.paf[l].data_ptr(), b.peaks, b.cands, b.conns, b.poses,
                              b.workspace.data_ptr(), b.ws_bytes, b.status.data_ptr(), self.streams[l].cuda_stream)

    def slot_of(self, cm_ptr):
        """(lane, index) of the frame place whose CM pointer hp_batcher_acquire returned."""
        for l, t in enumerate(self.cm):
            off = cm_ptr - t.data_ptr()
            if 0 <= off < t.numel() * t.element_size():
                return l, off // (t[0].numel() * t.element_size())
        raise ValueError("pointer outside the staging tensors")


def hp_batcher_create(skel, prm, lanes, depth):
    """Returns the batcher handle; `lanes` (a BatcherLanes) must outlive it."""
    cfg = _BatcherConfig(lanes.max_batch, int(depth), lanes.n_lanes)
    out = c_void_p()
    dt = HP_F32 if lanes.dtype == torch.float32 else HP_F16
    _check(lib().hp_batcher_create(dt, lanes.h, lanes.w, ctypes.byref(skel.c), ctypes.byref(prm.c), ctypes.byref(cfg),
                                   lanes.c, ctypes.byref(out)), "hp_batcher_create")
    return out


def hp_batcher_destroy(b):
    _check(lib().hp_batcher_destroy(b), "hp_batcher_destroy")


def hp_batcher_acquire(b, timeout_ms=0):
    """(cm pointer, paf pointer) of the next frame's place, or None when every lane is taken."""
    cm, paf = c_void_p(), c_void_p()
    rc = lib().hp_batcher_acquire(b, int(timeout_ms), ctypes.byref(cm), ctypes.byref(paf))
    if rc == HP_ERR_BUSY:
        return None
    _check(rc, "hp_batcher_acquire")
    return cm.value, paf.value


def hp_batcher_commit(b, tag, producer_stream=None, ready=False):
    st = c_void_p(producer_stream.cuda_stream) if producer_stream is not None else _stream()
    _check(lib().hp_batcher_commit(b, int(tag), st, 1 if ready else 0), "hp_batcher_commit")


def hp_batcher_submit(b, cm_frame, paf_frame, tag, timeout_ms=0, producer_stream=None, ready=False):
    """False when every lane is taken (nothing submitted)."""
    st = c_void_p(producer_stream.cuda_stream) if producer_stream is not None else _stream()
    rc = lib().hp_batcher_submit(b, int(timeout_ms), _dev(cm_frame), _dev(paf_frame), int(tag), st, 1 if ready else 0)
    if rc == HP_ERR_BUSY:
        return False
    _check(rc, "hp_batcher_submit")
    return True


def hp_batcher_flush(b):
    _check(lib().hp_batcher_flush(b), "hp_batcher_flush")


def hp_batcher_next(b, max_batch, timeout_ms=-1):
    """Oldest finished batch as a dict (lane, n_frames, seq, start_ns, done_ns, tags, commit_ns), None on time-out."""
    info = _BatchInfo()
    tags = (c_uint64 * max_batch)()
    cns = (c_int64 * max_batch)()
    rc = lib().hp_batcher_next(b, int(timeout_ms), ctypes.byref(info), tags, cns)
    if rc == HP_ERR_TIMEOUT:
        return None
    _check(rc, "hp_batcher_next")
    _check(info.rc, "hp_postprocess (batch %d)" % info.seq)
    n = info.n_frames
    return dict(lane=info.lane, n_frames=n, seq=info.seq, start_ns=info.start_ns, done_ns=info.done_ns,
                tags=[int(tags[k]) for k in range(n)], commit_ns=[int(cns[k]) for k in range(n)])


def hp_batcher_release(b, lane):
    _check(lib().hp_batcher_release(b, int(lane)), "hp_batcher_release")


def hp_batch_simulate(arrival_ns, max_batch, depth, n_lanes, service_base_ns, service_per_frame_ns):
    """Virtual-time run of the batch-slot decisions: (batch_seq, batch_size, done_ns) per frame."""
    arr = np.ascontiguousarray(arrival_ns, np.int64)
    n = len(arr)
    seq, size, done = np.zeros(n, np.int64), np.zeros(n, np.int32), np.zeros(n, np.int64)
    cfg = _BatcherConfig(int(max_batch), int(depth), int(n_lanes))
    _check(lib().hp_batch_simulate(n, arr.ctypes.data_as(POINTER(c_int64)), ctypes.byref(cfg),
                                   int(service_base_ns), int(service_per_frame_ns),
                                   seq.ctypes.data_as(POINTER(c_int64)), size.ctypes.data_as(POINTER(c_int32)),
                                   done.ctypes.data_as(POINTER(c_int64))), "hp_batch_simulate")
    return seq, size, done


def hp_batcher_drive(b, n_frames, interarrival_ns, cm_src=None, paf_src=None):
    """Load generator: (latency_ns, batch_size, elapsed_ns); frames are copied from cm_src / paf_src when given."""
    lat, size = np.zeros(n_frames, np.int64), np.zeros(n_frames, np.int32)
    el = c_int64()
    copy = cm_src is not None
    _check(lib().hp_batcher_drive(b, int(n_frames), int(interarrival_ns), 1 if copy else 0,
                                  _dev(cm_src) if copy else None, _dev(paf_src) if copy else None,
                                  int(cm_src.shape[0]) if copy else 0,
                                  lat.ctypes.data_as(POINTER(c_int64)), size.ctypes.data_as(POINTER(c_int32)),
                                  ctypes.byref(el)), "hp_batcher_drive")
    return lat, size, int(el.value)
