"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects invalid calls on the host before anything is enqueued."""
import ctypes
import os
import re
from ctypes import POINTER, byref, c_int32, c_void_p

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2108_11826_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2108_11826_amd import build
        build.build()
    return binding.lib()


def declared_functions():
    """Every function declared by the headers under include/ (hp.h: the operator boundary; hp_bench.h: measurement tooling)."""
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        src = open(os.path.join(ROOT, "include", header)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(hp_[a-z_0-9]+)\s*\(", src))
    return sorted(names)


def test_every_declared_symbol_is_exported(L):
    from paper_2108_11826_amd import binding
    names = declared_functions()
    assert {"hp_resize", "hp_find_peaks", "hp_score_limbs", "hp_assemble", "hp_postprocess",
            "hp_workspace_bytes", "hp_strerror"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert set(binding.EXPORTS) == set(names)


def test_the_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2108_11826_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith((".py", ".c")):
                assert "paper_2108_11826_amd" not in open(os.path.join(dirpath, f)).read(), f


def test_workspace_bytes(L):
    a = L.hp_workspace_bytes(8, 18, 19, 46, 82, 8, 128, 1024, 128)
    b = L.hp_workspace_bytes(8, 18, 19, 46, 82, 8, 256, 1024, 128)
    c = L.hp_workspace_bytes(16, 18, 19, 46, 82, 8, 128, 1024, 128)
    assert 0 < a < b and a < c and a % 256 == 0
    assert L.hp_workspace_bytes(8, 18, 19, 46, 82, 4, 128, 1024, 128) == 0      # scale
    assert L.hp_workspace_bytes(0, 18, 19, 46, 82, 8, 128, 1024, 128) == 0
    assert L.hp_workspace_bytes(8, 18, 19, 46, 82, 8, 1 << 20, 1024, 128) == 0  # beyond HP_MAX_CAP
    assert L.hp_workspace_bytes(8, 99, 19, 46, 82, 8, 128, 1024, 128) == 0      # beyond HP_MAX_PARTS


def test_strerror_and_names(L):
    assert L.hp_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert L.hp_strerror(code) not in (b"ok", b"unknown error")
    assert L.hp_strerror(-99) == b"unknown error"
    assert L.hp_version() >= 100
    assert L.hp_kernel_name(1) == b"resize_nms" and L.hp_kernel_name(99) == b"unknown"


FAKE = 0x10000   # a 256-aligned non-null address that is never dereferenced: these calls fail on the host


def descriptors(cap=64, ccap=64, pcap=16):
    from paper_2108_11826_amd import binding as B
    la = np.array([0, 1], np.int32)
    lb = np.array([1, 2], np.int32)
    sk = B.Skeleton(3, la, lb)
    prm = B.Params()
    pk = B._Peaks(FAKE, FAKE, FAKE, FAKE, cap)
    cd = B._Pairs(FAKE, FAKE, FAKE, FAKE, ccap)
    cn = B._Pairs(FAKE, FAKE, FAKE, FAKE, cap)
    ps = B._Poses(FAKE, FAKE, FAKE, FAKE, pcap)
    return sk, prm, pk, cd, cn, ps


def test_resize_rejects_bad_calls(L):
    assert L.hp_resize(None, 0, 1, 1, 4, 4, 8, FAKE, None) == -1
    assert L.hp_resize(FAKE, 0, 1, 1, 4, 4, 8, None, None) == -1
    assert L.hp_resize(FAKE, 7, 1, 1, 4, 4, 8, FAKE, None) == -2
    assert L.hp_resize(FAKE, 0, 1, 1, 4, 4, 4, FAKE, None) == -5
    assert L.hp_resize(FAKE, 0, 0, 1, 4, 4, 8, FAKE, None) == -1
    assert L.hp_resize(FAKE, 0, 1, 1, 4, 4, 8, FAKE + 4, None) == -1               # dst not 16-byte aligned
    assert L.hp_resize(FAKE, 0, 4096, 4096, 64, 64, 8, FAKE, None) == -5           # index space too large


def test_postprocess_rejects_bad_calls(L):
    sk, prm, pk, cd, cn, ps = descriptors()
    ws = L.hp_workspace_bytes(1, 3, 2, 4, 4, 8, 64, 64, 16)
    args = lambda **kw: [kw.get("cm", FAKE), FAKE, kw.get("dt", 0), 1, 4, 4, byref(kw.get("sk", sk).c),
                         byref(kw.get("prm", prm).c), kw.get("cm_hi", None), kw.get("paf_hi", None),
                         byref(kw.get("pk", pk)), byref(cd), byref(kw.get("cn", cn)), byref(ps),
                         kw.get("wsp", FAKE), kw.get("wsb", ws), kw.get("status", FAKE), None]
    assert L.hp_postprocess(*args(cm=None)) == -1
    assert L.hp_postprocess(*args(status=None)) == -1
    assert L.hp_postprocess(*args(dt=3)) == -2
    assert L.hp_postprocess(*args(cm_hi=FAKE)) == -1                # only one of the two optional outputs
    assert L.hp_postprocess(*args(wsb=ws - 1)) == -3
    assert L.hp_postprocess(*args(wsp=FAKE + 8)) == -3              # misaligned
    assert L.hp_postprocess(*args(wsp=None)) == -3
    from paper_2108_11826_amd import binding as B
    assert L.hp_postprocess(*args(prm=B.Params(scale=4))) == -5
    assert L.hp_postprocess(*args(prm=B.Params(n_samples=1))) == -1
    assert L.hp_postprocess(*args(prm=B.Params(min_valid_ratio=1.5))) == -1
    bad = B.Skeleton(3, np.array([0, 3], np.int32), np.array([1, 2], np.int32))     # part index out of range
    assert L.hp_postprocess(*args(sk=bad)) == -1
    small = B._Pairs(FAKE, FAKE, FAKE, FAKE, 8)                                     # conns cap < peaks cap
    assert L.hp_postprocess(*args(cn=small)) == -1
    huge = B._Peaks(FAKE, FAKE, FAKE, FAKE, 1 << 20)
    assert L.hp_postprocess(*args(pk=huge)) == -5
    # a one-row map 2^21 nodes wide: few enough elements, but hi-res row offsets would not fit the kernels' 24-bit products
    wide = args()
    wide[4], wide[5] = 1, 1 << 21
    wide[15] = 1 << 40
    assert L.hp_postprocess(*wide) == -5


def test_postprocess_static_rejects_on_the_host(L):
    """The entry point that allocates nothing: what hp_postprocess rejects it rejects, and sizes whose
    workspace does not fit its fixed array are refused before any GPU call is made."""
    from paper_2108_11826_amd import binding as B
    sk, prm, pk, cd, cn, ps = descriptors()
    args = lambda **kw: [kw.get("cm", FAKE), FAKE, kw.get("dt", 0), kw.get("N", 1), 4, 4, byref(sk.c),
                         byref(kw.get("prm", prm).c), kw.get("cm_hi", None), None,
                         byref(kw.get("pk", pk)), byref(kw.get("cd", cd)), byref(kw.get("cn", cn)), byref(ps),
                         kw.get("status", FAKE), None]
    assert L.hp_postprocess_static(*args(cm=None)) == -1
    assert L.hp_postprocess_static(*args(status=None)) == -1
    assert L.hp_postprocess_static(*args(dt=3)) == -2
    assert L.hp_postprocess_static(*args(cm_hi=FAKE)) == -1
    assert L.hp_postprocess_static(*args(prm=B.Params(scale=4))) == -5
    assert L.hp_postprocess_static(*args(pk=B._Peaks(FAKE, FAKE, FAKE, FAKE, 1 << 20))) == -5
    # 64 images x 2 limbs x 2^16 candidates of staging alone is 64 MiB: beyond the 8 MiB array
    big = B._Pairs(FAKE, FAKE, FAKE, FAKE, 1 << 16)
    assert L.hp_workspace_bytes(64, 3, 2, 4, 4, 8, 64, 1 << 16, 16) > 8 << 20
    assert L.hp_postprocess_static(*args(N=64, cd=big)) == -3
    src = open(os.path.join(ROOT, "include", "hp.h")).read()
    assert re.search(r"HP_STATIC_WS_BYTES\s*=\s*8\s*<<\s*20", src)


def test_staged_calls_reject_bad_calls(L):
    sk, prm, pk, cd, cn, ps = descriptors()
    ws = L.hp_workspace_bytes(1, 3, 2, 4, 4, 8, 64, 64, 16)
    assert L.hp_find_peaks(None, 1, 4, 3, 32, 32, 0.05, byref(pk), FAKE, ws, FAKE, None) == -1
    assert L.hp_find_peaks(FAKE, 1, 2, 3, 32, 32, 0.05, byref(pk), FAKE, ws, FAKE, None) == -1     # C_cm < K
    assert L.hp_find_peaks(FAKE, 1, 4, 3, 32, 32, 0.05, byref(pk), FAKE, 8, FAKE, None) == -3
    assert L.hp_find_peaks(FAKE, 1, 4, 3, 32, 32, float("nan"), byref(pk), FAKE, ws, FAKE, None) == -1
    assert L.hp_score_limbs(FAKE, 1, 33, 32, byref(sk.c), byref(prm.c), byref(pk), byref(cd), FAKE, ws, FAKE, None) == -1
    assert L.hp_score_limbs(FAKE, 1, 32, 32, byref(sk.c), byref(prm.c), byref(pk), byref(cd), FAKE, 16, FAKE, None) == -3
    assert L.hp_assemble(byref(sk.c), byref(prm.c), 0, byref(pk), byref(cd), byref(cn), byref(ps), FAKE, ws, FAKE, None) == -1
    assert L.hp_assemble(byref(sk.c), byref(prm.c), 1, byref(pk), byref(cd), byref(cn), byref(ps), FAKE, 16, FAKE, None) == -3
    assert L.hp_profile_begin(0) == -1
    assert L.hp_workspace_init(None, 1024, None) == -3
    assert L.hp_workspace_init(FAKE + 4, 1024, None) == -3
    assert L.hp_workspace_init(FAKE, 1022, None) == -3


def test_binding_fails_loudly_without_the_library(monkeypatch):
    from paper_2108_11826_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "lib_path", lambda: "/nonexistent/libhp.so")
    with pytest.raises(ImportError):
        binding.lib()


def test_preprocess_rejects_bad_calls(L):
    from ctypes import c_float
    fake = c_void_p(0x1000)                        # never dereferenced: every call below fails on the host
    al, be = (c_float * 4)(1, 1, 1, 1), (c_float * 4)(0, 0, 0, 0)
    ok = (fake, 1, 8, 8, 3, 0, fake, 8, 8, 0, al, be, None)

    def call(**kw):
        names = ("src", "N", "Hs", "Ws", "C", "dt", "dst", "Hd", "Wd", "rev", "alpha", "beta", "stream")
        a = dict(zip(names, ok))
        a.update(kw)
        return L.hp_preprocess(*[a[k] for k in names])

    assert call(src=None) == -1 and call(dst=None) == -1 and call(alpha=None) == -1 and call(beta=None) == -1
    assert call(N=0) == -1 and call(Hs=0) == -1 and call(Wd=-3) == -1 and call(C=0) == -1
    assert call(dt=7) == -2
    assert call(C=5) == -5 and call(Ws=20000) == -5 and call(Hd=16385) == -5 and call(N=70000) == -5
    assert call(dst=c_void_p(0x1002)) == -1        # fp32 output must be 4-byte aligned
    assert call(C=4, src=c_void_p(0x1001)) == -1   # four-channel pixels are read as aligned words


def test_batcher_rejects_bad_calls(L):
    from paper_2108_11826_amd import binding as B
    sk, prm, pk, cd, cn, ps = descriptors()
    ws = L.hp_workspace_bytes(4, 3, 2, 4, 4, 8, 64, 64, 16)

    def lanes(n, shared=False, wsp=FAKE, wsb=ws):
        arr = (B._Lane * n)()
        for l in range(n):
            base = FAKE if shared else FAKE * (l + 1)
            arr[l] = B._Lane(base, base, pk, cd, cn, ps, wsp + (0 if shared else l * 0x100000), wsb, base, None)
        return arr

    def create(cfg=(4, 1, 2), dt=0, h=4, w=4, skel=sk, params=prm, ln=None, out=True):
        c = B._BatcherConfig(*cfg)
        handle = c_void_p()
        rc = L.hp_batcher_create(dt, h, w, byref(skel.c) if skel else None, byref(params.c) if params else None,
                                 byref(c), ln if ln is not None else lanes(cfg[2]), byref(handle) if out else None)
        assert handle.value is None           # no batcher comes out of a failed call
        return rc

    assert create(out=False) == -1
    assert create(skel=None) == -1 and create(params=None) == -1
    assert create(dt=5) == -2
    assert create(cfg=(0, 1, 2)) == -1 and create(cfg=(4, 0, 2)) == -1 and create(cfg=(4, 3, 2)) == -1
    assert create(cfg=(4, 1, 65)) == -5 and create(cfg=(2048, 1, 2)) == -5
    assert create(h=0) == -1
    assert create(ln=lanes(2, shared=True)) == -1                  # lanes must not share buffers
    assert create(ln=lanes(2, wsb=ws - 256)) == -3                 # workspace sized for fewer frames than max_batch
    assert create(ln=lanes(2, wsp=FAKE + 8)) == -3
    assert create(params=B.Params(scale=4)) == -5
    assert create(params=B.Params(n_samples=1)) == -1
    # the other entry points refuse a null handle
    assert L.hp_batcher_destroy(None) == -1 and L.hp_batcher_flush(None) == -1
    assert L.hp_batcher_release(None, 0) == -1 and L.hp_batcher_commit(None, 0, None, 1) == -1
    assert L.hp_batcher_next(None, 0, None, None, None) == -1
    assert L.hp_batcher_drive(None, 1, 0, 0, None, None, 0, None, None, None) == -1
    assert L.hp_strerror(-6) != L.hp_strerror(-7) != L.hp_strerror(-8) != b"unknown error"


def test_draw_rejects_bad_calls(L):
    from ctypes import c_uint8
    sk, prm, pk, cd, cn, ps = descriptors()
    rgb = (c_uint8 * 96)()
    a, b = c_void_p(0x100000), c_void_p(0x900000)
    L.hp_draw_workspace_bytes.restype = ctypes.c_size_t
    need = L.hp_draw_workspace_bytes(1, 3, 2, 16, 8, 8)
    assert need > 0 and need % 16 == 0 and L.hp_draw_workspace_bytes(2, 3, 2, 16, 8, 8) > need
    assert L.hp_draw_workspace_bytes(1, 3, 2, 16, 4096, 4096) > need
    assert L.hp_draw_workspace_bytes(0, 3, 2, 16, 8, 8) == 0 and L.hp_draw_workspace_bytes(1, 99, 2, 16, 8, 8) == 0
    assert L.hp_draw_workspace_bytes(1, 3, 2, 16, 0, 8) == 0 and L.hp_draw_workspace_bytes(1, 3, 2, 16, 8, 20000) == 0
    ok = dict(src=a, dst=b, N=1, Hf=8, Wf=8, C=3, H=8, W=8, skel=byref(sk.c), pk=byref(pk), ps=byref(ps), lrgb=rgb,
              prgb=rgb, t=2, r=2, ws=c_void_p(FAKE), wsb=ctypes.c_size_t(need), stream=None)

    def call(**kw):
        x = dict(ok)
        x.update(kw)
        return L.hp_draw_poses(*[x[k] for k in ("src", "dst", "N", "Hf", "Wf", "C", "H", "W", "skel", "pk", "ps",
                                                 "lrgb", "prgb", "t", "r", "ws", "wsb", "stream")])

    assert call(src=None) == -1 and call(dst=None) == -1 and call(lrgb=None) == -1 and call(prgb=None) == -1
    assert call(skel=None) == -1 and call(pk=None) == -1 and call(ps=None) == -1
    assert call(N=0) == -1 and call(Hf=0) == -1 and call(W=-1) == -1 and call(t=-1) == -1 and call(r=-2) == -1
    assert call(C=1) == -5 and call(C=5) == -5
    assert call(Wf=20000) == -5 and call(H=16385) == -5 and call(N=70000) == -5 and call(t=2000) == -5
    assert call(dst=c_void_p(0x100000 + 50)) == -1          # overlaps the source without being it
    assert call(ws=None) == -3 and call(ws=c_void_p(FAKE + 16)) == -3 and call(wsb=ctypes.c_size_t(need - 1)) == -3


def test_smooth_rejects_bad_calls(L):
    a, b, t = c_void_p(0x100000), c_void_p(0x9000000), c_void_p(0x2000)
    ok = dict(src=a, dst=b, N=1, C=2, C_mem=3, H=16, W=16, taps=t, n=5, stream=None)

    def call(**kw):
        x = dict(ok)
        x.update(kw)
        return L.hp_smooth(*[x[k] for k in ("src", "dst", "N", "C", "C_mem", "H", "W", "taps", "n", "stream")])

    assert call(src=None) == -1 and call(dst=None) == -1 and call(taps=None) == -1
    assert call(N=0) == -1 and call(C=0) == -1 and call(C_mem=1) == -1 and call(H=0) == -1 and call(W=-4) == -1
    assert call(n=0) == -1 and call(n=4) == -1             # the tap vector has odd length
    assert call(n=67) == -5
    assert call(dst=a) == -1 and call(dst=c_void_p(0x100000 + 64)) == -1      # no smoothing in place


def test_refine_rejects_bad_calls(L):
    sk, prm, pk, cd, cn, ps = descriptors()
    a, x, y = c_void_p(0x100000), c_void_p(0x200000), c_void_p(0x300000)
    assert L.hp_refine_peaks(None, 1, 4, 3, 16, 16, byref(pk), x, y, None) == -1
    assert L.hp_refine_peaks(a, 1, 4, 3, 16, 16, byref(pk), None, y, None) == -1
    assert L.hp_refine_peaks(a, 1, 4, 3, 16, 16, None, x, y, None) == -1
    assert L.hp_refine_peaks(a, 0, 4, 3, 16, 16, byref(pk), x, y, None) == -1
    assert L.hp_refine_peaks(a, 1, 2, 3, 16, 16, byref(pk), x, y, None) == -1       # fewer channels than parts
    assert L.hp_refine_peaks(a, 1, 99, 99, 16, 16, byref(pk), x, y, None) == -5


def test_pp_decode_rejects_bad_calls(L):
    from paper_2108_11826_amd import binding as B
    sk = B.Skeleton(3, np.array([0, 1], np.int32), np.array([1, 2], np.int32))
    prm = B._PPParams(0.3, 0.3, 0.3, 1, 64.0, 64.0)
    dets = B._PPDets(FAKE, FAKE, FAKE, FAKE, 8)
    ps = B._Poses(FAKE, FAKE, FAKE, FAKE, 4)
    a = c_void_p(FAKE)
    ok = dict(resp=a, conf=a, box=a, edge=a, N=1, Gh=4, Gw=4, Nh=3, Nw=3, skel=byref(sk.c), prm=byref(prm), dets=byref(dets),
              poses=byref(ps), status=a, stream=None)

    def call(**kw):
        x = dict(ok)
        x.update(kw)
        return L.hp_pp_decode(*[x[k] for k in ("resp", "conf", "box", "edge", "N", "Gh", "Gw", "Nh", "Nw", "skel", "prm", "dets",
                                                "poses", "status", "stream")])

    assert call(resp=None) == -1 and call(edge=None) == -1 and call(status=None) == -1 and call(prm=None) == -1
    assert call(dets=None) == -1 and call(poses=None) == -1 and call(skel=None) == -1
    assert call(N=0) == -1 and call(Gh=0) == -1 and call(Nh=4) == -1 and call(Nw=0) == -1       # neighbourhoods are odd
    assert call(Gh=40, Gw=40) == -5 and call(Nh=33) == -5
    assert call(dets=byref(B._PPDets(FAKE, FAKE, FAKE, FAKE, 2048))) == -5
    # limbs that do not form a tree walked from the root: a child reached twice, a parent never reached
    twice = B.Skeleton(3, np.array([0, 0, 1], np.int32), np.array([1, 2, 2], np.int32))
    orphan = B.Skeleton(4, np.array([0, 2], np.int32), np.array([1, 3], np.int32))
    assert call(skel=byref(twice.c)) == -1 and call(skel=byref(orphan.c)) == -1
    assert call(prm=byref(B._PPParams(0.3, float("nan"), 0.3, 1, 64.0, 64.0))) == -1
    assert call(prm=byref(B._PPParams(0.3, 0.3, 0.3, 1, 0.0, 64.0))) == -1


def test_cf_decode_rejects_bad_calls(L):
    from paper_2108_11826_amd import binding as B
    sk = B.Skeleton(3, np.array([0, 1, 2], np.int32), np.array([1, 2, 0], np.int32))      # a cycle is a valid table
    prm = B._CFParams(0.1, 0.1, 0.2, 0.05, 4.0, 1, 8)
    lists = B._CFLists(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, 128)
    ps = B._CFPoses(FAKE, FAKE, FAKE, FAKE, 16)
    a = c_void_p(FAKE)
    need = L.hp_cf_workspace_bytes(2, 3, 3, 64, 128)
    assert need >= 2 * 3 * (64 + 128) * 32 and L.hp_cf_workspace_bytes(0, 3, 3, 64, 128) == 0
    ok = dict(pif=a, paf=a, N=2, Fh=10, Fw=12, skel=byref(sk.c), prm=byref(prm), lists=byref(lists), poses=byref(ps), ws=a,
              wsb=ctypes.c_size_t(need), status=a, stream=None)

    def call(**kw):
        x = dict(ok)
        x.update(kw)
        return L.hp_cf_decode(*[x[k] for k in ("pif", "paf", "N", "Fh", "Fw", "skel", "prm", "lists", "poses", "ws", "wsb",
                                                "status", "stream")])

    assert call(pif=None) == -1 and call(paf=None) == -1 and call(status=None) == -1 and call(ws=None) == -1
    assert call(prm=None) == -1 and call(lists=None) == -1 and call(poses=None) == -1 and call(skel=None) == -1
    assert call(N=0) == -1 and call(Fh=0) == -1 and call(Fw=-3) == -1
    assert call(wsb=ctypes.c_size_t(need - 1)) == -3 and call(ws=c_void_p(FAKE + 4)) == -3
    for bad in (B._CFParams(-0.1, 0.1, 0.2, 0.05, 4.0, 1, 8), B._CFParams(0.1, float("nan"), 0.2, 0.05, 4.0, 1, 8),
                B._CFParams(0.1, 0.1, 0.2, -1.0, 4.0, 1, 8), B._CFParams(0.1, 0.1, 0.2, 0.05, 4.0, -1, 8),
                B._CFParams(0.1, 0.1, 0.2, 0.05, 4.0, 1, 0)):
        assert call(prm=byref(bad)) == -1
    assert call(lists=byref(B._CFLists(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, 128))) == -1
    assert call(lists=byref(B._CFLists(FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 64, 128))) == -1
    big = L.hp_cf_workspace_bytes(2, 3, 3, 1025, 128)
    assert call(lists=byref(B._CFLists(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1025, 128)), wsb=ctypes.c_size_t(big)) == -5
    assert call(poses=byref(B._CFPoses(FAKE, FAKE, FAKE, FAKE, 1366))) == -5              # 3 * 1366 > 4096 joints in LDS
    assert call(prm=byref(B._CFParams(0.1, 0.1, 0.2, 0.05, 4.0, 1, 1 << 22))) == -5        # the map would pass 2^23 pixels a side


def test_cf_field_rejects_bad_calls(L):
    from paper_2108_11826_amd import binding as B
    prm = B._CFParams(0.1, 0.0, 0.0, 0.0, 0.0, 0, 8)
    a = c_void_p(FAKE)
    need = L.hp_cf_workspace_bytes(2, 5, 0, 64, 0)
    assert need >= 2 * 5 * 64 * 32
    ok = dict(pif=a, N=2, K=5, Fh=10, Fw=12, prm=byref(prm), cell=a, val=a, count=a, cap=64, out=a, ws=a,
              wsb=ctypes.c_size_t(need), status=a, stream=None)

    def call(**kw):
        x = dict(ok)
        x.update(kw)
        return L.hp_cf_field(*[x[k] for k in ("pif", "N", "K", "Fh", "Fw", "prm", "cell", "val", "count", "cap", "out", "ws",
                                               "wsb", "status", "stream")])

    assert call(pif=None) == -1 and call(out=None) == -1 and call(count=None) == -1 and call(prm=None) == -1
    assert call(N=0) == -1 and call(K=0) == -1 and call(cap=0) == -1 and call(Fh=0) == -1
    assert call(K=33) == -5 and call(cap=1025) == -5
    assert call(wsb=ctypes.c_size_t(need - 1)) == -3
