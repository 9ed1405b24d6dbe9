"""Seeded synthetic network outputs of the composite-field family (inputs to both implementations).

The paper names PifPaf (Section 2.3) and gives neither the tensors nor a part table.  The layout here follows the
cited method's description: an Fh x Fw grid of cells `stride` pixels apart; per part and cell an intensity field
(confidence, vector to the part in cell units, a spread unused by decoding, a scale in cell units); per limb and cell
an association field (confidence and, for each of the limb's two parts, a vector and a spread, in cell units).
The part table is the 17 body keypoints of the public COCO person format with its 19 connections, listed here in
this build's own order (the table has cycles on purpose: shoulders-hips, ears-shoulders).

Persons are planted from a standing template: cells within a part's scale of it get a confidence that falls with
distance and a vector that points to the part (jittered); cells near either end of a limb get association vectors
to both ends.  Weak clutter is added everywhere, some of it above the field thresholds.
"""
from dataclasses import dataclass

import numpy as np

from .skeletons import Skeleton, COCO18

_P17 = ("nose", "l_eye", "r_eye", "l_ear", "r_ear", "l_shoulder", "r_shoulder", "l_elbow", "r_elbow", "l_wrist",
        "r_wrist", "l_hip", "r_hip", "l_knee", "r_knee", "l_ankle", "r_ankle")
_T17 = tuple(COCO18.template[COCO18.part_names.index(p)] for p in _P17)
_L17 = (
    (15, 13), (13, 11), (16, 14), (14, 12), (11, 12), (5, 11), (6, 12), (5, 6), (5, 7), (6, 8), (7, 9), (8, 10),
    (1, 2), (0, 1), (0, 2), (1, 3), (2, 4), (3, 5), (4, 6),
)
CF_COCO17 = Skeleton("coco17_fields", _P17, _L17, _T17)


@dataclass(frozen=True)
class CFConfig:
    index: int
    skeleton: Skeleton
    batch: int
    Fh: int
    Fw: int
    n_people: int
    stride: int = 8
    scale_lo: float = 110.0     # person height in pixels
    scale_hi: float = 260.0
    dropout: float = 0.0        # chance that a part of a planted person is missing from the fields
    clutter: int = 40           # cells per image given a confidence above the thresholds at random
    pif_thr: float = 0.1
    paf_thr: float = 0.1
    seed_thr: float = 0.2
    grow_thr: float = 0.05
    rev_tol: float = 8.0
    min_parts: int = 3


CF_CONFIGS = [
    CFConfig(200, CF_COCO17, 1, 16, 20, 2, scale_lo=70.0, scale_hi=100.0, clutter=6),
    CFConfig(201, CF_COCO17, 4, 23, 41, 4, scale_lo=80.0, scale_hi=150.0, dropout=0.1, clutter=20),
    CFConfig(202, CF_COCO17, 8, 46, 82, 10, dropout=0.1),
]


def generate_cf(cfg):
    """-> dict(pif [N, K, 5, Fh, Fw], paf [N, L, 7, Fh, Fw], planted=[n][person] -> xy [K, 2] in pixels (nan = missing))."""
    rng = np.random.default_rng(9000 + cfg.index)
    sk = cfg.skeleton
    N, K, L, Fh, Fw, s = cfg.batch, sk.n_parts, sk.n_limbs, cfg.Fh, cfg.Fw, cfg.stride
    H, W = Fh * s, Fw * s
    pif = np.empty((N, K, 5, Fh, Fw), np.float32)
    pif[:, :, 0] = rng.uniform(0, 0.06, (N, K, Fh, Fw))
    pif[:, :, 1:3] = rng.normal(0, 1.0, (N, K, 2, Fh, Fw))
    pif[:, :, 3] = rng.uniform(0.2, 1.0, (N, K, Fh, Fw))
    pif[:, :, 4] = rng.uniform(0.1, 1.5, (N, K, Fh, Fw))
    paf = np.empty((N, L, 7, Fh, Fw), np.float32)
    paf[:, :, 0] = rng.uniform(0, 0.06, (N, L, Fh, Fw))
    paf[:, :, (1, 2, 4, 5)] = rng.normal(0, 1.5, (N, L, 4, Fh, Fw))
    paf[:, :, (3, 6)] = rng.uniform(0.2, 1.0, (N, L, 2, Fh, Fw))
    gy, gx = np.mgrid[0:Fh, 0:Fw]
    planted = []
    for n in range(N):
        persons = []
        for _ in range(cfg.n_people):
            scale = rng.uniform(cfg.scale_lo, cfg.scale_hi)
            cx, cy = rng.uniform(0.12, 0.88) * W, rng.uniform(0.35, 0.65) * H
            xy = sk.template_xy * scale + np.array([cx, cy]) + rng.normal(0, 1.5, (K, 2))
            sigma = np.full(K, 0.035 * scale)
            for k in range(K):
                inside = 1 <= xy[k, 0] <= W - 2 and 1 <= xy[k, 1] <= H - 2
                if not inside or rng.random() < cfg.dropout:
                    xy[k] = np.nan
            for k in range(K):
                if np.isnan(xy[k, 0]):
                    continue
                jx, jy = xy[k] / s                                    # in cell units
                d = np.hypot(gx - jx, gy - jy)
                near = d <= max(1.0, sigma[k] / s * 1.5)
                conf = rng.uniform(0.75, 0.98) * np.exp(-0.5 * (d / max(0.7, sigma[k] / s)) ** 2)
                upd = near & (conf > pif[n, k, 0])
                m = int(upd.sum())
                pif[n, k, 0][upd] = conf[upd]
                pif[n, k, 1][upd] = (jx - gx)[upd] + rng.normal(0, 0.04, m)
                pif[n, k, 2][upd] = (jy - gy)[upd] + rng.normal(0, 0.04, m)
                pif[n, k, 4][upd] = sigma[k] / s * rng.uniform(0.9, 1.1, m)
            for l in range(L):
                a, b = int(sk.limb_a[l]), int(sk.limb_b[l])
                if np.isnan(xy[a, 0]) or np.isnan(xy[b, 0]):
                    continue
                ax, ay = xy[a] / s
                bx, by = xy[b] / s
                d = np.minimum(np.hypot(gx - ax, gy - ay), np.hypot(gx - bx, gy - by))
                near = d <= 1.5
                conf = rng.uniform(0.7, 0.95) * np.exp(-0.5 * (d / 1.2) ** 2)
                upd = near & (conf > paf[n, l, 0])
                m = int(upd.sum())
                paf[n, l, 0][upd] = conf[upd]
                paf[n, l, 1][upd] = (ax - gx)[upd] + rng.normal(0, 0.05, m)
                paf[n, l, 2][upd] = (ay - gy)[upd] + rng.normal(0, 0.05, m)
                paf[n, l, 4][upd] = (bx - gx)[upd] + rng.normal(0, 0.05, m)
                paf[n, l, 5][upd] = (by - gy)[upd] + rng.normal(0, 0.05, m)
                paf[n, l, 3][upd] = rng.uniform(0.3, 0.6, m)
                paf[n, l, 6][upd] = rng.uniform(0.3, 0.6, m)
            persons.append(xy)
        # clutter above the thresholds: isolated cells, weak enough not to seed a recorded person of their own
        for _ in range(cfg.clutter):
            k, y, x = int(rng.integers(K)), int(rng.integers(Fh)), int(rng.integers(Fw))
            if pif[n, k, 0, y, x] < 0.1:
                pif[n, k, 0, y, x] = rng.uniform(0.1, 0.3)
            l = int(rng.integers(L))
            if paf[n, l, 0, y, x] < 0.1:
                paf[n, l, 0, y, x] = rng.uniform(0.1, 0.25)
        planted.append(persons)
    return dict(pif=pif, paf=paf, planted=planted)
