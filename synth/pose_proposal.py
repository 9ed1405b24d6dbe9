"""Seeded synthetic network outputs of the pose-proposal family (inputs to both implementations).

The paper names PoseProposal (Section 2.3) and gives neither the tensors nor a part table.  The layout here is this
build's own: a Gh x Gw grid over the image; per part k and cell, a responsibility and a confidence map (their product
is the detection score) and a box (centre offset inside the cell, width and height as fractions of the image); per
limb and cell, a connection value towards each cell of an Nh x Nw neighbourhood.  Persons are planted from the
skeleton template: the cell holding a part gets a high score and a tight box, its neighbours lower scores with
heavily overlapping boxes (which the suppression step has to remove), and the limb's connection value is set at the
offset between the two parts' cells.  Noise is added everywhere.
"""
from dataclasses import dataclass

import numpy as np

from .skeletons import Skeleton, COCO18

# the part tree of the pose-proposal workloads: a whole-person "instance" node on top of the 18 parts
PP_COCO19 = Skeleton("coco19_instance", COCO18.part_names + ("instance",), ((18, 1),) + COCO18.limbs[:17],
                     COCO18.template + ((0.0, -0.12),))


@dataclass(frozen=True)
class PPConfig:
    index: int
    skeleton: Skeleton
    batch: int
    Gh: int
    Gw: int
    n_people: int
    Nh: int = 9
    Nw: int = 9
    img_h: float = 384.0
    img_w: float = 384.0
    scale_lo: float = 90.0
    scale_hi: float = 220.0
    noise: float = 0.03
    dropout: float = 0.0
    det_thr: float = 0.3
    nms_thr: float = 0.3
    edge_thr: float = 0.3
    min_parts: int = 3


PP_CONFIGS = [
    PPConfig(100, PP_COCO19, 1, 12, 12, 2),
    PPConfig(101, PP_COCO19, 8, 12, 12, 4, dropout=0.1),
    PPConfig(102, PP_COCO19, 16, 24, 24, 10, img_h=768.0, img_w=768.0, dropout=0.15),
]


def generate_pp(cfg):
    """-> dict(resp, conf [N, K, Gh, Gw], box [N, K, 4, Gh, Gw], edge [N, L, Nh, Nw, Gh, Gw], planted=[n][person][k] cell or -1)."""
    rng = np.random.default_rng(7000 + cfg.index)
    sk = cfg.skeleton
    N, K, L, Gh, Gw = cfg.batch, sk.n_parts, sk.n_limbs, cfg.Gh, cfg.Gw
    resp = rng.uniform(0, cfg.noise * 4, (N, K, Gh, Gw)).astype(np.float32)
    conf = rng.uniform(0.3, 0.9, (N, K, Gh, Gw)).astype(np.float32)
    box = np.empty((N, K, 4, Gh, Gw), np.float32)
    box[:, :, 0:2] = rng.uniform(0, 1, (N, K, 2, Gh, Gw))
    box[:, :, 2:4] = rng.uniform(0.05, 0.2, (N, K, 2, Gh, Gw))
    edge = rng.uniform(0, cfg.noise * 4, (N, L, cfg.Nh, cfg.Nw, Gh, Gw)).astype(np.float32)
    cw, ch = cfg.img_w / Gw, cfg.img_h / Gh
    rh, rw = (cfg.Nh - 1) // 2, (cfg.Nw - 1) // 2
    planted = []
    for n in range(N):
        persons = []
        taken = set()
        for _ in range(cfg.n_people):
            scale = rng.uniform(cfg.scale_lo, cfg.scale_hi)
            cx, cy = rng.uniform(0.15, 0.85) * cfg.img_w, rng.uniform(0.3, 0.7) * cfg.img_h
            xy = sk.template_xy * scale + np.array([cx, cy]) + rng.normal(0, 2.0, (K, 2))
            cells = np.full(K, -1, np.int64)
            for k in range(K):
                if k != sk.limb_a[0] and rng.random() < cfg.dropout:
                    continue
                gx, gy = int(xy[k, 0] // cw), int(xy[k, 1] // ch)
                if not (0 <= gx < Gw and 0 <= gy < Gh) or (k, gy, gx) in taken:
                    continue
                taken.add((k, gy, gx))
                cells[k] = gy * Gw + gx
                size = (0.08 if k != K - 1 else 0.5) * scale
                resp[n, k, gy, gx] = rng.uniform(0.85, 0.99)
                conf[n, k, gy, gx] = rng.uniform(0.85, 0.99)
                box[n, k, :, gy, gx] = (xy[k, 0] / cw - gx, xy[k, 1] / ch - gy, size / cfg.img_w, size / cfg.img_h)
                # a weaker duplicate in a neighbouring cell, its box almost the same: suppression must remove it
                ny, nx = gy + int(rng.integers(-1, 2)), gx + int(rng.integers(-1, 2))
                if 0 <= ny < Gh and 0 <= nx < Gw and (k, ny, nx) not in taken and (ny, nx) != (gy, gx):
                    taken.add((k, ny, nx))
                    resp[n, k, ny, nx] = rng.uniform(0.6, 0.8)
                    conf[n, k, ny, nx] = rng.uniform(0.7, 0.8)
                    box[n, k, :, ny, nx] = (xy[k, 0] / cw - nx + rng.normal(0, 0.01), xy[k, 1] / ch - ny + rng.normal(0, 0.01),
                                            size / cfg.img_w, size / cfg.img_h)
            # the limb's connection value at the offset between its parts' cells (none when the child lies outside the
            # parent's neighbourhood: such a limb cannot be followed)
            for l in range(L):
                a, b = int(sk.limb_a[l]), int(sk.limb_b[l])
                if cells[a] < 0 or cells[b] < 0:
                    continue
                dy, dx = cells[b] // Gw - cells[a] // Gw, cells[b] % Gw - cells[a] % Gw
                if abs(dy) <= rh and abs(dx) <= rw:
                    edge[n, l, dy + rh, dx + rw, cells[a] // Gw, cells[a] % Gw] = rng.uniform(0.8, 0.99)
            persons.append(cells)
        planted.append(persons)
    return dict(resp=resp, conf=conf, box=box, edge=edge, planted=planted)
