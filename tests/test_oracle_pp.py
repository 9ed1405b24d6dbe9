"""Pins of the pose-proposal oracle (oracle/hp_pp_oracle.c): IoU in closed form, suppression against an independently
written greedy NMS and its defining properties, exact recovery of planted persons, hand-built parsing cases."""
import numpy as np
import pytest

import oracle
from synth import PPConfig, PP_CONFIGS, PP_COCO19, generate_pp


def test_iou_closed_forms():
    assert oracle.pp_iou([0, 0, 2, 2], [0, 0, 2, 2]) == 1.0
    assert oracle.pp_iou([0, 0, 2, 2], [2, 0, 4, 2]) == 0.0                 # touching edges do not overlap
    assert oracle.pp_iou([0, 0, 2, 2], [5, 5, 6, 6]) == 0.0
    assert oracle.pp_iou([0, 0, 2, 2], [1, 0, 3, 2]) == np.float32(2.0) / np.float32(6.0)   # half overlap: 2 / (4 + 4 - 2)
    assert oracle.pp_iou([0, 0, 4, 4], [1, 1, 3, 3]) == 0.25                # contained: 4 / 16
    assert oracle.pp_iou([0, 0, 0, 0], [0, 0, 0, 0]) == 0.0                 # empty boxes: no division by zero
    a, b = [0.5, 1.5, 3.25, 4.0], [1.0, 0.25, 5.0, 2.0]
    assert oracle.pp_iou(a, b) == oracle.pp_iou(b, a)


def greedy_nms(scores, boxes, thr):
    """Textbook greedy suppression in float64 on the already decoded boxes."""
    order = sorted(range(len(scores)), key=lambda i: (-scores[i], i))
    kept = []
    for i in order:
        ok = True
        for k in kept:
            a, b = boxes[k], boxes[i]
            iw, ih = min(a[2], b[2]) - max(a[0], b[0]), min(a[3], b[3]) - max(a[1], b[1])
            inter = iw * ih if iw > 0 and ih > 0 else 0.0
            den = (a[2] - a[0]) * (a[3] - a[1]) + (b[2] - b[0]) * (b[3] - b[1]) - inter
            if den > 0 and inter / den > thr + 1e-6:
                ok = False
                break
            assert not (den > 0 and abs(inter / den - thr) <= 1e-6)      # no borderline case in these inputs
        if ok:
            kept.append(i)
    return kept


@pytest.mark.parametrize("seed", range(12))
def test_detection_against_a_textbook_nms(seed):
    rng = np.random.default_rng(seed)
    Gh, Gw = int(rng.integers(3, 14)), int(rng.integers(3, 14))
    img_w, img_h = 320.0, 200.0
    resp = rng.random((Gh, Gw)).astype(np.float32)
    conf = rng.random((Gh, Gw)).astype(np.float32)
    box = np.stack([rng.random((Gh, Gw)), rng.random((Gh, Gw)), rng.uniform(0.05, 0.5, (Gh, Gw)),
                    rng.uniform(0.05, 0.5, (Gh, Gw))]).astype(np.float32)
    det_thr, nms_thr = 0.2, float(rng.choice([0.1, 0.3, 0.6]))
    cell, score, corners = oracle.pp_detect(resp, conf, box, img_w, img_h, det_thr, nms_thr)
    # the same candidates, decoded here in float64
    cw, ch = img_w / Gw, img_h / Gh
    s64 = resp.astype(np.float64) * conf.astype(np.float64)
    cand = [c for c in range(Gh * Gw) if np.float32(resp.ravel()[c] * conf.ravel()[c]) > np.float32(det_thr)]
    boxes = {}
    for c in cand:
        gy, gx = divmod(c, Gw)
        cx, cy = (gx + float(box[0, gy, gx])) * cw, (gy + float(box[1, gy, gx])) * ch
        w, h = float(box[2, gy, gx]) * img_w, float(box[3, gy, gx]) * img_h
        boxes[c] = (cx - w / 2, cy - h / 2, cx + w / 2, cy + h / 2)
    scores = [float(np.float32(resp.ravel()[c] * conf.ravel()[c])) for c in cand]
    kept = greedy_nms(scores, [boxes[c] for c in cand], nms_thr)
    assert cell.tolist() == [cand[i] for i in kept]
    assert np.allclose(score, [scores[i] for i in kept], rtol=1e-6)
    assert np.allclose(corners, [boxes[cand[i]] for i in kept], rtol=1e-5, atol=1e-4)
    # defining properties: kept boxes do not overlap beyond the threshold, scores descend
    for i in range(len(cell)):
        for j in range(i):
            assert oracle.pp_iou(corners[i], corners[j]) <= nms_thr
    assert np.all(np.diff(score) <= 0)


def test_planted_persons_come_back():
    for cfg in (PP_CONFIGS[0], PPConfig(110, PP_COCO19, 2, 24, 24, 3, img_h=768.0, img_w=768.0, scale_lo=150.0, scale_hi=200.0)):
        d = generate_pp(cfg)
        sk = cfg.skeleton
        out = oracle.pp_decode(d["resp"], d["conf"], d["box"], d["edge"], sk.limb_a, sk.limb_b, cfg.img_w, cfg.img_h,
                               cfg.det_thr, cfg.nms_thr, cfg.edge_thr, cfg.min_parts)
        for n in range(cfg.batch):
            slots, nparts, score = out["poses"][n]
            found = set()
            for p in range(len(slots)):
                found.add(tuple(int(out["dets"][n][k][0][slots[p, k]]) if slots[p, k] >= 0 else -1
                                for k in range(sk.n_parts)))
            # a planted person is recovered cell for cell as far as its limbs stay inside the neighbourhood
            rh = (cfg.Nh - 1) // 2
            rooted = [cells for cells in d["planted"][n] if cells[sk.limb_a[0]] >= 0]
            for cells in rooted:
                want = np.full(sk.n_parts, -1, np.int64)
                want[sk.limb_a[0]] = cells[sk.limb_a[0]]
                for a, b in zip(sk.limb_a, sk.limb_b):
                    near = want[a] >= 0 and cells[b] >= 0 and abs(cells[b] // cfg.Gw - want[a] // cfg.Gw) <= rh
                    if near and abs(cells[b] % cfg.Gw - want[a] % cfg.Gw) <= rh:
                        want[b] = cells[b]
                assert tuple(int(v) for v in want) in found
            assert len(slots) == len(rooted) > 0
            assert np.all(nparts >= cfg.min_parts) and np.all(score > 0)


def tiny(K=3, Gh=4, Gw=4, Nh=3, Nw=3):
    resp = np.zeros((1, K, Gh, Gw), np.float32)
    conf = np.ones((1, K, Gh, Gw), np.float32)
    box = np.zeros((1, K, 4, Gh, Gw), np.float32)
    box[:, :, 0:2] = 0.5
    box[:, :, 2:4] = 0.1
    edge = np.zeros((1, K - 1, Nh, Nw, Gh, Gw), np.float32)
    return resp, conf, box, edge


def decode(resp, conf, box, edge, limbs, **kw):
    la, lb = [a for a, _ in limbs], [b for _, b in limbs]
    prm = dict(img_w=64.0, img_h=64.0, det_thr=0.5, nms_thr=0.5, edge_thr=0.25, min_parts=1)
    prm.update(kw)
    out = oracle.pp_decode(resp, conf, box, edge, la, lb, prm["img_w"], prm["img_h"], prm["det_thr"], prm["nms_thr"],
                           prm["edge_thr"], prm["min_parts"])
    return out["dets"][0], out["poses"][0]


def test_parsing_rules_by_hand():
    limbs = ((0, 1), (1, 2))
    resp, conf, box, edge = tiny()
    # two roots (part 0) at cells (1,1) and (1,2); one part-1 detection at (2,1); one part-2 detection at (3,1)
    resp[0, 0, 1, 1], resp[0, 0, 1, 2] = 0.9, 0.8
    resp[0, 1, 2, 1] = 0.7
    resp[0, 2, 3, 1] = 0.6
    # both roots point at the part-1 cell: offsets (+1, 0) from (1,1) and (+1, -1) from (1,2)
    edge[0, 0, 2, 1, 1, 1] = 0.5
    edge[0, 0, 2, 0, 1, 2] = 0.75
    edge[0, 1, 2, 1, 2, 1] = 0.5                       # part 1 at (2,1) -> part 2 at (3,1)
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs)
    assert [d[0].tolist() for d in dets] == [[5, 6], [9], [13]]
    # the stronger root comes first and takes the detection although the second root's connection value is larger
    assert slots.tolist() == [[0, 0, 0], [1, -1, -1]] and nparts.tolist() == [3, 1]
    want = np.float32(0.9)
    for v in (0.5, 0.7, 0.5, 0.6):
        want = np.float32(want + np.float32(v))
    assert score[0] == want and score[1] == np.float32(0.8)
    # min_parts drops the second person but it had taken nothing anyway
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs, min_parts=2)
    assert slots.tolist() == [[0, 0, 0]]
    # a connection value equal to the threshold is not enough
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs, edge_thr=0.5)
    assert slots.tolist() == [[0, -1, -1], [1, 0, -1]]          # only the second root's 0.75 passes; limb 2's 0.5 does not
    # a child outside the neighbourhood is never attached: move part 2 two rows away from part 1
    resp[0, 2, 3, 1] = 0.0
    resp[0, 2, 0, 1] = 0.6
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs)
    assert slots.tolist() == [[0, 0, -1], [1, -1, -1]]
    # a detection with a score equal to the threshold is no candidate
    resp[0, 1, 2, 1] = 0.5
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs)
    assert len(dets[1][0]) == 0 and slots.tolist() == [[0, -1, -1], [1, -1, -1]]


def test_detections_taken_by_a_dropped_person_stay_taken():
    limbs = ((0, 1),)
    resp, conf, box, edge = tiny(K=2)
    resp[0, 0, 1, 1], resp[0, 0, 1, 2] = 0.9, 0.8
    resp[0, 1, 2, 1] = 0.7
    edge[0, 0, 2, 1, 1, 1] = 0.5
    edge[0, 0, 2, 0, 1, 2] = 0.75
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs, min_parts=3)
    assert len(slots) == 0
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs, min_parts=2)
    assert slots.tolist() == [[0, 0]]


def boxes_1d(xs, w, scores, img_w=64.0):
    """A 1 x n grid (cells 64 / n wide, image 64 x 16) with a box of width w centred at xs[i] in cell i."""
    n = len(xs)
    cw = img_w / n
    resp = np.array([scores], np.float32)
    conf = np.ones((1, n), np.float32)
    box = np.zeros((4, 1, n), np.float32)
    for i, x in enumerate(xs):
        box[:, 0, i] = (x / cw - i, 0.5, w / img_w, 0.5)
    return resp, conf, box


def test_equal_scores_are_taken_in_cell_order():
    resp, conf, box = boxes_1d([24.0, 24.0, 50.0], 8.0, [0.0, 0.0, 0.0])
    resp[0, :2] = 0.75                                  # two identical boxes with equal scores
    cell, score, corners = oracle.pp_detect(resp, conf, box, 64.0, 16.0, 0.5, 0.5)
    assert cell.tolist() == [0]
    resp[0, 2] = 0.75                                   # and a third, apart: listed after the first
    cell, score, corners = oracle.pp_detect(resp, conf, box, 64.0, 16.0, 0.5, 0.5)
    assert cell.tolist() == [0, 2]


def test_an_overlap_equal_to_the_threshold_is_allowed():
    # [0, 4] x [0, 4] and [1, 3] x [1, 3]: IoU = 4 / 16 exactly
    resp = np.array([[0.9, 0.8]], np.float32)
    conf = np.ones((1, 2), np.float32)
    box = np.zeros((4, 1, 2), np.float32)
    box[:, 0, 0] = (0.5, 0.5, 0.5, 1.0)
    box[:, 0, 1] = (-0.5, 0.5, 0.25, 0.5)
    cell, score, corners = oracle.pp_detect(resp, conf, box, 8.0, 4.0, 0.5, 0.25)
    assert corners.tolist() == [[0, 0, 4, 4], [1, 1, 3, 3]] and oracle.pp_iou(corners[0], corners[1]) == 0.25
    cell, _, _ = oracle.pp_detect(resp, conf, box, 8.0, 4.0, 0.5, float(np.nextafter(np.float32(0.25), np.float32(0))))
    assert cell.tolist() == [0]


def test_a_suppressed_box_suppresses_nothing():
    # A (0.9) overlaps B (0.8), B overlaps C (0.7), A and C are apart: B goes, C stays
    resp, conf, box = boxes_1d([10.0, 16.0, 22.0], 10.0, [0.9, 0.8, 0.7])
    cell, _, _ = oracle.pp_detect(resp, conf, box, 64.0, 16.0, 0.5, 0.2)
    assert cell.tolist() == [0, 2]


def test_the_neighbourhood_ends_where_it_says():
    # the child lies one column beyond a 3 x 3 neighbourhood; the value an index running over would find is set high
    limbs = ((0, 1),)
    resp, conf, box, edge = tiny(K=2, Gh=4, Gw=5)
    resp[0, 0, 1, 1] = 0.9
    resp[0, 1, 1, 3] = 0.8                              # dy = 0, dx = +2
    edge[0, 0, :, :, 1, 1] = 0.0
    edge[0, 0, 2, 0, 1, 1] = 0.9                        # offset (+1, -1): the entry right after (0, +1) in memory
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs)
    assert slots.tolist() == [[0, -1]]
    resp[0, 1, 1, 3], resp[0, 1, 1, 2] = 0.0, 0.8       # one column closer: inside, at offset (0, +1)
    edge[0, 0, 1, 2, 1, 1] = 0.6
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs)
    assert slots.tolist() == [[0, 0]]


def test_a_dropped_person_keeps_what_it_took_from_a_person_that_would_have_been_kept():
    limbs = ((0, 1), (0, 2))
    resp, conf, box, edge = tiny(K=3)
    resp[0, 0, 1, 1], resp[0, 0, 1, 2] = 0.9, 0.8       # two roots
    resp[0, 1, 2, 1] = 0.7                              # X, reachable from both
    resp[0, 2, 2, 2] = 0.6                              # Y, reachable from the second root only
    edge[0, 0, 2, 1, 1, 1] = 0.5
    edge[0, 0, 2, 0, 1, 2] = 0.75
    edge[0, 1, 2, 1, 1, 2] = 0.75
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs, min_parts=3)
    assert len(slots) == 0                              # the first root takes X and is dropped; the second is left with Y
    dets, (slots, nparts, score) = decode(resp, conf, box, edge, limbs, min_parts=2)
    assert slots.tolist() == [[0, 0, -1], [1, -1, 0]]
