"""Pins for the oracle's assembly (reading A) and for the whole chain.

Parity with the paper's own engine is unpinned (the paper prints no rule and no example):
what is pinned is that planted skeletons come back exactly, the structural invariants, and
hand-worked micro cases for each branch of the rule set."""
import numpy as np
import pytest

import oracle
from synth import COCO18, BODY25, SynthConfig, generate, DEFAULT_PARAMS, CONFIGS

E = (np.array([], np.int32), np.array([], np.int32), np.array([], np.float32))


def conn(*triples):
    i, j, s = zip(*triples)
    return np.array(i, np.int32), np.array(j, np.int32), np.array(s, np.float32)


# Tiny skeleton: parts 0,1,2,3; limbs (0,1) (1,2) (2,3) (3,0): the last one closes a cycle.
LA = np.array([0, 1, 2, 3], np.int32)
LB = np.array([1, 2, 3, 0], np.int32)
PS = [np.array([0.5, 0.25], np.float32) for _ in range(4)]       # two peaks per part, scores 0.5 / 0.25


def test_new_extend_and_cycle():
    # limb0 (0->1): peaks 0-0; limb1 (1->2): 0-0; limb2 (2->3): 0-0; limb3 (3->0): 0-0 closes the cycle
    slots, nparts, score = oracle.assemble(LA, LB, 4, PS, [conn((0, 0, 1.0))] * 4, 3)
    assert slots.tolist() == [[0, 0, 0, 0]] and nparts.tolist() == [4]
    # 0.5+0.5+1 (new) +0.5+1 (extend) +0.5+1 (extend) +1 (cycle)
    assert score[0] == np.float32(6.0)


def test_extend_from_b_side_and_min_parts():
    # limb1 first creates {1:0, 2:1}; limb0 has nothing; limb3 (3->0) creates {3:1, 0:1}; each has 2 parts
    slots, nparts, score = oracle.assemble(LA, LB, 4, PS, [E, conn((0, 1, 0.5)), E, conn((1, 1, 0.5))], 2)
    assert slots.tolist() == [[-1, 0, 1, -1], [1, -1, -1, 1]] and nparts.tolist() == [2, 2]
    assert score.tolist() == [0.5 + 0.25 + 0.5, 0.25 + 0.25 + 0.5]
    assert len(oracle.assemble(LA, LB, 4, PS, [E, conn((0, 1, 0.5)), E, conn((1, 1, 0.5))], 3)[0]) == 0
    # B-side owned, A-side free: limb1 creates {1:0,2:0}; limb0 (0->1) with j=0 owned -> fills part 0
    slots, nparts, score = oracle.assemble(LA[:2][::-1].copy(), LB[:2][::-1].copy(), 4, PS,
                                           [conn((0, 0, 1.0)), conn((1, 0, 2.0))], 3)
    assert slots.tolist() == [[1, 0, 0, -1]] and score[0] == np.float32(0.5 + 0.5 + 1.0 + 0.25 + 2.0)


def test_slot_conflict_is_skipped():
    # person {0:0, 1:0}; then limb0's second connection (1, ...) cannot exist twice per peak, so build the
    # conflict through the cycle limb: persons P0 = {0:0,1:0}, then limb (3->0) conn (0, 1) creates P1 = {3:0, 0:1};
    # limb order: (0,1), (3,0), (1,3)?  use a custom table: limbs (0,1) (3,0) (1,3)
    la = np.array([0, 3, 1], np.int32)
    lb = np.array([1, 0, 3], np.int32)
    # (0,1): 0-0 -> P0 {0:0,1:0}.  (3,0): 0-1 -> P1 {3:0,0:1}.  (1,3): 0-0 joins P0 and P1, but both hold part 0 -> skip.
    slots, nparts, score = oracle.assemble(la, lb, 4, PS, [conn((0, 0, 1.0)), conn((0, 1, 1.0)), conn((0, 0, 1.0))], 2)
    assert slots.tolist() == [[0, 0, -1, -1], [1, -1, -1, 0]]
    assert score.tolist() == [2.0, 0.5 + 0.25 + 1.0]
    # (1,3): 0-1 instead: peak 1 of part 3 is free, P0's slot 3 is empty -> extend P0
    slots, nparts, score = oracle.assemble(la, lb, 4, PS, [conn((0, 0, 1.0)), conn((0, 1, 1.0)), conn((0, 1, 1.0))], 2)
    assert slots.tolist() == [[0, 0, -1, 1], [1, -1, -1, 0]]
    # one-side-owned with the other slot already filled: P0 {0:0,1:0}; limb (0,1) again as a 4th limb with conn (0,1):
    la2 = np.array([0, 0], np.int32)
    lb2 = np.array([1, 1], np.int32)
    slots, nparts, score = oracle.assemble(la2, lb2, 4, PS, [conn((0, 0, 1.0)), conn((0, 1, 1.0))], 2)
    assert slots.tolist() == [[0, 0, -1, -1]] and score[0] == np.float32(2.0)


def test_merge_keeps_the_earlier_person():
    # limbs (2,3) first -> P0 {2:0,3:0}; (0,1) -> P1 {0:0,1:0}; (1,2) joins them: merge P1 into P0
    la = np.array([2, 0, 1], np.int32)
    lb = np.array([3, 1, 2], np.int32)
    slots, nparts, score = oracle.assemble(la, lb, 4, PS, [conn((0, 0, 1.0)), conn((1, 1, 1.0)), conn((1, 0, 0.5))], 3)
    assert slots.tolist() == [[1, 1, 0, 0]] and nparts.tolist() == [4]
    assert score[0] == np.float32((0.5 + 0.5 + 1.0) + (0.25 + 0.25 + 1.0) + 0.5)
    # after the merge the moved peaks belong to the survivor: a later cycle limb (3,0) adds only its score
    la = np.array([2, 0, 1, 3], np.int32)
    lb = np.array([3, 1, 2, 0], np.int32)
    slots, nparts, score2 = oracle.assemble(la, lb, 4, PS, [conn((0, 0, 1.0)), conn((1, 1, 1.0)), conn((1, 0, 0.5)),
                                                            conn((0, 1, 0.125))], 3)
    assert slots.tolist() == [[1, 1, 0, 0]] and score2[0] == score[0] + np.float32(0.125)


def test_merge_survivor_keeps_its_creation_rank():
    # limbs (2,3) -> P0 {2:0,3:0}; (0,1) twice -> P1 {0:0,1:0}, P2 {0:1,1:1}; (1,2): peak 1 of part 1 (P2) to
    # peak 0 of part 2 (P0): P2 merges into P0, and the output order is creation order: P0+P2 first, then P1.
    la = np.array([2, 0, 1], np.int32)
    lb = np.array([3, 1, 2], np.int32)
    slots, nparts, score = oracle.assemble(la, lb, 4, PS, [conn((0, 0, 1.0)), conn((0, 0, 1.0), (1, 1, 1.0)),
                                                            conn((1, 0, 0.5))], 2)
    assert slots.tolist() == [[1, 1, 0, 0], [0, 0, -1, -1]] and nparts.tolist() == [4, 2]


def planted_cfg(sk, n_people, h, w):
    return SynthConfig(90, sk, 2, h, w, n_people, scale_lo=170.0, scale_hi=230.0, jitter_sd=2.0,
                       noise_sd=0.0, placement="grid")


@pytest.mark.parametrize("sk,n_people,h,w", [(COCO18, 6, 70, 100), (BODY25, 4, 64, 92)])
def test_planted_skeletons_come_back(sk, n_people, h, w):
    """Noise-free, non-overlapping people: persons <-> planted people is a bijection, every slot is
    filled and every slot's peak lies within the lo-res quantisation (4 px, plus rounding) of its joint."""
    cfg = planted_cfg(sk, n_people, h, w)
    b = generate(cfg)
    r = oracle.postprocess(b.cm, b.paf, sk.limb_a, sk.limb_b, DEFAULT_PARAMS, threads=4)
    for n in range(cfg.batch):
        slots, nparts, score = r["poses"][n]
        truth = b.people[n]
        assert not np.isnan(truth).any()
        assert len(slots) == n_people and np.all(nparts == sk.n_parts)
        used = set()
        for p in range(len(slots)):
            xy = np.array([[r["peaks"][n][c][0][slots[p, c]], r["peaks"][n][c][1][slots[p, c]]]
                           for c in range(sk.n_parts)], np.float64)
            d = np.abs(truth - xy[None]).max(axis=2).max(axis=1)      # worst joint error per planted person
            who = int(np.argmin(d))
            assert d[who] <= 4.6 and who not in used
            used.add(who)


@pytest.mark.parametrize("ci", [0, 1, 2])
def test_invariants_on_noisy_configs(ci):
    cfg = CONFIGS[ci]
    b = generate(cfg, images=range(min(cfg.batch, 2)))
    sk = cfg.skeleton
    r = oracle.postprocess(b.cm, b.paf, sk.limb_a, sk.limb_b, DEFAULT_PARAMS, threads=4)
    r1 = oracle.postprocess(b.cm, b.paf, sk.limb_a, sk.limb_b, DEFAULT_PARAMS, threads=1)
    for n in range(len(b.people)):
        slots, nparts, score = r["poses"][n]
        assert np.array_equal(slots, r1["poses"][n][0]) and np.array_equal(score, r1["poses"][n][2])
        assert np.array_equal(nparts, (slots >= 0).sum(axis=1)) and np.all(nparts >= DEFAULT_PARAMS.min_parts)
        for c in range(sk.n_parts):
            col = slots[:, c][slots[:, c] >= 0]
            assert len(set(col.tolist())) == len(col)                 # a peak has at most one owner
            assert np.all(col < len(r["peaks"][n][c][0]))
        for l, (a, bb) in enumerate(sk.limbs):
            mi, mj, ms = r["conns"][n][l]
            cand = set(zip(*[x.tolist() for x in r["candidates"][n][l][:2]]))
            assert set(zip(mi.tolist(), mj.tolist())) <= cand
        assert len(slots) > 0
