"""Pins for the oracle's greedy matching (reading M: strict order score desc, i asc, j asc)."""
import numpy as np
from hypothesis import given, settings, strategies as st
from scipy.optimize import linear_sum_assignment

import oracle


def brute_greedy(ci, cj, cs):
    """Independent formulation: repeatedly take the best remaining candidate
    (largest score, then smallest i, then smallest j) and delete everything sharing an end with it."""
    rem = list(zip(cs.tolist(), ci.tolist(), cj.tolist()))
    out = []
    while rem:
        best = min(rem, key=lambda t: (-t[0], t[1], t[2]))
        out.append((best[1], best[2], best[0]))
        rem = [t for t in rem if t[1] != best[1] and t[2] != best[2]]
    return out


def cands(nA, nB, density, seed, levels=None):
    rng = np.random.default_rng(seed)
    mask = rng.random((nA, nB)) < density
    i, j = np.nonzero(mask)
    s = rng.random(len(i)).astype(np.float32) + np.float32(0.01)
    if levels:
        s = (np.ceil(s * levels) / levels).astype(np.float32)      # force score ties
    return i.astype(np.int32), j.astype(np.int32), s


@settings(max_examples=200, deadline=None)
@given(st.integers(1, 9), st.integers(1, 9), st.floats(0.1, 1.0), st.integers(0, 2 ** 31 - 1), st.sampled_from([None, 3]))
def test_brute_force(nA, nB, density, seed, levels):
    ci, cj, cs = cands(nA, nB, density, seed, levels)
    mi, mj, ms = oracle.match_limb(ci, cj, cs, nA, nB)
    assert list(zip(mi.tolist(), mj.tolist(), ms.tolist())) == brute_greedy(ci, cj, cs)


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 30), st.integers(1, 30), st.integers(0, 2 ** 31 - 1))
def test_properties(nA, nB, seed):
    ci, cj, cs = cands(nA, nB, 0.4, seed, levels=5)
    mi, mj, ms = oracle.match_limb(ci, cj, cs, nA, nB)
    # a matching
    assert len(set(mi.tolist())) == len(mi) and len(set(mj.tolist())) == len(mj)
    # acceptance order follows the strict order
    keys = [(-s, i, j) for i, j, s in zip(mi.tolist(), mj.tolist(), ms.tolist())]
    assert keys == sorted(keys)
    # maximal, and every rejected candidate lost to a better accepted one
    acc = {(i, j): s for i, j, s in zip(mi.tolist(), mj.tolist(), ms.tolist())}
    for i, j, s in zip(ci.tolist(), cj.tolist(), cs.tolist()):
        if (i, j) in acc:
            assert acc[(i, j)] == s
            continue
        rivals = [(-s2, i2, j2) for (i2, j2), s2 in acc.items() if i2 == i or j2 == j]
        assert rivals and min(rivals) < (-s, i, j)
    # input order does not matter
    perm = np.random.default_rng(seed).permutation(len(ci))
    mi2, mj2, ms2 = oracle.match_limb(ci[perm], cj[perm], cs[perm], nA, nB)
    assert np.array_equal(mi, mi2) and np.array_equal(mj, mj2) and np.array_equal(ms, ms2)


def test_equals_optimal_assignment_when_dominant():
    """Library pin: if every chosen entry is the maximum of both its row and its column,
    greedy and the optimal assignment (scipy) coincide."""
    rng = np.random.default_rng(9)
    n = 12
    perm = rng.permutation(n)
    M = rng.random((n, n)).astype(np.float32) * 0.4
    M[np.arange(n), perm] = 0.5 + rng.random(n).astype(np.float32) * 0.5
    i, j = np.nonzero(np.ones_like(M, bool))
    mi, mj, ms = oracle.match_limb(i, j, M[i, j], n, n)
    r, c = linear_sum_assignment(M.astype(np.float64), maximize=True)
    got = dict(zip(mi.tolist(), mj.tolist()))
    assert got == dict(zip(r.tolist(), c.tolist())) == dict(zip(range(n), perm.tolist()))
    assert np.all(np.diff(ms) <= 0)


def test_tie_break_and_empty():
    ci = np.array([1, 0, 1, 0], np.int32)
    cj = np.array([1, 1, 0, 0], np.int32)
    cs = np.array([0.5, 0.5, 0.5, 0.5], np.float32)
    mi, mj, ms = oracle.match_limb(ci, cj, cs, 2, 2)
    assert list(zip(mi.tolist(), mj.tolist())) == [(0, 0), (1, 1)]
    e = np.array([], np.int32)
    mi, mj, ms = oracle.match_limb(e, e, e.astype(np.float32), 3, 0)
    assert len(mi) == 0
