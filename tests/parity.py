"""Helpers shared by the GPU parity tests: run both sides on the same seeded inputs and compare.

Bar: integers, orders and counts bit-exact; floats within 1e-5 relative (the arithmetic is
specified operation by operation, so they are expected to be bit-identical, which is checked too)."""
import os

import numpy as np

RTOL = 1e-5
ATOL = 1e-30
THREADS = min(16, len(os.sched_getaffinity(0)))


def close(g, o):
    g = np.asarray(g, np.float32)
    o = np.asarray(o, np.float32)
    return g.shape == o.shape and bool(np.all(np.abs(g - o) <= RTOL * np.maximum(np.abs(g), np.abs(o)) + ATOL))


def assert_lists_equal(kind, gpu, ora, exact_floats=True):
    """gpu / ora: [n][c] -> (int array, int array, float array)."""
    assert len(gpu) == len(ora)
    for n in range(len(ora)):
        assert len(gpu[n]) == len(ora[n])
        for c in range(len(ora[n])):
            ga, gb, gs = gpu[n][c]
            oa, ob, os_ = ora[n][c]
            where = f"{kind} image {n} index {c}"
            assert len(ga) == len(oa), f"{where}: count {len(ga)} vs {len(oa)}"
            assert np.array_equal(ga, oa) and np.array_equal(gb, ob), where
            assert close(gs, os_), where
            if exact_floats:
                assert np.array_equal(np.asarray(gs, np.float32).view(np.uint32),
                                      np.asarray(os_, np.float32).view(np.uint32)), where + " (bits)"


def assert_poses_equal(gpu, ora):
    assert len(gpu) == len(ora)
    for n in range(len(ora)):
        gs, gn, gsc = gpu[n]
        os_, on, osc = ora[n]
        assert gs.shape == os_.shape, f"poses image {n}: {gs.shape} vs {os_.shape}"
        assert np.array_equal(gs, os_), f"pose slots image {n}"
        assert np.array_equal(gn, on), f"pose nparts image {n}"
        assert close(gsc, osc), f"pose scores image {n}"
        assert np.array_equal(gsc.view(np.uint32), osc.view(np.uint32)), f"pose scores image {n} (bits)"


def run_oracle(batch, params, threads=THREADS):
    import oracle
    sk = batch.config.skeleton
    return oracle.postprocess(batch.cm, batch.paf, sk.limb_a, sk.limb_b, params, threads=threads)


def caps_for(ora, slack=1.25):
    """Capacities large enough for an oracle result (what a caller would provision)."""
    pk = max(len(p[0]) for im in ora["peaks"] for p in im)
    cc = max(len(c[0]) for im in ora["candidates"] for c in im)
    pp = max(len(p[1]) for p in ora["poses"])
    r = lambda v: max(16, int(v * slack) + 8)
    return r(pk), r(cc), r(pp)
