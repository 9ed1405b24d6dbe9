"""The dynamic batch slot's decisions (hp_batch_simulate runs the library's own state machine in
virtual time) against a small model written here from the rule of Section 2.2.2 and against
cases whose answer is known in closed form.  No GPU is needed."""
import os

import numpy as np
import pytest


@pytest.fixture(scope="module")
def hp():
    from paper_2108_11826_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2108_11826_amd import build
        build.build()
    import paper_2108_11826_amd as m
    return m


def model(arrival, max_batch, depth, n_lanes, base, per):
    """Event loop written from the rule: a frame starts the collecting batch when fewer than `depth`
    batches run, otherwise the batch keeps collecting up to max_batch; a finishing batch (seen in
    start order) starts the oldest full batch, else the collecting one; with every lane taken a
    frame waits for the next completion.  A lane is free again when its batch is seen finished."""
    n = len(arrival)
    seq_of, size_of, done_of = [None] * n, [None] * n, [None] * n
    running = []          # [seen_time, frames] in start order
    full = []             # closed batches waiting for the GPU
    cur = []              # the collecting batch
    last_seen, seq, now, k = 0, 0, 0, 0

    def start(frames, t):
        nonlocal last_seen, seq
        last_seen = max(last_seen, t + base + per * len(frames))
        running.append((last_seen, frames))
        for f in frames:
            seq_of[f], size_of[f], done_of[f] = seq, len(frames), last_seen
        seq += 1

    def lanes_taken():
        return len(running) + len(full) + (1 if cur else 0)

    while k < n or running or full or cur:
        arrival_first = k < n and (not running or arrival[k] <= running[0][0])
        if arrival_first and (cur or lanes_taken() < n_lanes):
            now = max(now, arrival[k])
            cur.append(k)
            k += 1
            if len(running) < depth:
                start(cur, now)
                cur = []
            elif len(cur) == max_batch:
                full.append(cur)
                cur = []
            continue
        if running:
            t, _ = running.pop(0)
            now = max(now, t)
            while len(running) < depth and (full or cur):
                if full:
                    start(full.pop(0), now)
                else:
                    start(cur, now)
                    cur = []
            continue
        start(cur, now)    # the stream ended with frames collected and nothing running
        cur = []
    return np.array(seq_of), np.array(size_of), np.array(done_of)


def test_slow_arrivals_are_never_batched(hp):
    # the GPU is idle at every arrival: each frame is its own batch and waits for nothing
    arr = np.arange(50) * 1_000_000
    seq, size, done = hp.hp_batch_simulate(arr, 8, 1, 2, 40_000, 5_000)
    assert np.array_equal(seq, np.arange(50))
    assert np.all(size == 1)
    assert np.array_equal(done - arr, np.full(50, 45_000))


def test_a_burst_fills_the_slot(hp):
    # everything arrives at once: the first frame finds the GPU idle, the rest collect to max_batch
    arr = np.zeros(30, np.int64)
    seq, size, done = hp.hp_batch_simulate(arr, 8, 1, 2, 40_000, 5_000)
    assert size.tolist() == [1] + [8] * 24 + [5] * 5
    assert seq.tolist() == [0] + [1] * 8 + [2] * 8 + [3] * 8 + [4] * 5
    # batches run back to back: 45, then +80 each, the last one +65 us
    assert sorted(set(done.tolist())) == [45_000, 125_000, 205_000, 285_000, 350_000]


def test_steady_state_batch_size_under_load(hp):
    # arrivals every 10 us, service 40 + 5 n us, one batch at a time: a batch of n frames takes as long
    # as it takes n frames to arrive when 40 + 5 n = 10 n, so the batch size settles at 8
    arr = np.arange(400) * 10_000
    seq, size, done = hp.hp_batch_simulate(arr, 16, 1, 2, 40_000, 5_000)
    assert np.all(size[100:300] == 8)
    # the same load against a slot of 4: the GPU cannot keep up (60 us per 4 frames), every batch is full
    seq, size, done = hp.hp_batch_simulate(arr, 4, 1, 2, 40_000, 5_000)
    assert np.all(size[8:-4] == 4)
    lat = done - arr
    assert lat[-1] > lat[50] > lat[10]      # and the delay grows without bound


def test_batches_shrink_again_when_the_load_drops(hp):
    arr = np.concatenate([np.arange(100) * 5_000, 500_000 + 5_000 * 100 + np.arange(50) * 500_000])
    seq, size, done = hp.hp_batch_simulate(arr, 8, 1, 3, 40_000, 5_000)
    assert size[10:90].max() == 8 and size[10:90].mean() > 6
    assert np.all(size[110:] == 1)


@pytest.mark.parametrize("seed", range(40))
def test_against_the_model(hp, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 300))
    max_batch = int(rng.integers(1, 12))
    n_lanes = int(rng.integers(1, 6))
    depth = int(rng.integers(1, n_lanes + 1))
    base, per = int(rng.integers(0, 60_000)), int(rng.integers(0, 9_000))
    gap = rng.choice([0, 1_000, 10_000, 100_000])
    arr = np.cumsum(rng.exponential(gap, n).astype(np.int64)) if gap else np.zeros(n, np.int64)
    if seed % 5 == 0:       # bursts with pauses
        arr = np.sort(np.concatenate([arr[: n // 2], arr[n // 2:] + 3_000_000]))
    got = hp.hp_batch_simulate(arr, max_batch, depth, n_lanes, base, per)
    want = model(arr.tolist(), max_batch, depth, n_lanes, base, per)
    for g, w_ in zip(got, want):
        assert np.array_equal(g, w_)
    seq, size, done = got
    # what holds for any input: order kept, sizes consistent, nothing finishes before it could
    assert np.all(np.diff(seq) >= 0) and np.all(np.diff(done) >= 0)
    assert size.max() <= max_batch
    for s in np.unique(seq):
        assert np.count_nonzero(seq == s) == size[seq == s][0]
    assert np.all(done - arr >= base + per * size)


def test_simulate_rejects_bad_calls(hp):
    from paper_2108_11826_amd import HPError
    with pytest.raises(HPError):
        hp.hp_batch_simulate([0, 1], 0, 1, 1, 1, 1)        # max_batch
    with pytest.raises(HPError):
        hp.hp_batch_simulate([0, 1], 4, 3, 2, 1, 1)        # depth > lanes
    with pytest.raises(HPError):
        hp.hp_batch_simulate([5, 1], 4, 1, 2, 1, 1)        # arrivals out of order
    with pytest.raises(HPError):
        hp.hp_batch_simulate([0, 1], 4, 1, 2, -1, 1)
    seq, size, done = hp.hp_batch_simulate([], 4, 1, 2, 1, 1)
    assert len(seq) == 0
