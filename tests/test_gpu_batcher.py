"""GPU tests of the streaming front (hp_batcher_*): whatever batch a frame ends up in, its result is
the oracle's result for that frame, frames leave in arrival order, and the batch slot grows only
while batches are running."""
import numpy as np
import pytest
import torch

from synth import CONFIGS, BENCH_CAPS, COCO18, BODY25, SynthConfig, generate, DEFAULT_PARAMS
from parity import assert_lists_equal, assert_poses_equal, run_oracle, caps_for

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def hp():
    import paper_2108_11826_amd as m
    return m


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


class Rig:
    """A workload, its oracle result and a batcher over freshly allocated lanes."""

    def __init__(self, cfg, n_lanes, max_batch, depth, caps=None):
        m = hp()
        self.m = m
        self.cfg = cfg
        self.batch = generate(cfg)
        self.ora = run_oracle(self.batch, DEFAULT_PARAMS)
        sk = cfg.skeleton
        cap, ccap, pcap = caps or caps_for(self.ora)
        dtype = torch.float16 if cfg.dtype == "float16" else torch.float32
        self.lanes = m.BatcherLanes(n_lanes, max_batch, sk.n_parts, sk.n_limbs, cfg.h, cfg.w, cap, ccap, pcap, dtype, DEV)
        self.skel = m.Skeleton(sk.n_parts, sk.limb_a, sk.limb_b)
        p = DEFAULT_PARAMS
        self.prm = m.Params(p.peak_thr, p.paf_thr, p.n_samples, p.min_valid_ratio, p.min_parts, p.scale)
        self.cm, self.paf = to_dev(self.batch.cm), to_dev(self.batch.paf)
        self.n_img = self.cm.shape[0]
        self.max_batch = max_batch
        torch.cuda.synchronize()
        self.b = m.hp_batcher_create(self.skel, self.prm, self.lanes, depth)
        self.seen = []           # (tag, batch size) in the order results came out
        self.sizes = []          # batch sizes in hand-out order
        self.next_seq = 0

    def submit(self, tag, **kw):
        i = tag % self.n_img
        return self.m.hp_batcher_submit(self.b, self.cm[i], self.paf[i], tag, **kw)

    def take(self, timeout_ms=20000, release=True):
        """Takes one finished batch and checks every frame of it against the oracle's result for that frame."""
        info = self.m.hp_batcher_next(self.b, self.max_batch, timeout_ms)
        if info is None:
            return None
        assert self.next_seq is None or info["seq"] == self.next_seq
        self.next_seq = info["seq"] + 1
        n = info["n_frames"]
        assert 1 <= n <= self.max_batch and len(info["tags"]) == n
        assert info["done_ns"] >= info["start_ns"] >= max(info["commit_ns"])
        buf = self.lanes.buf[info["lane"]]
        assert buf.host_status() == 0
        pick = [t % self.n_img for t in info["tags"]]
        assert_lists_equal("peaks", buf.host_peaks()[0][:n], [self.ora["peaks"][i] for i in pick])
        assert_lists_equal("candidates", buf.host_cands()[0][:n], [self.ora["candidates"][i] for i in pick])
        assert_lists_equal("connections", buf.host_conns()[0][:n], [self.ora["conns"][i] for i in pick])
        assert_poses_equal(buf.host_poses()[0][:n], [self.ora["poses"][i] for i in pick])
        self.seen += [(t, n) for t in info["tags"]]
        self.sizes.append(n)
        if release:
            self.m.hp_batcher_release(self.b, info["lane"])
        return info

    def close(self):
        self.m.hp_batcher_destroy(self.b)
        self.b = None


def hold_stream(stream, ms=30):
    """Keeps `stream` busy for some tens of milliseconds (a chain of matrix products)."""
    with torch.cuda.stream(stream):
        a = torch.ones((2048, 2048), device=DEV)
        for _ in range(max(1, ms // 2) * 4):
            a = (a @ a) * 1e-4
    return a


SMALL3 = SynthConfig(13, COCO18, 3, 33, 47, 6, noise_sd=0.02, dropout=0.1, n_spurious=10)
SMALL_F16 = SynthConfig(14, BODY25, 2, 31, 65, 5, noise_sd=0.02, dtype="float16")


@pytest.mark.parametrize("cfg", [SMALL3, SMALL_F16, CONFIGS[2]], ids=["syn13", "syn14-f16", "cfg2"])
def test_frames_handed_in_slower_than_the_gpu_are_never_batched(cfg):
    caps = BENCH_CAPS[2] if cfg is CONFIGS[2] else None
    r = Rig(cfg, n_lanes=2, max_batch=4, depth=1, caps=caps)
    for tag in range(2 * r.n_img + 1):
        assert r.submit(tag)
        info = r.take()
        assert info is not None and info["n_frames"] == 1 and info["tags"] == [tag]
    assert r.take(timeout_ms=0) is None
    r.close()


def test_the_slot_fills_while_a_batch_is_running():
    # lane 0's stream is held busy, so the first frame's batch stays "running": the next 16 frames fill the two
    # other lanes, the 18th finds every lane taken; results then come out in arrival order
    r = Rig(CONFIGS[2], n_lanes=3, max_batch=8, depth=1, caps=BENCH_CAPS[2])
    keep = hold_stream(r.lanes.streams[0], 40)
    for tag in range(17):
        assert r.submit(tag)
    assert r.submit(17) is False
    first = r.take()
    assert first["n_frames"] == 1 and first["lane"] == 0
    assert r.submit(17)                    # lane 0 is free again and collects while lane 1 runs ...
    r.m.hp_batcher_flush(r.b)              # ... until the stream of frames ends
    while len(r.seen) < 18:
        assert r.take() is not None
    assert r.sizes[:3] == [1, 8, 8] and sum(r.sizes) == 18
    assert [t for t, _ in r.seen] == list(range(18))
    del keep
    r.close()


def test_one_lane_runs_batches_of_changing_size():
    # the same lane (buffers and workspace laid out for 8 frames) runs 8, 1, 5, 8, 3 frames in turn
    r = Rig(CONFIGS[2], n_lanes=2, max_batch=8, depth=1, caps=BENCH_CAPS[2])
    tag = 0
    for k in (8, 1, 5, 8, 3):
        keep = hold_stream(r.lanes.streams[0], 20)
        assert r.submit(tag)               # a batch of one on lane 0, behind the held stream
        tag += 1
        for _ in range(k):                 # lane 1 collects k frames meanwhile
            assert r.submit(tag)
            tag += 1
        r.m.hp_batcher_flush(r.b)
        a, b = r.take(), r.take()
        assert (a["lane"], a["n_frames"]) == (0, 1) and (b["lane"], b["n_frames"]) == (1, k)
        del keep
    assert [t for t, _ in r.seen] == list(range(tag))
    r.close()


def test_two_batches_in_flight():
    r = Rig(CONFIGS[1], n_lanes=4, max_batch=4, depth=2, caps=BENCH_CAPS[1])
    keep0, keep1 = hold_stream(r.lanes.streams[0], 30), hold_stream(r.lanes.streams[1], 30)
    for tag in range(10):                  # 1 + 1 start at once (two may run), then 4 + 4 collect
        assert r.submit(tag)
    assert r.submit(10) is False
    while len(r.seen) < 10:
        assert r.take() is not None
    assert r.sizes == [1, 1, 4, 4]
    assert [t for t, _ in r.seen] == list(range(10))
    del keep0, keep1
    r.close()


def test_frames_written_in_place_by_a_producer_stream():
    # the producer writes each frame into the slot it was given, on its own stream, after a long-running piece of
    # work: the batch must wait for that write (without the ordering it would read the zeros the slots start with)
    r = Rig(SMALL3, n_lanes=2, max_batch=4, depth=1)
    producer = torch.cuda.Stream()
    for tag in range(6):
        place = r.m.hp_batcher_acquire(r.b)
        assert place is not None
        lane, idx = r.lanes.slot_of(place[0])
        keep = hold_stream(producer, 4)
        with torch.cuda.stream(producer):
            r.lanes.cm[lane][idx].copy_(r.cm[tag % r.n_img], non_blocking=True)
            r.lanes.paf[lane][idx].copy_(r.paf[tag % r.n_img], non_blocking=True)
        r.m.hp_batcher_commit(r.b, tag, producer_stream=producer, ready=False)
        if tag % 2 == 1:
            r.m.hp_batcher_flush(r.b)
            while len(r.seen) <= tag:
                assert r.take() is not None
        del keep
    assert [t for t, _ in r.seen] == list(range(6))
    r.close()


def test_call_order_and_back_pressure():
    m = hp()
    r = Rig(SMALL3, n_lanes=2, max_batch=2, depth=1)
    with pytest.raises(m.HPError) as e:
        m.hp_batcher_commit(r.b, 0, ready=True)                 # nothing acquired
    assert e.value.code == -8
    with pytest.raises(m.HPError) as e:
        m.hp_batcher_release(r.b, 0)                            # lane not handed out
    assert e.value.code == -8
    with pytest.raises(m.HPError) as e:
        m.hp_batcher_next(r.b, r.max_batch, -1)                 # nothing can finish: an unlimited wait is refused
    assert e.value.code == -8
    assert m.hp_batcher_next(r.b, r.max_batch, 0) is None
    assert m.hp_batcher_acquire(r.b) is not None
    with pytest.raises(m.HPError) as e:
        m.hp_batcher_acquire(r.b)                               # one place at a time
    assert e.value.code == -8
    with pytest.raises(m.HPError) as e:
        m.hp_batcher_flush(r.b)                                 # not while a place is acquired
    assert e.value.code == -8
    # the acquired place is lane 0, index 0: fill it by hand and hand it over
    r.lanes.cm[0][0].copy_(r.cm[0])
    r.lanes.paf[0][0].copy_(r.paf[0])
    torch.cuda.synchronize()
    m.hp_batcher_commit(r.b, 0, ready=True)
    a = r.take(release=False)                                   # lane 0 held by the consumer
    assert a["lane"] == 0 and a["n_frames"] == 1
    assert r.submit(1)                                          # lane 1 runs at once
    b = r.take(release=False)
    assert b["lane"] == 1
    assert r.submit(2) is False                                 # both lanes held: back pressure
    assert r.submit(2, timeout_ms=20) is False
    m.hp_batcher_release(r.b, 0)
    with pytest.raises(m.HPError):
        m.hp_batcher_release(r.b, 0)                            # released twice
    assert r.submit(2)
    c = r.take()
    assert c["lane"] == 0 and c["tags"] == [2]
    # destroy with lane 1 still held and a batch still running on lane 0
    keep = hold_stream(r.lanes.streams[0], 10)
    assert r.submit(3)
    del keep
    r.close()


@pytest.mark.parametrize("copy", [False, True], ids=["in_place", "copied"])
def test_load_generator(copy):
    m = hp()
    r = Rig(CONFIGS[2], n_lanes=4, max_batch=8, depth=2, caps=BENCH_CAPS[2])
    for l in range(r.lanes.n_lanes):       # in-place mode uses the staging tensors as they are: fill them
        r.lanes.cm[l].copy_(r.cm)
        r.lanes.paf[l].copy_(r.paf)
    torch.cuda.synchronize()
    src = (r.cm, r.paf) if copy else (None, None)
    # one frame every 2 ms: the GPU is idle at every arrival
    lat, size, elapsed = m.hp_batcher_drive(r.b, 50, 2_000_000, *src)
    # (a stall of the host thread for more than one period would pair two frames: allow a few)
    assert np.count_nonzero(size == 1) >= 45 and size.max() <= 2 and np.all(lat > 0) and np.median(lat) < 1_000_000
    assert elapsed >= 49 * 2_000_000
    # as fast as the frames are taken: batches form
    lat, size, elapsed = m.hp_batcher_drive(r.b, 2000, 0, *src)
    assert size.min() >= 1 and size.max() <= 8 and size.max() > 1
    assert np.all(lat > 0) and elapsed > 0
    # the batcher is idle again and still gives the oracle's results
    r.next_seq = None                      # the load generator took its batches itself
    for tag in range(3):
        assert r.submit(tag)
        assert r.take()["n_frames"] == 1
    r.close()


def test_producer_and_consumer_threads_with_random_pauses():
    # two host threads, as the front is meant to be used: one hands frames in (copied or written in place, at random
    # paces, flushing now and then), one takes batches, checks every frame against the oracle and releases lanes late
    import threading
    import time
    m = hp()
    r = Rig(SMALL3, n_lanes=4, max_batch=5, depth=2)
    n_frames = 400
    rng = np.random.default_rng(3)
    pauses = rng.choice([0.0, 0.0, 0.0, 1e-4, 1e-3], n_frames)
    in_place = rng.random(n_frames) < 0.3
    errors = []

    def produce():
        try:
            stream = torch.cuda.Stream()
            for tag in range(n_frames):
                if pauses[tag]:
                    time.sleep(pauses[tag])
                if in_place[tag]:
                    place = None
                    while place is None:
                        place = m.hp_batcher_acquire(r.b, timeout_ms=50)
                    lane, idx = r.lanes.slot_of(place[0])
                    with torch.cuda.stream(stream):
                        r.lanes.cm[lane][idx].copy_(r.cm[tag % r.n_img], non_blocking=True)
                        r.lanes.paf[lane][idx].copy_(r.paf[tag % r.n_img], non_blocking=True)
                    m.hp_batcher_commit(r.b, tag, producer_stream=stream, ready=False)
                else:
                    while not r.submit(tag, timeout_ms=50, ready=True):
                        pass
                if tag % 37 == 36:
                    m.hp_batcher_flush(r.b)
            m.hp_batcher_flush(r.b)
        except Exception as e:      # surfaced by the main thread
            errors.append(e)

    t = threading.Thread(target=produce)
    t.start()
    deadline = time.time() + 60
    held = []
    while len(r.seen) < n_frames and time.time() < deadline and not errors:
        info = r.take(timeout_ms=200, release=False)
        if info is None:
            continue
        held.append(info["lane"])
        if len(held) > 1 or rng.random() < 0.5:      # keep a lane for a while now and then
            for lane in held:
                m.hp_batcher_release(r.b, lane)
            held = []
    for lane in held:
        m.hp_batcher_release(r.b, lane)
    t.join(timeout=30)
    assert not errors, errors
    assert [tag for tag, _ in r.seen] == list(range(n_frames))
    assert max(r.sizes) <= 5 and sum(r.sizes) == n_frames
    r.close()
