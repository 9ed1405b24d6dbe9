// Streaming front of the operator: the dynamic batch slot of Section 2.2.2 in front of
// hp_postprocess (hp_batcher_*), its virtual-time simulation and a load generator.
// Host code but for one copy kernel; every decision is taken by BatchPolicy, every step of the
// operator by hp_postprocess.
#include <string.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "batch_policy.h"
#include "hp_dev.h"

namespace hp {

struct Lane {
    hp_lane d;
    hipEvent_t done_ev = nullptr;    // recorded after the batch's last kernel
    hipEvent_t ready_ev = nullptr;   // orders the lane's stream after a producer's stream
    hp_batch_info info;
    std::vector<uint64_t> tags;
    std::vector<int64_t> commit_ns;
};

}  // namespace hp

struct hp_batcher {
    std::mutex mu;
    std::condition_variable cv_run;    // a batch started (wakes the batcher's thread)
    std::condition_variable cv_done;   // a batch finished
    std::condition_variable cv_free;   // a lane was released
    hp::BatchPolicy pol;
    std::vector<hp::Lane> lanes;
    hp_dtype dt;
    int h, w, K, L, max_batch, device;
    std::vector<int32_t> limb_a, limb_b;
    hp_skeleton skel;
    hp_params prm;
    size_t cm_frame_bytes, paf_frame_bytes;
    uint64_t next_seq = 0;
    int acq_lane = -1, acq_index = -1;
    std::deque<int> handoff;           // started batches the batcher's thread still has to enqueue, in order
    bool stop = false;
    std::thread waiter;
    std::chrono::steady_clock::time_point t0;

    hp_batcher(int max_batch_, int depth, int n_lanes) : pol(max_batch_, depth, n_lanes), lanes((size_t)n_lanes) {}

    int64_t now() const
    {
        return std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0).count();
    }
};

namespace hp {

static size_t elem_bytes(hp_dtype dt) { return dt == HP_F16 ? 2 : 4; }

// Copies one frame (its CM and its PAF tensor) into a lane's staging tensors in one launch,
// 16 bytes per thread; a launch costs the host a fraction of what two memcpy calls do.
__global__ __launch_bounds__(kBlock) void k_copy_frame(const uint4 *__restrict__ cm_src, uint4 *__restrict__ cm_dst,
                                                       unsigned n_cm, const uint4 *__restrict__ paf_src,
                                                       uint4 *__restrict__ paf_dst, unsigned n_paf)
{
    const unsigned t = blockIdx.x * kBlock + threadIdx.x;
    if (t < n_cm)
        cm_dst[t] = cm_src[t];
    else if (t - n_cm < n_paf)
        paf_dst[t - n_cm] = paf_src[t - n_cm];
}

static hipError_t copy_frame(const void *cm_src, void *cm_dst, size_t cm_bytes, const void *paf_src, void *paf_dst,
                             size_t paf_bytes, hipStream_t s)
{
    const uintptr_t bits = (uintptr_t)cm_src | (uintptr_t)cm_dst | (uintptr_t)paf_src | (uintptr_t)paf_dst | cm_bytes | paf_bytes;
    if ((bits & 15) == 0 && (cm_bytes + paf_bytes) / 16 < (1ull << 31)) {
        const unsigned n_cm = (unsigned)(cm_bytes / 16), n_paf = (unsigned)(paf_bytes / 16);
        const unsigned blocks = (n_cm + n_paf + kBlock - 1) / kBlock;
        k_copy_frame<<<blocks, kBlock, 0, s>>>((const uint4 *)cm_src, (uint4 *)cm_dst, n_cm, (const uint4 *)paf_src,
                                              (uint4 *)paf_dst, n_paf);
        return hipGetLastError();
    }
    hipError_t e = hipMemcpyAsync(cm_dst, cm_src, cm_bytes, hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return e;
    return hipMemcpyAsync(paf_dst, paf_src, paf_bytes, hipMemcpyDeviceToDevice, s);
}

// Enqueues one batch: the operator on the lane's first n frames, then the event that marks its end.
// The lane is in the running state, so nothing else touches its buffers; may run without b->mu.
static void launch_lane(hp_batcher *b, int l)
{
    Lane &ln = b->lanes[(size_t)l];
    ln.info.start_ns = b->now();
    int rc = postprocess(ln.d.cm_lo, ln.d.paf_lo, b->dt, ln.info.n_frames, b->max_batch, b->h, b->w, &b->skel, &b->prm,
                         nullptr, nullptr, &ln.d.peaks, &ln.d.cands, &ln.d.conns, &ln.d.poses, ln.d.workspace,
                         ln.d.ws_bytes, ln.d.status, ln.d.stream, false);
    // the event is recorded even after a failed call: the lane then completes at once and
    // carries the error to hp_batcher_next
    if (hipEventRecord(ln.done_ev, (hipStream_t)ln.d.stream) != hipSuccess && rc == HP_OK) rc = HP_ERR_HIP;
    ln.info.rc = rc;
}

// Takes over the batches the policy decided to start.  Called with b->mu held.  A batch that
// starts while nothing else runs is enqueued here and now, on the caller's thread: the GPU is
// idle and the frame's delay is what counts.  Otherwise the batcher's thread enqueues it, so
// that a producer handing in frames under load never pays for kernel launches.
static void take_over(hp_batcher *b, const std::vector<int> &start, bool may_launch_here)
{
    if (start.empty()) return;
    const bool idle_before = b->handoff.empty() && b->pol.running() == (int)start.size();
    for (int l : start) {
        Lane &ln = b->lanes[(size_t)l];
        ln.info.lane = l;
        ln.info.n_frames = b->pol.frames(l);
        ln.info.seq = b->next_seq++;
        ln.info.reserved = 0;
        ln.info.rc = HP_OK;
        ln.info.start_ns = ln.info.done_ns = 0;
        if (may_launch_here && idle_before && l == start.front())
            launch_lane(b, l);
        else
            b->handoff.push_back(l);
    }
    b->cv_run.notify_one();
}

// The batcher's thread: enqueues the batches handed to it, in order, and polls the end of the
// oldest running batch (it spins only while a batch is in flight, and sleeps otherwise); a
// finished batch releases what the policy starts next.  Exits when asked to stop and nothing runs.
static void dispatcher_main(hp_batcher *b)
{
    (void)hipSetDevice(b->device);
    std::unique_lock<std::mutex> lk(b->mu);
    for (;;) {
        b->cv_run.wait(lk, [&] { return b->stop || !b->handoff.empty() || b->pol.oldest_running() >= 0; });
        if (!b->handoff.empty()) {
            const int l = b->handoff.front();
            b->handoff.pop_front();
            lk.unlock();
            launch_lane(b, l);
            lk.lock();
            continue;
        }
        const int l = b->pol.oldest_running();
        if (l < 0) {
            if (b->stop) return;
            continue;
        }
        Lane &ln = b->lanes[(size_t)l];
        lk.unlock();
        const hipError_t e = hipEventQuery(ln.done_ev);
        if (e == hipErrorNotReady) {
            __builtin_ia32_pause();
            lk.lock();
            continue;
        }
        const int64_t t = b->now();
        lk.lock();
        if (e != hipSuccess && ln.info.rc == HP_OK) ln.info.rc = HP_ERR_HIP;
        ln.info.done_ns = t;
        std::vector<int> start;
        b->pol.complete(start);
        take_over(b, start, false);
        b->cv_done.notify_all();
    }
}

template <typename Pred>
static bool wait_for(std::condition_variable &cv, std::unique_lock<std::mutex> &lk, int timeout_ms, Pred pred)
{
    if (timeout_ms == 0) return pred();
    if (timeout_ms < 0) {
        cv.wait(lk, pred);
        return true;
    }
    return cv.wait_for(lk, std::chrono::milliseconds(timeout_ms), pred);
}

}  // namespace hp

using namespace hp;

extern "C" {

int hp_batcher_create(hp_dtype dt, int h, int w, const hp_skeleton *skel, const hp_params *prm,
                      const hp_batcher_config *cfg, const hp_lane *lanes, hp_batcher **out)
{
    if (!out) return HP_ERR_INVALID_ARG;
    *out = nullptr;
    if (!skel || !prm || !cfg || !lanes || !skel->limb_a || !skel->limb_b) return HP_ERR_INVALID_ARG;
    if (dt != HP_F32 && dt != HP_F16) return HP_ERR_DTYPE;
    if (cfg->max_batch <= 0 || cfg->n_lanes <= 0 || cfg->depth <= 0 || cfg->depth > cfg->n_lanes) return HP_ERR_INVALID_ARG;
    if (cfg->max_batch > HP_MAX_BATCH || cfg->n_lanes > HP_MAX_LANES) return HP_ERR_UNSUPPORTED;
    if (skel->n_parts <= 0 || skel->n_limbs <= 0) return HP_ERR_INVALID_ARG;
    if (skel->n_parts > HP_MAX_PARTS || skel->n_limbs > HP_MAX_LIMBS) return HP_ERR_UNSUPPORTED;
    if (h <= 0 || w <= 0) return HP_ERR_INVALID_ARG;
    for (int l = 0; l < cfg->n_lanes; ++l) {
        const hp_lane &d = lanes[l];
        if (!d.cm_lo || !d.paf_lo || !d.status) return HP_ERR_INVALID_ARG;
        for (int m = 0; m < l; ++m)
            if (lanes[m].cm_lo == d.cm_lo || lanes[m].paf_lo == d.paf_lo || lanes[m].workspace == d.workspace ||
                lanes[m].status == d.status)
                return HP_ERR_INVALID_ARG;
    }
    hp_batcher *b = new (std::nothrow) hp_batcher(cfg->max_batch, cfg->depth, cfg->n_lanes);
    if (!b) return HP_ERR_INVALID_ARG;
    b->dt = dt;
    b->h = h;
    b->w = w;
    b->K = skel->n_parts;
    b->L = skel->n_limbs;
    b->max_batch = cfg->max_batch;
    b->limb_a.assign(skel->limb_a, skel->limb_a + skel->n_limbs);
    b->limb_b.assign(skel->limb_b, skel->limb_b + skel->n_limbs);
    b->skel.n_parts = b->K;
    b->skel.n_limbs = b->L;
    b->skel.limb_a = b->limb_a.data();
    b->skel.limb_b = b->limb_b.data();
    b->prm = *prm;
    b->cm_frame_bytes = elem_bytes(dt) * (size_t)(b->K + 1) * h * w;
    b->paf_frame_bytes = elem_bytes(dt) * (size_t)(2 * b->L) * h * w;
    b->t0 = std::chrono::steady_clock::now();
    int rc = HP_OK;
    for (int l = 0; l < cfg->n_lanes && rc == HP_OK; ++l) {
        Lane &ln = b->lanes[(size_t)l];
        ln.d = lanes[l];
        ln.tags.resize((size_t)cfg->max_batch);
        ln.commit_ns.resize((size_t)cfg->max_batch);
        memset(&ln.info, 0, sizeof(ln.info));
        // everything hp_postprocess checks, for a full batch, with nothing enqueued
        rc = postprocess(ln.d.cm_lo, ln.d.paf_lo, dt, cfg->max_batch, cfg->max_batch, h, w, &b->skel, &b->prm, nullptr,
                         nullptr, &ln.d.peaks, &ln.d.cands, &ln.d.conns, &ln.d.poses, ln.d.workspace, ln.d.ws_bytes,
                         ln.d.status, ln.d.stream, true);
    }
    if (rc == HP_OK && hipGetDevice(&b->device) != hipSuccess) rc = HP_ERR_HIP;
    for (int l = 0; l < cfg->n_lanes && rc == HP_OK; ++l) {
        Lane &ln = b->lanes[(size_t)l];
        if (hipEventCreateWithFlags(&ln.done_ev, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&ln.ready_ev, hipEventDisableTiming) != hipSuccess)
            rc = HP_ERR_HIP;
    }
    if (rc != HP_OK) {
        for (Lane &ln : b->lanes) {
            if (ln.done_ev) (void)hipEventDestroy(ln.done_ev);
            if (ln.ready_ev) (void)hipEventDestroy(ln.ready_ev);
        }
        delete b;
        return rc;
    }
    b->waiter = std::thread(dispatcher_main, b);
    *out = b;
    return HP_OK;
}

int hp_batcher_destroy(hp_batcher *b)
{
    if (!b) return HP_ERR_INVALID_ARG;
    {
        std::unique_lock<std::mutex> lk(b->mu);
        b->pol.cancel();
        // full batches still waiting for the GPU are run to completion; the open one is dropped
        b->cv_done.wait(lk, [&] { return b->pol.running() == 0 && b->pol.waiting() == 0; });
        b->stop = true;
        b->cv_run.notify_all();
    }
    b->waiter.join();
    int rc = HP_OK;
    for (Lane &ln : b->lanes) {
        if (hipEventDestroy(ln.done_ev) != hipSuccess) rc = HP_ERR_HIP;
        if (hipEventDestroy(ln.ready_ev) != hipSuccess) rc = HP_ERR_HIP;
    }
    delete b;
    return rc;
}

int hp_batcher_acquire(hp_batcher *b, int timeout_ms, void **cm_slot, void **paf_slot)
{
    if (!b || !cm_slot || !paf_slot) return HP_ERR_INVALID_ARG;
    std::unique_lock<std::mutex> lk(b->mu);
    if (b->pol.pending()) return HP_ERR_STATE;
    int lane = -1, index = -1;
    const bool ok = wait_for(b->cv_free, lk, timeout_ms, [&] { return b->pol.acquire(lane, index); });
    if (!ok) return HP_ERR_BUSY;
    b->acq_lane = lane;
    b->acq_index = index;
    const Lane &ln = b->lanes[(size_t)lane];
    *cm_slot = (char *)ln.d.cm_lo + (size_t)index * b->cm_frame_bytes;
    *paf_slot = (char *)ln.d.paf_lo + (size_t)index * b->paf_frame_bytes;
    return HP_OK;
}

int hp_batcher_commit(hp_batcher *b, uint64_t tag, void *producer_stream, int ready)
{
    if (!b) return HP_ERR_INVALID_ARG;
    std::unique_lock<std::mutex> lk(b->mu);
    if (!b->pol.pending()) return HP_ERR_STATE;
    Lane &ln = b->lanes[(size_t)b->acq_lane];
    int rc = HP_OK;
    if (!ready && producer_stream != ln.d.stream) {
        // the batch must not start before the producer's enqueued work has written the frame
        if (hipEventRecord(ln.ready_ev, (hipStream_t)producer_stream) != hipSuccess ||
            hipStreamWaitEvent((hipStream_t)ln.d.stream, ln.ready_ev, 0) != hipSuccess)
            rc = HP_ERR_HIP;
    }
    if (rc != HP_OK) {
        b->pol.cancel();
        return rc;
    }
    ln.tags[(size_t)b->acq_index] = tag;
    ln.commit_ns[(size_t)b->acq_index] = b->now();
    std::vector<int> start;
    b->pol.commit(start);
    take_over(b, start, true);
    return HP_OK;
}

int hp_batcher_submit(hp_batcher *b, int timeout_ms, const void *cm_frame, const void *paf_frame, uint64_t tag,
                      void *producer_stream, int ready)
{
    if (!b || !cm_frame || !paf_frame) return HP_ERR_INVALID_ARG;
    void *cm_slot, *paf_slot;
    int rc = hp_batcher_acquire(b, timeout_ms, &cm_slot, &paf_slot);
    if (rc != HP_OK) return rc;
    hipStream_t ls;
    hipEvent_t ev;
    {
        std::unique_lock<std::mutex> lk(b->mu);
        ls = (hipStream_t)b->lanes[(size_t)b->acq_lane].d.stream;
        ev = b->lanes[(size_t)b->acq_lane].ready_ev;
    }
    // the open lane cannot start while a place is acquired, so its stream is ours to enqueue on
    bool ok = true;
    if (!ready && producer_stream != (void *)ls)
        ok = hipEventRecord(ev, (hipStream_t)producer_stream) == hipSuccess && hipStreamWaitEvent(ls, ev, 0) == hipSuccess;
    ok = ok && copy_frame(cm_frame, cm_slot, b->cm_frame_bytes, paf_frame, paf_slot, b->paf_frame_bytes, ls) == hipSuccess;
    if (!ok) {
        std::unique_lock<std::mutex> lk(b->mu);
        b->pol.cancel();
        return HP_ERR_HIP;
    }
    return hp_batcher_commit(b, tag, nullptr, 1);
}

int hp_batcher_flush(hp_batcher *b)
{
    if (!b) return HP_ERR_INVALID_ARG;
    std::unique_lock<std::mutex> lk(b->mu);
    std::vector<int> start;
    if (!b->pol.flush(start)) return HP_ERR_STATE;
    take_over(b, start, true);
    return HP_OK;
}

int hp_batcher_next(hp_batcher *b, int timeout_ms, hp_batch_info *info, uint64_t *tags, int64_t *commit_ns)
{
    if (!b || !info) return HP_ERR_INVALID_ARG;
    std::unique_lock<std::mutex> lk(b->mu);
    if (timeout_ms < 0 && b->pol.idle()) return HP_ERR_STATE;
    if (!wait_for(b->cv_done, lk, timeout_ms, [&] { return b->pol.finished() > 0; })) return HP_ERR_TIMEOUT;
    int lane = -1;
    b->pol.pop_done(lane);
    const Lane &ln = b->lanes[(size_t)lane];
    *info = ln.info;
    for (int k = 0; k < ln.info.n_frames; ++k) {
        if (tags) tags[k] = ln.tags[(size_t)k];
        if (commit_ns) commit_ns[k] = ln.commit_ns[(size_t)k];
    }
    return HP_OK;
}

int hp_batcher_release(hp_batcher *b, int lane)
{
    if (!b) return HP_ERR_INVALID_ARG;
    std::unique_lock<std::mutex> lk(b->mu);
    if (!b->pol.release(lane)) return HP_ERR_STATE;
    b->cv_free.notify_all();
    return HP_OK;
}

int hp_batch_simulate(int n_frames, const int64_t *arrival_ns, const hp_batcher_config *cfg, int64_t service_base_ns,
                      int64_t service_per_frame_ns, int64_t *batch_seq, int32_t *batch_size, int64_t *done_ns)
{
    if (n_frames < 0 || !cfg || (n_frames > 0 && (!arrival_ns || !batch_seq || !batch_size || !done_ns)))
        return HP_ERR_INVALID_ARG;
    if (cfg->max_batch <= 0 || cfg->n_lanes <= 0 || cfg->depth <= 0 || cfg->depth > cfg->n_lanes) return HP_ERR_INVALID_ARG;
    if (cfg->max_batch > HP_MAX_BATCH || cfg->n_lanes > HP_MAX_LANES) return HP_ERR_UNSUPPORTED;
    if (service_base_ns < 0 || service_per_frame_ns < 0) return HP_ERR_INVALID_ARG;
    for (int k = 1; k < n_frames; ++k)
        if (arrival_ns[k] < arrival_ns[k - 1]) return HP_ERR_INVALID_ARG;

    BatchPolicy pol(cfg->max_batch, cfg->depth, cfg->n_lanes);
    std::vector<std::vector<int>> members((size_t)cfg->n_lanes);   // frames of each lane's batch
    std::deque<int64_t> seen_q;     // completion time seen for each running batch, start order
    int64_t last_seen = 0, seq = 0;
    int64_t now = 0;
    auto start_all = [&](const std::vector<int> &start) {
        for (int l : start) {
            const int n = pol.frames(l);
            const int64_t fin = now + service_base_ns + (int64_t)n * service_per_frame_ns;
            last_seen = fin > last_seen ? fin : last_seen;
            seen_q.push_back(last_seen);
            for (int f : members[(size_t)l]) {
                batch_seq[f] = seq;
                batch_size[f] = n;
                done_ns[f] = last_seen;
            }
            ++seq;
        }
    };
    int next = 0;
    while (next < n_frames || pol.running() > 0 || pol.waiting() > 0 || pol.open_frames() > 0) {
        const bool have_arrival = next < n_frames;
        const bool have_done = !seen_q.empty();
        std::vector<int> start;
        // an arrival is handled first when it is not later than the next completion
        if (have_arrival && (!have_done || arrival_ns[next] <= seen_q.front())) {
            int lane, index;
            const int64_t t = arrival_ns[next] > now ? arrival_ns[next] : now;
            if (pol.acquire(lane, index)) {
                now = t;
                if (index == 0) members[(size_t)lane].clear();
                members[(size_t)lane].push_back(next);
                pol.commit(start);
                start_all(start);
                ++next;
                continue;
            }
            if (!have_done) return HP_ERR_STATE;   // cannot happen: a taken lane is running or waiting
        }
        if (have_done) {
            now = seen_q.front() > now ? seen_q.front() : now;
            seen_q.pop_front();
            pol.complete(start);
            int lane;
            while (pol.pop_done(lane)) pol.release(lane);
            start_all(start);
            continue;
        }
        // frames are left in the open batch and nothing runs: the stream has ended
        pol.flush(start);
        start_all(start);
    }
    return HP_OK;
}

int hp_batcher_drive(hp_batcher *b, int n_frames, int64_t interarrival_ns, int copy_frames, const void *cm_src,
                     const void *paf_src, int n_src, int64_t *latency_ns, int32_t *batch_size, int64_t *elapsed_ns)
{
    if (!b || n_frames <= 0 || interarrival_ns < 0) return HP_ERR_INVALID_ARG;
    if (copy_frames && (!cm_src || !paf_src || n_src <= 0)) return HP_ERR_INVALID_ARG;
    {
        std::unique_lock<std::mutex> lk(b->mu);
        if (!b->pol.idle() || b->pol.open_frames() > 0 || b->pol.pending()) return HP_ERR_STATE;
    }
    constexpr int kWaitMs = 20000;   // a batch of any built size finishes far sooner; bounds every wait
    std::atomic<int> target(n_frames);   // frames the consumer has to see; lowered when the producer fails
    int consumer_rc = HP_OK;
    int64_t last_done = 0;
    const int64_t t_start = b->now();
    std::thread consumer([&] {
        (void)hipSetDevice(b->device);
        std::vector<uint64_t> tags((size_t)b->max_batch);
        int got = 0, waited_ms = 0;
        while (got < target.load()) {
            hp_batch_info info;
            int rc = hp_batcher_next(b, 50, &info, tags.data(), nullptr);
            if (rc == HP_ERR_TIMEOUT && (waited_ms += 50) < kWaitMs) continue;
            if (rc != HP_OK) {
                consumer_rc = rc;
                return;
            }
            waited_ms = 0;
            if (info.rc != HP_OK) consumer_rc = info.rc;
            for (int k = 0; k < info.n_frames; ++k) {
                const uint64_t f = tags[(size_t)k];
                if (latency_ns) latency_ns[f] = info.done_ns - (t_start + (int64_t)f * interarrival_ns);
                if (batch_size) batch_size[f] = info.n_frames;
            }
            last_done = info.done_ns;
            got += info.n_frames;
            (void)hp_batcher_release(b, info.lane);
        }
    });
    int rc = HP_OK;
    int handed = 0;
    for (int k = 0; k < n_frames && rc == HP_OK; ++k) {
        const int64_t due = t_start + (int64_t)k * interarrival_ns;
        while (b->now() < due) {
        }
        if (copy_frames) {
            const size_t f = (size_t)(k % n_src);
            rc = hp_batcher_submit(b, kWaitMs, (const char *)cm_src + f * b->cm_frame_bytes,
                                   (const char *)paf_src + f * b->paf_frame_bytes, (uint64_t)k, nullptr, 1);
        } else {
            void *cm_slot, *paf_slot;
            rc = hp_batcher_acquire(b, kWaitMs, &cm_slot, &paf_slot);
            if (rc == HP_OK) rc = hp_batcher_commit(b, (uint64_t)k, nullptr, 1);
        }
        if (rc == HP_OK) ++handed;
    }
    target.store(handed);
    const int frc = hp_batcher_flush(b);
    if (rc == HP_OK) rc = frc;
    consumer.join();
    if (rc == HP_OK) rc = consumer_rc;
    if (elapsed_ns) *elapsed_ns = last_done - t_start;
    return rc;
}

}  // extern "C"
