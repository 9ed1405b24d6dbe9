// The dynamic batch slot (Section 2.2.2 of the paper) as a host-side state machine, free of any
// GPU call so that the streaming front and the virtual-time simulation run the same decisions.
//
// Frames are collected in "lanes" (one batch each, with buffers and a stream of their own):
//   free -> open (collecting frames) -> [full, waiting for the GPU] -> running -> done -> held -> free
// At most `depth` batches run at once.  A frame that arrives while fewer than `depth` run closes
// the open batch at once, so the batch stays small while the GPU keeps up; while `depth` are
// running the open batch keeps collecting, up to max_batch frames, and is taken as soon as a
// running batch completes.  Batches start and are handed out in the order their first frame came.
#pragma once

#include <deque>
#include <vector>

namespace hp {

class BatchPolicy {
public:
    enum State : int { kFree = 0, kOpen, kFull, kRunning, kDone, kHeld };

    BatchPolicy(int max_batch, int depth, int n_lanes)
        : max_batch_(max_batch), depth_(depth), state_((size_t)n_lanes, kFree), count_((size_t)n_lanes, 0)
    {
    }

    // Place of the next frame (lane, index in its batch).  False when every lane is taken.
    bool acquire(int &lane, int &index)
    {
        if (pending_) return false;
        if (open_ < 0) {
            for (size_t l = 0; l < state_.size(); ++l)
                if (state_[l] == kFree) {
                    open_ = (int)l;
                    break;
                }
            if (open_ < 0) return false;
            state_[(size_t)open_] = kOpen;
            count_[(size_t)open_] = 0;
        }
        pending_ = true;
        lane = open_;
        index = count_[(size_t)open_];
        return true;
    }

    // Gives an acquired place back unused.
    void cancel()
    {
        if (!pending_) return;
        pending_ = false;
        if (count_[(size_t)open_] == 0) {
            state_[(size_t)open_] = kFree;
            open_ = -1;
        }
    }

    // The acquired frame is in place.  Lanes to start now are appended to `start`, in order.
    bool commit(std::vector<int> &start)
    {
        if (!pending_) return false;
        pending_ = false;
        ++count_[(size_t)open_];
        schedule(start);
        if (open_ >= 0 && count_[(size_t)open_] == max_batch_) close_open();
        return true;
    }

    // Closes the open batch whatever its size; it starts as soon as fewer than `depth` run.
    bool flush(std::vector<int> &start)
    {
        if (pending_) return false;
        if (open_ >= 0 && count_[(size_t)open_] > 0) close_open();
        schedule(start);
        return true;
    }

    // The oldest running batch has finished.
    bool complete(std::vector<int> &start)
    {
        if (run_q_.empty()) return false;
        const int lane = run_q_.front();
        run_q_.pop_front();
        state_[(size_t)lane] = kDone;
        done_q_.push_back(lane);
        schedule(start);
        return true;
    }

    // Hands out the oldest finished batch; the caller holds its lane until release().
    bool pop_done(int &lane)
    {
        if (done_q_.empty()) return false;
        lane = done_q_.front();
        done_q_.pop_front();
        state_[(size_t)lane] = kHeld;
        return true;
    }

    bool release(int lane)
    {
        if (lane < 0 || (size_t)lane >= state_.size() || state_[(size_t)lane] != kHeld) return false;
        state_[(size_t)lane] = kFree;
        count_[(size_t)lane] = 0;
        return true;
    }

    int oldest_running() const { return run_q_.empty() ? -1 : run_q_.front(); }
    int running() const { return (int)run_q_.size(); }
    int waiting() const { return (int)full_q_.size(); }
    int finished() const { return (int)done_q_.size(); }
    int open_frames() const { return open_ >= 0 ? count_[(size_t)open_] : 0; }
    bool pending() const { return pending_; }
    int frames(int lane) const { return count_[(size_t)lane]; }
    State state(int lane) const { return state_[(size_t)lane]; }
    int lanes() const { return (int)state_.size(); }
    int max_batch() const { return max_batch_; }
    // true when no call but acquire/commit can make a batch finish
    bool idle() const { return run_q_.empty() && full_q_.empty() && done_q_.empty(); }

private:
    void close_open()
    {
        state_[(size_t)open_] = kFull;
        full_q_.push_back(open_);
        open_ = -1;
    }

    void schedule(std::vector<int> &start)
    {
        while ((int)run_q_.size() < depth_) {
            int lane;
            if (!full_q_.empty()) {
                lane = full_q_.front();
                full_q_.pop_front();
            } else if (open_ >= 0 && count_[(size_t)open_] > 0 && !pending_) {
                lane = open_;
                open_ = -1;
            } else {
                break;
            }
            state_[(size_t)lane] = kRunning;
            run_q_.push_back(lane);
            start.push_back(lane);
        }
    }

    int max_batch_, depth_;
    std::vector<State> state_;
    std::vector<int> count_;
    int open_ = -1;
    bool pending_ = false;
    std::deque<int> full_q_, run_q_, done_q_;
};

}  // namespace hp
