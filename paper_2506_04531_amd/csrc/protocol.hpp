// Host-side protocol state of one local parameter server: the queue of
// arrived messages, the counters t / t_last and the life cycle of the
// accumulated update (HALoS Algorithm 1, LPS block; queue rule of Sec. 4.1
// item 2).  Pure C++, no device code: everything here is integers.
#pragma once

#include <cstddef>
#include <cstdint>
#include <deque>
#include <vector>

namespace halos {

enum Phase : int32_t {
    PHASE_ACCUMULATING = 0,   // collecting updates, nothing in flight
    PHASE_SENT = 1,           // frozen update waits for the global server
    PHASE_RETURNING = 2,      // global server applied it; its model is on the way back
    PHASE_QUEUED = 3          // that model sits in this server's queue
};

enum ItemKind : int32_t { ITEM_NONE = 0, ITEM_DELTA = 1, ITEM_GLOBAL = 2 };

enum ProtoResult : int32_t { PROTO_OK = 0, PROTO_BAD_ARG = 1, PROTO_BAD_STATE = 2 };

struct QueueItem {
    int32_t kind;
    int32_t worker;
};

struct UpdateOutcome {
    bool accumulate;     // this update is added to the accumulated update
    bool freezes;        // ... and it completes it (t - t_last reached K)
};

class LpsProtocol {
public:
    explicit LpsProtocol(int32_t n_workers, int32_t K)
        : K_(K), worker_queued_(n_workers, 0) {}

    int32_t n_workers() const { return (int32_t)worker_queued_.size(); }
    int64_t t() const { return t_; }
    int64_t t_last() const { return t_last_; }
    int32_t K() const { return K_; }
    int32_t phase() const { return phase_; }
    int32_t queued() const { return (int32_t)queue_.size(); }

    ProtoResult set_K(int32_t K) {
        if (K < 1) return PROTO_BAD_ARG;
        K_ = K;
        return PROTO_OK;
    }

    // A delta from `worker` arrives.
    ProtoResult can_push_delta(int32_t worker) const {
        if (worker < 0 || worker >= n_workers()) return PROTO_BAD_ARG;
        if (worker_queued_[worker]) return PROTO_BAD_STATE;
        return PROTO_OK;
    }
    void push_delta(int32_t worker) {
        worker_queued_[worker] = 1;
        queue_.push_back(QueueItem{ITEM_DELTA, worker});
    }

    // The global model arrives.
    ProtoResult can_push_global() const { return phase_ == PHASE_RETURNING ? PROTO_OK : PROTO_BAD_STATE; }
    void push_global() {
        phase_ = PHASE_QUEUED;
        queue_.push_back(QueueItem{ITEM_GLOBAL, -1});
    }

    // Head of the queue without removing it.
    QueueItem head() const { return queue_.empty() ? QueueItem{ITEM_NONE, -1} : queue_.front(); }

    // What applying the delta at the head will mean for the accumulated update (counter and send test of the LPS block).
    // The send test is "t - t_last >= K and nothing in flight": identical to the paper's
    // "t - t_last = K" whenever K changes only at merges, and it cannot be skipped over when a
    // caller lowers K in between.
    UpdateOutcome preview_update() const {
        UpdateOutcome o;
        o.accumulate = (phase_ == PHASE_ACCUMULATING);
        o.freezes = o.accumulate && (t_ + 1 - t_last_ >= K_);
        return o;
    }
    void commit_update() {
        UpdateOutcome o = preview_update();
        QueueItem it = queue_.front();
        queue_.pop_front();
        worker_queued_[it.worker] = 0;
        t_ += 1;
        if (o.freezes) phase_ = PHASE_SENT;
    }

    // An averaged step: the first `count` items (all deltas) become ONE update with their mean.
    bool head_is_deltas(int32_t count) const { return are_deltas(0, count); }
    // Are the `count` items from position `first` on all worker deltas?
    bool are_deltas(int32_t first, int32_t count) const {
        if (first < 0 || count < 1 || (std::size_t)first + (std::size_t)count > queue_.size()) return false;
        for (int32_t i = first; i < first + count; ++i) if (queue_[i].kind != ITEM_DELTA) return false;
        return true;
    }
    QueueItem item(int32_t i) const { return queue_[i]; }
    void commit_average(int32_t count) {
        UpdateOutcome o = preview_update();
        for (int32_t i = 0; i < count; ++i) {
            worker_queued_[queue_.front().worker] = 0;
            queue_.pop_front();
        }
        t_ += 1;
        if (o.freezes) phase_ = PHASE_SENT;
    }

    // The merge branch of the LPS block.
    void commit_merge() {
        queue_.pop_front();
        t_last_ = t_;
        phase_ = PHASE_ACCUMULATING;
    }

    // Global server consumed the frozen update (Alg. 1, GPS block).
    ProtoResult can_consume() const { return phase_ == PHASE_SENT ? PROTO_OK : PROTO_BAD_STATE; }
    void consume() { phase_ = PHASE_RETURNING; }

private:
    int64_t t_ = 0;
    int64_t t_last_ = 0;
    int32_t K_;
    int32_t phase_ = PHASE_ACCUMULATING;
    std::deque<QueueItem> queue_;
    std::vector<char> worker_queued_;
};

// Where a server stands in its cycle of d updates under delayed Nesterov momentum (Sec. 5.1; App. D, delays d_l
// and d_g): the first update of a cycle restarts the gradient buffer, the d-th refreshes the momentum.  d = 1 is
// the plain rule (every update refreshes; no buffer).
enum CyclePos : int32_t { POS_FIRST = 1, POS_INNER = 2, POS_REFRESH = 3 };

class MomentumCycle {
public:
    int32_t d() const { return d_; }
    int32_t seen() const { return seen_; }          // updates since the last refresh, 0 .. d-1

    // The delay may change only between cycles.
    ProtoResult set_d(int32_t d) {
        if (d < 1) return PROTO_BAD_ARG;
        if (seen_ != 0) return PROTO_BAD_STATE;
        d_ = d;
        return PROTO_OK;
    }

    // Position of the NEXT update.  For d = 1 it is a refresh that is also the first.
    CyclePos next() const {
        if (seen_ + 1 >= d_) return POS_REFRESH;
        return seen_ == 0 ? POS_FIRST : POS_INNER;
    }
    void commit() { seen_ = (seen_ + 1 >= d_) ? 0 : seen_ + 1; }

private:
    int32_t d_ = 1;
    int32_t seen_ = 0;
};

}  // namespace halos
