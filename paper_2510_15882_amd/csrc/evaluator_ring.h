// The Evaluator's record ring (paper: Section "Stage 2: Runtime Fine-Grained
// Adjustment" - the Evaluator keeps per-path completion times of recent
// collective calls).  Every split call takes one record holding the events that
// bracket its paths; finished records are turned into per-path times, oldest
// first, without blocking the caller.
//
// The ring knows nothing about HIP: the event type and the three operations on
// it come in through `Api`, so the same code runs against the HIP runtime in
// the library and against a scripted clock in the host-only tests.
//
//   Api::query(ev)            0 = completed, 1 = not yet, anything else = error code
//   Api::wait(ev)             0 = completed, anything else = error code
//   Api::elapsed(a, b, &sec)  0 = ok (seconds from a to b), anything else = error code
//
// Error codes are passed through to the caller unchanged.
#ifndef FLEXLINK_EVALUATOR_RING_H
#define FLEXLINK_EVALUATOR_RING_H

#include <cstddef>
#include <cstdint>
#include <vector>

namespace flex {

constexpr int kRingMaxPaths = 4;

template <class Event>
struct TimingRecord {
    Event fork{};
    Event done[kRingMaxPaths]{};
    uint32_t used_mask = 0;   // bit p: path p carried part of the message
    int coll = 0;
    int size_class = 0;
    bool adaptive = false;
    uint64_t generation = 0;  // generation of the shares the call was split by
};

template <class Event, class Api>
class EvaluatorRing {
   public:
    using Record = TimingRecord<Event>;

    explicit EvaluatorRing(size_t capacity = 0) : ring_(capacity) {}
    void resize(size_t capacity) { ring_.assign(capacity, Record()); head_ = count_ = 0; }
    size_t capacity() const { return ring_.size(); }
    size_t in_flight() const { return count_; }
    uint64_t blocking_reads() const { return blocking_reads_; }
    std::vector<Record>& records() { return ring_; }

    // The record for a new split call.  With every record in flight the oldest
    // one is waited for first (counted in blocking_reads).  The caller fills in
    // the record and records its events; until it has done so successfully it
    // may give the record back with abandon().
    template <class Sink>
    int acquire(Api& api, Sink&& sink, Record** out) {
        if (count_ == ring_.size()) {
            ++blocking_reads_;
            bool popped = false;
            if (int st = pop_oldest(api, sink, true, &popped)) return st;
        }
        Record* rec = &ring_[(head_ + count_) % ring_.size()];
        rec->used_mask = 0;
        ++count_;
        *out = rec;
        return 0;
    }

    // Give back the record acquire() handed out last: the call it was meant for
    // failed part-way, so its events say nothing.
    void abandon() {
        if (count_ > 0) --count_;
    }

    // Read back finished records, oldest first; stop at the first unfinished one
    // (block = false) or wait for every record (block = true).  sink(record, T)
    // receives the per-path seconds (0 for paths the call did not use).
    template <class Sink>
    int poll(Api& api, Sink&& sink, bool block) {
        while (count_ > 0) {
            bool popped = false;
            if (int st = pop_oldest(api, sink, block, &popped)) return st;
            if (!popped) break;
        }
        return 0;
    }

   private:
    template <class Sink>
    int pop_oldest(Api& api, Sink&& sink, bool block, bool* popped) {
        Record& rec = ring_[head_];
        *popped = false;
        // the highest path's event is recorded last: test it first
        for (int p = kRingMaxPaths - 1; p >= 0; --p) {
            if (!(rec.used_mask & (1u << p))) continue;
            const int st = block ? api.wait(rec.done[p]) : api.query(rec.done[p]);
            if (!block && st == 1) return 0;  // still running
            if (st != 0) return st;
        }
        double T[kRingMaxPaths] = {0, 0, 0, 0};
        for (int p = 0; p < kRingMaxPaths; ++p) {
            if (!(rec.used_mask & (1u << p))) continue;
            if (int st = api.elapsed(rec.fork, rec.done[p], &T[p])) return st;
        }
        // the record leaves the ring before the sink runs: a sink that fails
        // must not see the same record again
        head_ = (head_ + 1) % ring_.size();
        --count_;
        *popped = true;
        sink(rec, T);
        return 0;
    }

    std::vector<Record> ring_;
    size_t head_ = 0, count_ = 0;
    uint64_t blocking_reads_ = 0;
};

}  // namespace flex

#endif
