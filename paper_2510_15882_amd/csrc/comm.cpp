// Communicator: partitions each collective over the device path and one or two
// host-staged paths, runs them concurrently (fork/join by events), and feeds the
// per-path completion times back to the balancer (the paper's Evaluator).
// Paper: Design; Section "Communicator"; Section "Two-Stage Load Balancing
// Strategy".
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <new>
#include <vector>

#include "evaluator_ring.h"
#include "flexlink_internal.h"

namespace flex {

static thread_local char g_last_error[512] = "";

int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
    return status;
}

}  // namespace flex

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return flex::fail(FLEX_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));    \
    } while (0)

#define LAUNCH_TRY(expr)                                                                       \
    do {                                                                                       \
        int e_ = (expr);                                                                       \
        if (e_ != 0)                                                                           \
            return flex::fail(FLEX_ERR_HIP, "kernel launch failed: %s",                        \
                              hipGetErrorString((hipError_t)e_));                              \
    } while (0)

namespace {

constexpr size_t kRingSize = 256;    // timing records that may be in flight
constexpr size_t kMaxTuneRounds = 128;  // iterations of Algorithm 1 kept for flex_comm_tune_trace
constexpr int kMaxAux = FLEX_MAX_PATHS - 1;

// The Evaluator's three event operations on the HIP runtime.
struct HipEventApi {
    int query(hipEvent_t e) {
        hipError_t q = hipEventQuery(e);
        if (q == hipSuccess) return 0;
        if (q == hipErrorNotReady) return 1;
        return flex::fail(FLEX_ERR_HIP, "hipEventQuery failed: %s", hipGetErrorString(q));
    }
    int wait(hipEvent_t e) {
        hipError_t q = hipEventSynchronize(e);
        return q == hipSuccess ? 0 : flex::fail(FLEX_ERR_HIP, "hipEventSynchronize failed: %s", hipGetErrorString(q));
    }
    int elapsed(hipEvent_t a, hipEvent_t b, double* seconds) {
        float ms = 0.f;
        hipError_t q = hipEventElapsedTime(&ms, a, b);
        if (q != hipSuccess) return flex::fail(FLEX_ERR_HIP, "hipEventElapsedTime failed: %s", hipGetErrorString(q));
        *seconds = ms * 1e-3;
        return 0;
    }
};
using Ring = flex::EvaluatorRing<hipEvent_t, HipEventApi>;
using TimingRecord = Ring::Record;

struct SizeClass {
    flex::Balancer bal;
    bool tuned = false;       // produced by flex_comm_tune / flex_comm_set_shares (else borrowed)
    uint64_t generation = 0;  // bumped whenever the shares change
    std::vector<flex_tune_round_t> rounds;  // Algorithm 1 as flex_comm_tune ran it
    uint32_t rounds_run = 0;
};

struct CollState {
    uint32_t mode = FLEX_SPLIT_STATIC;
    uint32_t static_units[FLEX_MAX_PATHS] = {0, 0, 0, 0};  // [0] unused
    std::map<int, SizeClass> classes;
    uint64_t calls = 0, split_calls = 0, samples = 0;
    uint64_t last_count = 0;
    uint64_t last_start[FLEX_MAX_PATHS + 1] = {0, 0, 0, 0, 0};
    double last_t[FLEX_MAX_PATHS] = {0, 0, 0, 0};
    double sum_t[FLEX_MAX_PATHS] = {0, 0, 0, 0};
};

int size_class_of(size_t bytes) {
    int c = 0;
    while (bytes > 1) {
        bytes >>= 1;
        ++c;
    }
    return c;
}

double median_of(std::vector<double> v) {
    if (v.empty()) return 0.0;
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return (n & 1) ? v[n / 2] : (v[n / 2 - 1] + v[n / 2]) / 2.0;
}

// median absolute deviation
double mad_of(const std::vector<double>& v) {
    const double m = median_of(v);
    std::vector<double> d;
    for (double x : v) d.push_back(std::fabs(x - m));
    return median_of(d);
}

// What the consumer stage of a host path does with a step once it sits in the
// pinned slot.
struct HostJob {
    int npeers = 0;
    const char* peer_src[FLEX_MAX_RANKS];  // start of each peer's part (device memory)
    // AllGather: where each peer's part goes.  DMA-engine reduce: device scratch.
    char* peer_dst[FLEX_MAX_RANKS];
    // reduce in rank order into out_part; the local rank's part is read in place
    bool reduce = false;
    int dtype = 0;
    int nranks = 0;
    int local_index = 0;  // position of the local rank among the nranks inputs
    const char* local_src = nullptr;
    char* out_part = nullptr;
};

// One host-staged path: a ring of pinned slots, a producer and a consumer
// stream (plus, for the hybrid engine, a third one for the kernels that finish
// a step out of the device staging buffers), and the slot hand-over state.
struct HostPath {
    int engine = FLEX_ENGINE_HYBRID;
    hipStream_t s_up = nullptr, s_down = nullptr, s_fin = nullptr;
    std::vector<void*> pinned;
    std::vector<hipEvent_t> ev_full, ev_empty;
    // hybrid engine: one device staging buffer per slot, filled by the DMA
    // engine and drained by a kernel on s_fin
    std::vector<char*> stage;
    std::vector<hipEvent_t> ev_staged, ev_stage_free;
    // FLEX_SYNC_COUNTERS: one pair of 64-bit counters per slot (signal memory) and
    // how often each slot has been used so far
    std::vector<uint64_t*> sem_full, sem_empty;
    std::vector<uint64_t> slot_uses;
    // hybrid engine with event hand-over: one in-order stream ("lane") per
    // slot that runs a step from start to end - copy kernel, DMA copy, finishing
    // kernel - so that no DMA copy ever has a cross-stream wait or another DMA
    // copy in front of it (either costs tens of microseconds of hand-off on this
    // runtime, a kernel in front of it does not)
    std::vector<hipStream_t> lane;
    std::vector<hipEvent_t> ev_up, ev_end;
    hipStream_t tail = nullptr;  // stream the last call's final step ended on

    uint64_t chunk_seq = 0;  // steps staged since creation; slot = seq % num_slots
    char* scratch = nullptr;  // DMA engine, reductions only: one stripe per peer
    size_t scratch_stride = 0;

    bool lanes() const { return !lane.empty(); }
    hipStream_t last_stream() const { return lanes() ? tail : engine == FLEX_ENGINE_HYBRID ? s_fin : s_down; }

    void quiesce() {
        for (hipStream_t st : {s_up, s_down, s_fin})
            if (st) (void)hipStreamSynchronize(st);
        for (hipStream_t st : lane) (void)hipStreamSynchronize(st);
    }

    void destroy() {
        quiesce();
        for (auto* vec : {&ev_full, &ev_empty, &ev_staged, &ev_stage_free, &ev_up, &ev_end})
            for (auto e : *vec) (void)hipEventDestroy(e);
        for (auto p : sem_full) (void)hipFree(p);
        for (auto p : sem_empty) (void)hipFree(p);
        for (auto p : pinned) (void)hipHostFree(p);
        for (auto p : stage) (void)hipFree(p);
        if (scratch) (void)hipFree(scratch);
        for (hipStream_t st : {s_up, s_down, s_fin})
            if (st) (void)hipStreamDestroy(st);
        for (hipStream_t st : lane) (void)hipStreamDestroy(st);
        *this = HostPath();
    }
};

}  // namespace

struct flex_comm {
    int device = 0;
    int nranks = 0, rank = 0;
    size_t max_bytes = 0;
    flex_config_t cfg;
    flex::LaunchShape reduce_shape, copy_shape;            // device path
    // kernels that touch pinned memory: few workgroups (producer copy, consumer reduce, consumer copy)
    flex::LaunchShape link_reduce_shape, link_copy_shape, link_down_copy_shape;
    flex::LaunchShape stage_reduce_shape, stage_copy_shape;  // hybrid engine: kernels that drain a staging buffer

    int naux = 0;  // auxiliary (host-staged) paths: path index 1 + a
    HostPath aux[kMaxAux];
    int npaths() const { return 1 + naux; }

    Ring ring;
    HipEventApi events;
    // split calls the Evaluator does not sample are forked and joined with
    // ordering-only events (a timing event costs about 2 us of stream time)
    hipEvent_t fork_untimed = nullptr;
    hipEvent_t join_untimed[kMaxAux] = {nullptr, nullptr, nullptr};
    uint64_t split_seq = 0;  // split calls issued so far, all collectives
    hipEvent_t t0 = nullptr, t1 = nullptr;  // whole-call timing in flex_comm_tune

    CollState coll[4];  // indexed by flex_coll

    // ---- host-staged path --------------------------------------------------
    // Move `bytes` bytes per peer through the path's ring of pinned slots, step
    // by step: producer stage (device -> pinned slot) on s_up, consumer stage
    // (pinned slot -> device) on s_down.  A slot is refilled only after the
    // consumer that drained it and drained only after the producer that filled
    // it, so the producer of one step overlaps the consumer of the previous one:
    // PCIe carries both directions at once.  The slot of a step is its sequence
    // number modulo the ring size, counted since the communicator was created.
    // In a slot the peers' pieces lie back to back (stride = the step's size
    // rounded up to 256 bytes), so the hybrid engine brings a whole step back
    // with one DMA copy.
    int host_path(HostPath& hp, const HostJob& job, size_t bytes, hipEvent_t fork) {
        if (hp.lanes()) return host_path_lanes(hp, job, bytes, fork);
        HIP_TRY(hipStreamWaitEvent(hp.s_up, fork, 0));
        const size_t nslots = hp.pinned.size();
        const size_t es = job.reduce ? flex::dtype_size(job.dtype) : 1;
        const std::vector<uint64_t> steps = flex::plan_steps(bytes, cfg.chunk_bytes, cfg.min_step_bytes);
        const int engine = hp.engine;
        const bool counters = cfg.slot_sync == FLEX_SYNC_COUNTERS;

        size_t off = 0;
        for (const uint64_t n : steps) {
            const size_t slot = hp.chunk_seq % nslots;
            const bool reused = hp.chunk_seq >= nslots;
            const size_t stride = (n + 255) / 256 * 256;
            char* base = (char*)hp.pinned[slot];
            const void* up_src[FLEX_MAX_RANKS];
            void* up_dst[FLEX_MAX_RANKS];
            uint64_t nn[FLEX_MAX_RANKS];
            for (int j = 0; j < job.npeers; ++j) {
                up_src[j] = job.peer_src[j] + off;
                up_dst[j] = base + (size_t)j * stride;
                nn[j] = n;
            }
            const uint64_t use = counters ? hp.slot_uses[slot] : 0;  // this is use number `use` of the slot

            // producer stage: the slot must have been drained by its previous use
            if (counters) {
                if (use > 0)
                    HIP_TRY(hipStreamWaitValue64(hp.s_up, hp.sem_empty[slot], use, hipStreamWaitValueGte,
                                                 ~0ull));
            } else if (reused) {
                HIP_TRY(hipStreamWaitEvent(hp.s_up, hp.ev_empty[slot], 0));
            }
            if (engine == FLEX_ENGINE_SDMA) {
                for (int j = 0; j < job.npeers; ++j)
                    HIP_TRY(hipMemcpyAsync(up_dst[j], up_src[j], n, hipMemcpyDeviceToHost, hp.s_up));
            } else {
                LAUNCH_TRY(flex::launch_gather_copy(up_src, up_dst, nn, job.npeers, link_copy_shape, hp.s_up));
            }
            // hand the filled slot over to the consumer stage
            if (counters) {
                HIP_TRY(hipStreamWriteValue64(hp.s_up, hp.sem_full[slot], use + 1, 0));
                HIP_TRY(hipStreamWaitValue64(hp.s_down, hp.sem_full[slot], use + 1, hipStreamWaitValueGte,
                                             ~0ull));
            } else {
                HIP_TRY(hipEventRecord(hp.ev_full[slot], hp.s_up));
                HIP_TRY(hipStreamWaitEvent(hp.s_down, hp.ev_full[slot], 0));
            }

            // consumer stage
            if (engine == FLEX_ENGINE_HYBRID) {
                // one DMA copy brings the step into the slot's staging buffer ...
                char* stage = hp.stage[slot];
                if (reused) HIP_TRY(hipStreamWaitEvent(hp.s_down, hp.ev_stage_free[slot], 0));
                HIP_TRY(hipMemcpyAsync(stage, base, (size_t)(job.npeers - 1) * stride + n, hipMemcpyHostToDevice,
                                       hp.s_down));
                HIP_TRY(hipEventRecord(hp.ev_staged[slot], hp.s_down));
                // ... and a kernel on the third stream finishes the step from there
                HIP_TRY(hipStreamWaitEvent(hp.s_fin, hp.ev_staged[slot], 0));
                if (job.reduce) {
                    const void* in[FLEX_MAX_RANKS];
                    int j = 0;
                    for (int r = 0; r < job.nranks; ++r)
                        in[r] = (r == job.local_index) ? (const void*)(job.local_src + off)
                                                       : (const void*)(stage + (size_t)(j++) * stride);
                    LAUNCH_TRY(flex::launch_reduce_n(in, job.nranks, job.out_part + off, n / es, job.dtype,
                                                     stage_reduce_shape, hp.s_fin));
                } else {
                    const void* dn_src[FLEX_MAX_RANKS];
                    void* dn_dst[FLEX_MAX_RANKS];
                    for (int j = 0; j < job.npeers; ++j) {
                        dn_src[j] = stage + (size_t)j * stride;
                        dn_dst[j] = job.peer_dst[j] + off;
                    }
                    LAUNCH_TRY(flex::launch_gather_copy(dn_src, dn_dst, nn, job.npeers, stage_copy_shape, hp.s_fin));
                }
                HIP_TRY(hipEventRecord(hp.ev_stage_free[slot], hp.s_fin));
            } else if (engine == FLEX_ENGINE_KERNEL && job.reduce) {
                // the reduce kernel reads the peers straight from the pinned slot
                const void* in[FLEX_MAX_RANKS];
                int j = 0;
                for (int r = 0; r < job.nranks; ++r)
                    in[r] = (r == job.local_index) ? (const void*)(job.local_src + off) : up_dst[j++];
                LAUNCH_TRY(flex::launch_reduce_n(in, job.nranks, job.out_part + off, n / es, job.dtype,
                                                 link_reduce_shape, hp.s_down));
            } else if (engine == FLEX_ENGINE_KERNEL) {
                const void* dn_src[FLEX_MAX_RANKS];
                void* dn_dst[FLEX_MAX_RANKS];
                for (int j = 0; j < job.npeers; ++j) {
                    dn_src[j] = up_dst[j];
                    dn_dst[j] = job.peer_dst[j] + off;
                }
                LAUNCH_TRY(flex::launch_gather_copy(dn_src, dn_dst, nn, job.npeers, link_down_copy_shape, hp.s_down));
            } else {
                for (int j = 0; j < job.npeers; ++j)
                    HIP_TRY(hipMemcpyAsync(job.peer_dst[j] + off, up_dst[j], n, hipMemcpyHostToDevice, hp.s_down));
            }
            // the pinned slot is free again once s_down's part of the step is done
            if (counters) {
                HIP_TRY(hipStreamWriteValue64(hp.s_down, hp.sem_empty[slot], use + 1, 0));
                hp.slot_uses[slot] = use + 1;
            } else {
                HIP_TRY(hipEventRecord(hp.ev_empty[slot], hp.s_down));
            }
            ++hp.chunk_seq;
            off += n;
        }
        if (engine == FLEX_ENGINE_SDMA && job.reduce) {
            // DMA engine: the peers' parts now sit in device scratch (peer_dst)
            const void* in[FLEX_MAX_RANKS];
            int j = 0;
            for (int r = 0; r < job.nranks; ++r)
                in[r] = (r == job.local_index) ? (const void*)job.local_src : (const void*)job.peer_dst[j++];
            LAUNCH_TRY(flex::launch_reduce_n(in, job.nranks, job.out_part, bytes / es, job.dtype, reduce_shape,
                                             hp.s_down));
        }
        return FLEX_OK;
    }

    // The same for the hybrid engine with event hand-over.  Step k runs from
    // start to end on lane k mod L, an in-order stream with its own pinned slot
    // and staging buffer: copy kernel (device -> pinned slot), DMA copy (pinned
    // slot -> staging buffer), finishing kernel (reduce, or place the pieces).
    // Stream order alone protects the slot and the staging buffer.  The copy
    // kernels of successive steps are chained by events, so that they follow one
    // another on the upstream direction of the link while the DMA copies of
    // earlier steps occupy the downstream one; with three lanes the hand-off
    // between a DMA copy and the kernel behind it is hidden as well.
    int host_path_lanes(HostPath& hp, const HostJob& job, size_t bytes, hipEvent_t fork) {
        const size_t L = hp.lane.size();
        const size_t es = job.reduce ? flex::dtype_size(job.dtype) : 1;
        const std::vector<uint64_t> steps = flex::plan_steps(bytes, cfg.chunk_bytes, cfg.min_step_bytes);
        if (steps.empty()) {
            hp.tail = hp.lane[0];
            HIP_TRY(hipStreamWaitEvent(hp.tail, fork, 0));
            return FLEX_OK;
        }
        bool used[64] = {false};
        size_t off = 0, prev = L;  // prev: lane of the step before (L = none yet)
        for (const uint64_t n : steps) {
            const size_t l = hp.chunk_seq % L;
            hipStream_t st = hp.lane[l];
            const size_t stride = (n + 255) / 256 * 256;
            char* base = (char*)hp.pinned[l];
            char* stage = hp.stage[l];
            if (!used[l]) {
                HIP_TRY(hipStreamWaitEvent(st, fork, 0));
                used[l] = true;
            }
            if (prev != L && prev != l) HIP_TRY(hipStreamWaitEvent(st, hp.ev_up[prev], 0));
            const void* up_src[FLEX_MAX_RANKS];
            void* up_dst[FLEX_MAX_RANKS];
            uint64_t nn[FLEX_MAX_RANKS];
            for (int j = 0; j < job.npeers; ++j) {
                up_src[j] = job.peer_src[j] + off;
                up_dst[j] = base + (size_t)j * stride;
                nn[j] = n;
            }
            LAUNCH_TRY(flex::launch_gather_copy(up_src, up_dst, nn, job.npeers, link_copy_shape, st));
            HIP_TRY(hipEventRecord(hp.ev_up[l], st));
            HIP_TRY(hipMemcpyAsync(stage, base, (size_t)(job.npeers - 1) * stride + n, hipMemcpyHostToDevice, st));
            if (job.reduce) {
                const void* in[FLEX_MAX_RANKS];
                int j = 0;
                for (int r = 0; r < job.nranks; ++r)
                    in[r] = (r == job.local_index) ? (const void*)(job.local_src + off)
                                                   : (const void*)(stage + (size_t)(j++) * stride);
                LAUNCH_TRY(flex::launch_reduce_n(in, job.nranks, job.out_part + off, n / es, job.dtype,
                                                 stage_reduce_shape, st));
            } else {
                const void* dn_src[FLEX_MAX_RANKS];
                void* dn_dst[FLEX_MAX_RANKS];
                for (int j = 0; j < job.npeers; ++j) {
                    dn_src[j] = stage + (size_t)j * stride;
                    dn_dst[j] = job.peer_dst[j] + off;
                }
                LAUNCH_TRY(flex::launch_gather_copy(dn_src, dn_dst, nn, job.npeers, stage_copy_shape, st));
            }
            prev = l;
            ++hp.chunk_seq;
            off += n;
        }
        // the lane of the last step collects the others: the path is done when it is
        hp.tail = hp.lane[prev];
        for (size_t l = 0; l < L; ++l) {
            if (!used[l] || l == prev) continue;
            HIP_TRY(hipEventRecord(hp.ev_end[l], hp.lane[l]));
            HIP_TRY(hipStreamWaitEvent(hp.tail, hp.ev_end[l], 0));
        }
        return FLEX_OK;
    }

    // ---- Evaluator ---------------------------------------------------------
    SizeClass* find_class(int c, int size_class) {
        auto& m = coll[c].classes;
        auto it = m.find(size_class);
        return it == m.end() ? nullptr : &it->second;
    }

    // Size class for an adaptive call: its own, else a copy of the nearest
    // tuned one of the same collective, else none.
    SizeClass* class_for_call(int c, int size_class) {
        if (SizeClass* sc = find_class(c, size_class)) return sc;
        auto& m = coll[c].classes;
        const SizeClass* best = nullptr;
        int best_d = 0;
        for (auto& kv : m) {
            if (!kv.second.tuned) continue;
            int d = std::abs(kv.first - size_class);
            if (!best || d < best_d) {
                best = &kv.second;
                best_d = d;
            }
        }
        if (!best) return nullptr;
        SizeClass fresh;
        fresh.bal = best->bal;
        fresh.bal.finish_tuning();
        fresh.bal.window.clear();
        fresh.tuned = false;
        return &(m[size_class] = fresh);
    }

    // One finished split call: book its per-path times and, in adaptive mode,
    // hand them to the size class's balancer (Stage 2).
    void consume(const TimingRecord& rec, const double* T) {
        CollState& cs = coll[rec.coll];
        ++cs.samples;
        for (int p = 0; p < FLEX_MAX_PATHS; ++p) {
            cs.last_t[p] = T[p];
            cs.sum_t[p] += T[p];
        }
        if (rec.adaptive && cs.mode == FLEX_SPLIT_ADAPTIVE) {
            SizeClass* sc = find_class(rec.coll, rec.size_class);
            // a call issued before the last share change says nothing about the new shares
            if (sc && sc->generation == rec.generation && sc->bal.stage == FLEX_STAGE_RUNTIME) {
                uint32_t before[FLEX_MAX_PATHS];
                memcpy(before, sc->bal.shares, sizeof before);
                if (sc->bal.update(T) && memcmp(before, sc->bal.shares, sizeof before) != 0) ++sc->generation;
            }
        }
    }

    int poll(bool block) {
        return ring.poll(events, [this](const TimingRecord& rec, const double* T) { consume(rec, T); }, block);
    }

    // Evaluator poll in front of a collective call: event queries are not
    // allowed while the caller's stream is being captured, so records wait.
    int poll_before_call(hipStream_t stream) {
        if (ring.in_flight() == 0) return FLEX_OK;
        hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
        HIP_TRY(hipStreamIsCapturing(stream, &capture));
        return capture == hipStreamCaptureStatusNone ? poll(false) : FLEX_OK;
    }

    // Share, in units, that each auxiliary path of a call of `bytes` per rank
    // uses now (units[0] is not used), and the generation of those shares.
    void units_for_call(int c, size_t bytes, uint32_t* units, bool* adaptive, uint64_t* generation) {
        CollState& cs = coll[c];
        *adaptive = false;
        *generation = 0;
        for (int p = 0; p < FLEX_MAX_PATHS; ++p) units[p] = 0;
        if (nranks < 2) return;
        if (cs.mode == FLEX_SPLIT_STATIC) {
            for (int p = 1; p < npaths(); ++p) units[p] = cs.static_units[p];
            return;
        }
        SizeClass* sc = class_for_call(c, size_class_of(bytes));
        if (!sc || sc->bal.npaths < 2) return;
        *adaptive = true;
        *generation = sc->generation;
        for (int p = 1; p < npaths() && p < sc->bal.npaths; ++p)
            units[p] = std::min(sc->bal.shares[p], cfg.max_host_units);
    }

    int check_device() const {
        int cur = -1;
        HIP_TRY(hipGetDevice(&cur));
        if (cur != device)
            return flex::fail(FLEX_ERR_STATE, "communicator belongs to device %d, current device is %d",
                              device, cur);
        return FLEX_OK;
    }

    // Segment starts of a call: path p carries elements [start[p], start[p+1]).
    bool split_message(int c, size_t count, size_t es, uint64_t* start, bool* adaptive, uint64_t* generation) {
        uint32_t units[FLEX_MAX_PATHS];
        units_for_call(c, count * es, units, adaptive, generation);
        flex::partition_paths(count, units, npaths(), cfg.balancer.share_total, cfg.split_align_elems,
                              cfg.min_split_bytes / es, start);
        for (int p = npaths(); p < FLEX_MAX_PATHS; ++p) start[p + 1] = count;
        CollState& cs = coll[c];
        cs.last_count = count;
        for (int p = 0; p <= FLEX_MAX_PATHS; ++p) cs.last_start[p] = start[p];
        return start[1] < count;  // some auxiliary path carries data
    }

    // A split call records timing events that the Evaluator reads back with
    // the host clock running; inside a stream capture they would never fire.
    int begin_split_call(int c, size_t bytes, bool adaptive, uint64_t generation, hipStream_t stream,
                         TimingRecord** rec_out) {
        hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
        HIP_TRY(hipStreamIsCapturing(stream, &capture));
        if (capture != hipStreamCaptureStatusNone)
            return flex::fail(FLEX_ERR_STATE,
                              "a call that uses a host path cannot be captured into a graph: set the host "
                              "share to 0 for captured calls");
        *rec_out = nullptr;
        if (split_seq++ % cfg.sample_every != 0) {  // not sampled: no record, no timing events
            ++coll[c].split_calls;
            return FLEX_OK;
        }
        TimingRecord* rec;
        int st = ring.acquire(events, [this](const TimingRecord& r, const double* T) { consume(r, T); }, &rec);
        if (st) return st;
        ++coll[c].split_calls;
        rec->coll = c;
        rec->size_class = size_class_of(bytes);
        rec->adaptive = adaptive;
        rec->generation = generation;
        *rec_out = rec;
        return FLEX_OK;
    }

    // A split call failed after begin_split_call: its record's events say
    // nothing, so the record goes back; whatever the call did enqueue on the
    // side streams is waited for, so that nothing of it still runs on the
    // caller's buffers when the error is returned.
    int abandon_split_call(int c, bool sampled, int status) {
        if (sampled) ring.abandon();
        --coll[c].split_calls;
        for (int a = 0; a < naux; ++a) aux[a].quiesce();
        return status;
    }

    // AllReduce, or (c == FLEX_REDUCESCATTER) the same reduction over the
    // local rank's slice of every input
    int reduce(int c, const char* who, const void* const* bufs, void* out, size_t count, int dtype,
               hipStream_t stream);
    int split_reduce(TimingRecord* rec, const uint64_t* start, const void* const* bufs, void* out, int dtype,
                     hipStream_t stream);
    int reducescatter(const void* const* bufs, void* out, size_t recv_count, int dtype, hipStream_t stream);
    // AllGather, or (c == FLEX_ALLTOALL) the same gather over the pieces the
    // peers address to the local rank
    int gather(int c, const char* who, const void* const* slices, void* out, size_t count, int dtype,
               hipStream_t stream);
    int split_gather(TimingRecord* rec, const uint64_t* start, const void* const* src, void* const* dst,
                     const uint64_t* bytes, const void* const* slices, size_t es, hipStream_t stream);
    int alltoall(const void* const* bufs, void* out, size_t count, int dtype, hipStream_t stream);
    int collective(int c, const void* const* bufs, void* out, size_t count, int dtype, hipStream_t stream) {
        if (c == FLEX_REDUCESCATTER) return reducescatter(bufs, out, count, dtype, stream);
        if (c == FLEX_ALLTOALL) return alltoall(bufs, out, count, dtype, stream);
        return c == FLEX_ALLREDUCE ? reduce(c, "flex_allreduce_local", bufs, out, count, dtype, stream)
                                   : gather(c, "flex_allgather_local", bufs, out, count, dtype, stream);
    }
    int validate(const char* who, const void* const* bufs, const void* out, size_t count, int dtype);
    int measure_split(int c, const void* const* bufs, void* out, size_t count, int dtype,
                      hipStream_t stream, const uint32_t* units, double* T);
    int time_calls(int c, const void* const* bufs, void* out, size_t count, int dtype, hipStream_t stream,
                   const uint32_t* units, uint32_t reps, bool warm, std::vector<double>* seconds);
};

int flex_comm::validate(const char* who, const void* const* bufs, const void* out, size_t count,
                        int dtype) {
    const size_t es = flex::dtype_size(dtype);
    if (es == 0) return flex::fail(FLEX_ERR_UNSUPPORTED, "%s: unknown dtype %d", who, dtype);
    if (!bufs) return flex::fail(FLEX_ERR_INVALID_ARG, "%s: rank pointer array is NULL", who);
    if (count > max_bytes / es)
        return flex::fail(FLEX_ERR_INVALID_ARG, "%s: %zu elements exceed max_bytes_per_rank %zu", who,
                          count, max_bytes);
    if (count == 0) return FLEX_OK;
    if (!out) return flex::fail(FLEX_ERR_INVALID_ARG, "%s: out is NULL", who);
    if ((uintptr_t)out % es)
        return flex::fail(FLEX_ERR_INVALID_ARG, "%s: out is not aligned to the element size", who);
    for (int r = 0; r < nranks; ++r) {
        if (!bufs[r]) return flex::fail(FLEX_ERR_INVALID_ARG, "%s: rank %d pointer is NULL", who, r);
        if ((uintptr_t)bufs[r] % es)
            return flex::fail(FLEX_ERR_INVALID_ARG, "%s: rank %d pointer is not aligned to the element size",
                              who, r);
    }
    return check_device();
}

int flex_comm::reducescatter(const void* const* bufs, void* out, size_t recv_count, int dtype,
                             hipStream_t stream) {
    const size_t es = flex::dtype_size(dtype);
    if (es == 0) return flex::fail(FLEX_ERR_UNSUPPORTED, "flex_reducescatter_local: unknown dtype %d", dtype);
    if (!bufs) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_reducescatter_local: rank pointer array is NULL");
    if (recv_count > max_bytes / es / (size_t)nranks)
        return flex::fail(FLEX_ERR_INVALID_ARG,
                          "flex_reducescatter_local: %d x %zu elements exceed max_bytes_per_rank %zu", nranks,
                          recv_count, max_bytes);
    // rank r's slice of every contribution starts rank * recv_count elements in
    const void* slice[FLEX_MAX_RANKS];
    for (int r = 0; r < nranks; ++r) {
        if (recv_count > 0 && !bufs[r])
            return flex::fail(FLEX_ERR_INVALID_ARG, "flex_reducescatter_local: rank %d pointer is NULL", r);
        slice[r] = (const char*)bufs[r] + (size_t)rank * recv_count * es;
    }
    return reduce(FLEX_REDUCESCATTER, "flex_reducescatter_local", slice, out, recv_count, dtype, stream);
}

int flex_comm::reduce(int c, const char* who, const void* const* bufs, void* out, size_t count, int dtype,
                      hipStream_t stream) {
    int st = validate(who, bufs, out, count, dtype);
    if (st) return st;
    CollState& cs = coll[c];
    ++cs.calls;
    if (count == 0) return FLEX_OK;
    st = poll_before_call(stream);
    if (st) return st;

    const size_t es = flex::dtype_size(dtype);
    uint64_t start[FLEX_MAX_PATHS + 1];
    bool adaptive;
    uint64_t generation;
    if (!split_message(c, count, es, start, &adaptive, &generation)) {
        LAUNCH_TRY(flex::launch_reduce_n(bufs, nranks, out, count, dtype, reduce_shape, stream));
        return FLEX_OK;
    }
    for (int a = 0; a < naux; ++a) {
        const size_t part = (start[a + 2] - start[a + 1]) * es;
        if (aux[a].engine == FLEX_ENGINE_SDMA && part > aux[a].scratch_stride)
            return flex::fail(FLEX_ERR_INVALID_ARG,
                              "%s: host part of %zu bytes exceeds the scratch sized by max_host_units (%zu bytes "
                              "per peer)", who, part, aux[a].scratch_stride);
    }

    TimingRecord* rec;
    st = begin_split_call(c, count * es, adaptive, generation, stream, &rec);
    if (st) return st;
    st = split_reduce(rec, start, bufs, out, dtype, stream);
    return st ? abandon_split_call(c, rec != nullptr, st) : FLEX_OK;
}

int flex_comm::split_reduce(TimingRecord* rec, const uint64_t* start, const void* const* bufs, void* out,
                            int dtype, hipStream_t stream) {
    const size_t es = flex::dtype_size(dtype);
    // fork (rec == nullptr: the Evaluator does not sample this call)
    hipEvent_t fork = rec ? rec->fork : fork_untimed;
    HIP_TRY(hipEventRecord(fork, stream));

    // device path: head of the message, straight from HBM
    if (start[1] > 0) {
        LAUNCH_TRY(flex::launch_reduce_n(bufs, nranks, out, start[1], dtype, reduce_shape, stream));
        if (rec) rec->used_mask |= 1u;
    }
    if (rec) HIP_TRY(hipEventRecord(rec->done[0], stream));

    // host paths: every peer's part goes device -> pinned slot -> device and is
    // reduced in the same rank order; the local contribution never leaves HBM
    for (int a = 0; a < naux; ++a) {
        const uint64_t lo = start[a + 1], hi = start[a + 2];
        if (hi == lo) continue;
        HostPath& hp = aux[a];
        HostJob job;
        job.reduce = true;
        job.dtype = dtype;
        job.nranks = nranks;
        job.local_index = rank;
        job.local_src = (const char*)bufs[rank] + lo * es;
        job.out_part = (char*)out + lo * es;
        for (int r = 0; r < nranks; ++r) {
            if (r == rank) continue;
            job.peer_src[job.npeers] = (const char*)bufs[r] + lo * es;
            job.peer_dst[job.npeers] = hp.scratch ? hp.scratch + (size_t)job.npeers * hp.scratch_stride : nullptr;
            ++job.npeers;
        }
        int st = host_path(hp, job, (hi - lo) * es, fork);
        if (st) return st;
        hipEvent_t done = rec ? rec->done[a + 1] : join_untimed[a];
        HIP_TRY(hipEventRecord(done, hp.last_stream()));
        if (rec) rec->used_mask |= 1u << (a + 1);
        HIP_TRY(hipStreamWaitEvent(stream, done, 0));  // join
    }
    return FLEX_OK;
}

int flex_comm::alltoall(const void* const* bufs, void* out, size_t count, int dtype, hipStream_t stream) {
    const size_t es = flex::dtype_size(dtype);
    if (es == 0) return flex::fail(FLEX_ERR_UNSUPPORTED, "flex_alltoall_local: unknown dtype %d", dtype);
    if (!bufs) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_alltoall_local: rank pointer array is NULL");
    if (count > max_bytes / es / (size_t)nranks)
        return flex::fail(FLEX_ERR_INVALID_ARG,
                          "flex_alltoall_local: %d x %zu elements exceed max_bytes_per_rank %zu", nranks, count,
                          max_bytes);
    // what rank r sends to the local rank sits rank * count elements into r's buffer
    const void* piece[FLEX_MAX_RANKS];
    for (int r = 0; r < nranks; ++r) {
        if (count > 0 && !bufs[r])
            return flex::fail(FLEX_ERR_INVALID_ARG, "flex_alltoall_local: rank %d pointer is NULL", r);
        piece[r] = (const char*)bufs[r] + (size_t)rank * count * es;
    }
    return gather(FLEX_ALLTOALL, "flex_alltoall_local", piece, out, count, dtype, stream);
}

int flex_comm::gather(int c, const char* who, const void* const* slices, void* out, size_t count, int dtype,
                      hipStream_t stream) {
    int st = validate(who, slices, out, count, dtype);
    if (st) return st;
    CollState& cs = coll[c];
    ++cs.calls;
    if (count == 0) return FLEX_OK;
    st = poll_before_call(stream);
    if (st) return st;

    const size_t es = flex::dtype_size(dtype);
    const size_t slice_bytes = count * es;
    uint64_t start[FLEX_MAX_PATHS + 1];
    bool adaptive;
    uint64_t generation;
    const bool split = split_message(c, count, es, start, &adaptive, &generation);

    const void* src[FLEX_MAX_RANKS];
    void* dst[FLEX_MAX_RANKS];
    uint64_t bytes[FLEX_MAX_RANKS];
    for (int r = 0; r < nranks; ++r) {
        src[r] = slices[r];
        dst[r] = (char*)out + (size_t)r * slice_bytes;
        bytes[r] = (r == rank) ? slice_bytes : start[1] * es;  // local slice: whole, on the device path
    }
    if (!split) {
        LAUNCH_TRY(flex::launch_gather_copy(src, dst, bytes, nranks, copy_shape, stream));
        return FLEX_OK;
    }

    TimingRecord* rec;
    st = begin_split_call(c, slice_bytes, adaptive, generation, stream, &rec);
    if (st) return st;
    st = split_gather(rec, start, src, dst, bytes, slices, es, stream);
    return st ? abandon_split_call(c, rec != nullptr, st) : FLEX_OK;
}

int flex_comm::split_gather(TimingRecord* rec, const uint64_t* start, const void* const* src, void* const* dst,
                            const uint64_t* bytes, const void* const* slices, size_t es, hipStream_t stream) {
    hipEvent_t fork = rec ? rec->fork : fork_untimed;
    HIP_TRY(hipEventRecord(fork, stream));

    LAUNCH_TRY(flex::launch_gather_copy(src, dst, bytes, nranks, copy_shape, stream));
    if (rec) {
        rec->used_mask |= 1u;
        HIP_TRY(hipEventRecord(rec->done[0], stream));
    }

    for (int a = 0; a < naux; ++a) {
        const uint64_t lo = start[a + 1], hi = start[a + 2];
        if (hi == lo) continue;
        HostPath& hp = aux[a];
        HostJob job;
        for (int r = 0; r < nranks; ++r) {
            if (r == rank) continue;
            job.peer_src[job.npeers] = (const char*)slices[r] + lo * es;
            job.peer_dst[job.npeers] = (char*)dst[r] + lo * es;
            ++job.npeers;
        }
        int st = host_path(hp, job, (hi - lo) * es, fork);
        if (st) return st;
        hipEvent_t done = rec ? rec->done[a + 1] : join_untimed[a];
        HIP_TRY(hipEventRecord(done, hp.last_stream()));
        if (rec) rec->used_mask |= 1u << (a + 1);
        HIP_TRY(hipStreamWaitEvent(stream, done, 0));
    }
    return FLEX_OK;
}

// MeasurePathTimings of Algorithm 1: median per-path time of cfg.tune_reps
// calls at fixed shares.  units[p], p >= 1: share of auxiliary path p.
// T[path] in seconds.
int flex_comm::measure_split(int c, const void* const* bufs, void* out, size_t count, int dtype,
                             hipStream_t stream, const uint32_t* units, double* T) {
    CollState& cs = coll[c];
    cs.mode = FLEX_SPLIT_STATIC;
    for (int p = 1; p < FLEX_MAX_PATHS; ++p) cs.static_units[p] = p < npaths() ? units[p] : 0;
    std::vector<double> t[FLEX_MAX_PATHS];
    for (uint32_t k = 0; k < cfg.tune_reps + 1; ++k) {
        split_seq = 0;  // MeasurePathTimings samples every call
        const uint64_t before = cs.samples;
        int st = collective(c, bufs, out, count, dtype, stream);
        if (st) return st;
        st = poll(true);
        if (st) return st;
        if (cs.samples == before)
            return flex::fail(FLEX_ERR_STATE, "flex_comm_tune: a split call produced no timing sample");
        if (k == 0) continue;  // first call warms the paths up
        for (int p = 0; p < FLEX_MAX_PATHS; ++p) t[p].push_back(cs.last_t[p]);
    }
    for (int p = 0; p < FLEX_MAX_PATHS; ++p) T[p] = median_of(t[p]);
    return FLEX_OK;
}

// Whole-call times at fixed shares: events on the caller's stream around each of
// `reps` calls (after one untimed call if `warm`), appended to *seconds.
int flex_comm::time_calls(int c, const void* const* bufs, void* out, size_t count, int dtype, hipStream_t stream,
                          const uint32_t* units, uint32_t reps, bool warm, std::vector<double>* seconds) {
    CollState& cs = coll[c];
    cs.mode = FLEX_SPLIT_STATIC;
    for (int p = 1; p < FLEX_MAX_PATHS; ++p) cs.static_units[p] = (units && p < npaths()) ? units[p] : 0;
    for (uint32_t k = 0; k < reps + (warm ? 1u : 0u); ++k) {
        HIP_TRY(hipEventRecord(t0, stream));
        int st = collective(c, bufs, out, count, dtype, stream);
        if (st) return st;
        HIP_TRY(hipEventRecord(t1, stream));
        HIP_TRY(hipEventSynchronize(t1));
        st = poll(true);
        if (st) return st;
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, t0, t1));
        if (!warm || k > 0) seconds->push_back(ms * 1e-3);
    }
    return FLEX_OK;
}

extern "C" {

int flex_config_default(flex_config_t* cfg) {
    if (!cfg) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_config_default: cfg is NULL");
    memset(cfg, 0, sizeof *cfg);
    cfg->struct_size = (uint32_t)sizeof *cfg;
    cfg->chunk_bytes = 4u << 20;
    cfg->num_slots = 2;
    cfg->max_host_units = 2500;
    cfg->split_align_elems = 2048;
    cfg->min_split_bytes = 64u << 10;
    cfg->tune_reps = 5;
    cfg->probe_units = 200;
    cfg->tune_accept_check = 1;
    cfg->accept_pairs = 3;
    // Launch shape found best on MI355X for the 8 x 256 MiB AllReduce followed by
    // the 8 x 32 MiB AllGather on buffers that are cold in the memory-side cache:
    // one wavefront per workgroup, one 16-byte vector per lane and input, one
    // workgroup per tile, one load in flight per wavefront in the reduce, loads
    // and stores both marked non-temporal.  (When the same 256 MiB output is
    // rewritten call after call it stays resident in the 256 MB memory-side
    // cache and plain stores are a few percent faster.)
    cfg->launch_shape = FLEX_SHAPE_WAVE;
    cfg->reduce_serial_loads = 1;
    cfg->reduce_nontemporal = 3;
    cfg->reduce_lds_reserve = 5632;
    cfg->copy_nontemporal = 3;
    cfg->host_engine = FLEX_ENGINE_KERNEL;
    cfg->host_blocks = 8;
    cfg->host_down_blocks = 6;
    cfg->sample_every = 1;
    cfg->host_die_shift = 2;
    cfg->min_step_bytes = 256u << 10;
    cfg->slot_sync = FLEX_SYNC_EVENTS;
    cfg->num_aux_paths = 1;
    flex::balancer_cfg_default(&cfg->balancer);
    return FLEX_OK;
}

static bool hints_ok(uint32_t nt) { return nt == 0 || nt == 1 || nt == 3; }

int flex_comm_create(flex_comm_t** comm, int nranks, int rank, size_t max_bytes_per_rank,
                     const flex_config_t* cfg) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_create: comm is NULL");
    *comm = nullptr;
    if (nranks < 1 || nranks > FLEX_MAX_RANKS || rank < 0 || rank >= nranks)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_create: nranks %d / rank %d out of range", nranks,
                          rank);
    flex_config_t c;
    flex_config_default(&c);
    if (cfg) {
        if (cfg->struct_size != sizeof(flex_config_t))
            return flex::fail(FLEX_ERR_INVALID_ARG,
                              "flex_comm_create: cfg->struct_size is %u, this library's flex_config_t has %zu bytes "
                              "(start from flex_config_default)", cfg->struct_size, sizeof(flex_config_t));
        c = *cfg;
    }
    const flex_balancer_cfg_t& b = c.balancer;
    if (c.chunk_bytes < 4096 || c.chunk_bytes % 256 || c.num_slots < 1 || c.num_slots > 64 ||
        c.host_engine > FLEX_ENGINE_SDMA || c.slot_sync > FLEX_SYNC_COUNTERS || c.host_blocks < 1 ||
        c.host_blocks > 65536 || c.host_down_blocks < 1 || c.host_down_blocks > 65536 || c.sample_every < 1 || c.min_step_bytes == 0 || c.num_aux_paths < 1 || c.num_aux_paths > 2 ||
        c.host_die_shift > 3 || c.reduce_serial_loads > 2 || c.reduce_lds_reserve > 65536 || c.launch_shape > FLEX_SHAPE_BLOCK ||
        !hints_ok(c.reduce_nontemporal) || !hints_ok(c.copy_nontemporal) || b.share_total == 0 ||
        c.max_host_units > b.share_total || c.split_align_elems == 0 || c.tune_reps < 1 || c.accept_pairs < 1 ||
        c.probe_units == 0 || b.window == 0 || b.initial_step == 0 || b.runtime_step == 0)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_create: configuration out of range");

    flex_comm* m = new (std::nothrow) flex_comm;
    if (!m) return flex::fail(FLEX_ERR_NOMEM, "flex_comm_create: out of host memory");
    m->nranks = nranks;
    m->rank = rank;
    m->max_bytes = max_bytes_per_rank;
    m->cfg = c;

#define CREATE_TRY(expr)                                                                      \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) {                                                               \
            int code_ = (e_ == hipErrorOutOfMemory) ? FLEX_ERR_NOMEM : FLEX_ERR_HIP;          \
            flex::fail(code_, "flex_comm_create: %s failed: %s", #expr, hipGetErrorString(e_)); \
            flex_comm_destroy(m);                                                             \
            return code_;                                                                     \
        }                                                                                     \
    } while (0)

    CREATE_TRY(hipGetDevice(&m->device));
    int cus = 0;
    CREATE_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, m->device));
    const uint32_t threads = c.launch_shape == FLEX_SHAPE_BLOCK ? 256u : 64u;
    m->reduce_shape = {threads, 1, c.reduce_nontemporal, (uint32_t)cus, 0};
    // 16 tiles per compute unit: half of the wavefront slots of the chip
    m->reduce_shape.serial_min_tiles = c.reduce_serial_loads == 2 ? 1u
                                       : c.reduce_serial_loads == 1 ? 16u * (uint32_t)cus : 0u;
    // left to itself the library keeps both loads of a two-rank sum in flight at every size
    m->reduce_shape.serial_min_inputs = c.reduce_serial_loads == 1 ? 3u : 1u;
    m->copy_shape = {threads, 1, c.copy_nontemporal, (uint32_t)cus, 0};
    m->reduce_shape.serial_lds_bytes = c.reduce_lds_reserve;
    // kernels that read or write pinned memory over PCIe: a fixed, small number
    // of workgroups striding over the step, kept on few dies, so that waves
    // waiting on the link do not crowd the device path off the memory system
    m->link_reduce_shape = {256, 1, 0, (uint32_t)cus, c.host_down_blocks, c.host_die_shift};
    m->link_copy_shape = {256, 2, 0, (uint32_t)cus, c.host_blocks, c.host_die_shift};
    // reading pinned memory is latency-bound: four vectors in flight per lane (about 110 KiB in all
    // with one workgroup per peer) bring 35 GB/s back where two bring 29
    m->link_down_copy_shape = {256, 4, 0, (uint32_t)cus, c.host_blocks, c.host_die_shift};
    // hybrid engine: kernels that drain a staging buffer run at HBM speed and
    // are over in microseconds; all loads of a tile in flight
    m->stage_reduce_shape = {256, 1, 0, (uint32_t)cus, 0};
    m->stage_copy_shape = {256, 2, 0, (uint32_t)cus, 0};
    CREATE_TRY(hipEventCreate(&m->t0));
    CREATE_TRY(hipEventCreate(&m->t1));
    CREATE_TRY(hipEventCreateWithFlags(&m->fork_untimed, hipEventDisableTiming));
    for (auto& e : m->join_untimed) CREATE_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));

    if (nranks > 1) {
        if (c.slot_sync == FLEX_SYNC_COUNTERS) {
            int can = 0;
            CREATE_TRY(hipDeviceGetAttribute(&can, hipDeviceAttributeCanUseStreamWaitValue, m->device));
            if (!can) {
                flex::fail(FLEX_ERR_UNSUPPORTED, "flex_comm_create: device has no stream wait-value support");
                flex_comm_destroy(m);
                return FLEX_ERR_UNSUPPORTED;
            }
        }
        // DMA-engine scratch: per peer, the largest part a call may route to the
        // path (rounded up by one alignment quantum of the widest element)
        unsigned __int128 part = (unsigned __int128)max_bytes_per_rank * c.max_host_units;
        size_t per_peer = (size_t)((part + b.share_total - 1) / b.share_total);
        per_peer += (size_t)c.split_align_elems * 4 * 2;
        per_peer = std::min(per_peer, max_bytes_per_rank);
        per_peer = (per_peer + 255) / 256 * 256;
        const size_t slot_bytes = c.chunk_bytes * (size_t)(nranks - 1);

        m->naux = (int)c.num_aux_paths;
        for (int a = 0; a < m->naux; ++a) {
            HostPath& hp = m->aux[a];
            // the first auxiliary path uses the configured engine, the second the DMA engines
            // (or the copy kernels, if the first one has the DMA engines)
            hp.engine = a == 0 ? (int)c.host_engine
                               : (c.host_engine == FLEX_ENGINE_SDMA ? FLEX_ENGINE_KERNEL : FLEX_ENGINE_SDMA);
            const bool hybrid = hp.engine == FLEX_ENGINE_HYBRID;
            const bool lanes = hybrid && c.slot_sync == FLEX_SYNC_EVENTS;
            // side streams at the default priority
            if (!lanes) {
                CREATE_TRY(hipStreamCreateWithFlags(&hp.s_up, hipStreamNonBlocking));
                CREATE_TRY(hipStreamCreateWithFlags(&hp.s_down, hipStreamNonBlocking));
                if (hybrid) CREATE_TRY(hipStreamCreateWithFlags(&hp.s_fin, hipStreamNonBlocking));
            }
            for (uint32_t s = 0; s < c.num_slots; ++s) {
                if (lanes) {
                    hipStream_t st = nullptr;
                    CREATE_TRY(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
                    hp.lane.push_back(st);
                    for (auto* vec : {&hp.ev_up, &hp.ev_end}) {
                        hipEvent_t e = nullptr;
                        CREATE_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
                        vec->push_back(e);
                    }
                }
                void* p = nullptr;
                CREATE_TRY(hipHostMalloc(&p, slot_bytes, hipHostMallocDefault));
                hp.pinned.push_back(p);
                for (auto* vec : {&hp.ev_full, &hp.ev_empty}) {
                    hipEvent_t e = nullptr;
                    CREATE_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
                    vec->push_back(e);
                }
                if (hybrid) {
                    char* d = nullptr;
                    CREATE_TRY(hipMalloc((void**)&d, slot_bytes));
                    hp.stage.push_back(d);
                    for (auto* vec : {&hp.ev_staged, &hp.ev_stage_free}) {
                        hipEvent_t e = nullptr;
                        CREATE_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
                        vec->push_back(e);
                    }
                }
                if (c.slot_sync == FLEX_SYNC_COUNTERS) {
                    // stream memory operations need signal memory, 8 bytes per allocation
                    for (auto* vec : {&hp.sem_full, &hp.sem_empty}) {
                        uint64_t* sem = nullptr;
                        CREATE_TRY(hipExtMallocWithFlags((void**)&sem, 8, hipMallocSignalMemory));
                        vec->push_back(sem);
                        CREATE_TRY(hipMemset(sem, 0, 8));
                    }
                    hp.slot_uses.push_back(0);
                }
            }
            hp.scratch_stride = per_peer;
            if (hp.engine == FLEX_ENGINE_SDMA && c.max_host_units > 0 && max_bytes_per_rank > 0)
                CREATE_TRY(hipMalloc((void**)&hp.scratch, per_peer * (size_t)(nranks - 1)));
        }
        if (c.slot_sync == FLEX_SYNC_COUNTERS) CREATE_TRY(hipDeviceSynchronize());

        m->ring.resize(kRingSize);
        for (auto& rec : m->ring.records()) {
            CREATE_TRY(hipEventCreate(&rec.fork));
            for (int p = 0; p < 1 + m->naux; ++p) CREATE_TRY(hipEventCreate(&rec.done[p]));
        }
    }
#undef CREATE_TRY
    *comm = m;
    return FLEX_OK;
}

int flex_comm_destroy(flex_comm_t* m) {
    if (!m) return FLEX_OK;
    for (auto& hp : m->aux) hp.destroy();
    for (auto& rec : m->ring.records()) {
        if (rec.fork) (void)hipEventDestroy(rec.fork);
        for (auto e : rec.done)
            if (e) (void)hipEventDestroy(e);
    }
    if (m->t0) (void)hipEventDestroy(m->t0);
    if (m->t1) (void)hipEventDestroy(m->t1);
    if (m->fork_untimed) (void)hipEventDestroy(m->fork_untimed);
    for (auto e : m->join_untimed)
        if (e) (void)hipEventDestroy(e);
    delete m;
    return FLEX_OK;
}

int flex_allreduce_local(flex_comm_t* comm, const void* const* rank_bufs, void* out, size_t count,
                         int dtype, int op, void* hip_stream) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_allreduce_local: comm is NULL");
    if (op != FLEX_SUM) return flex::fail(FLEX_ERR_UNSUPPORTED, "flex_allreduce_local: unknown op %d", op);
    return comm->reduce(FLEX_ALLREDUCE, "flex_allreduce_local", rank_bufs, out, count, dtype,
                        (hipStream_t)hip_stream);
}

int flex_reducescatter_local(flex_comm_t* comm, const void* const* rank_bufs, void* out, size_t recv_count,
                             int dtype, int op, void* hip_stream) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_reducescatter_local: comm is NULL");
    if (op != FLEX_SUM) return flex::fail(FLEX_ERR_UNSUPPORTED, "flex_reducescatter_local: unknown op %d", op);
    return comm->reducescatter(rank_bufs, out, recv_count, dtype, (hipStream_t)hip_stream);
}

int flex_allgather_local(flex_comm_t* comm, const void* const* rank_slices, void* out,
                         size_t slice_count, int dtype, void* hip_stream) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_allgather_local: comm is NULL");
    return comm->gather(FLEX_ALLGATHER, "flex_allgather_local", rank_slices, out, slice_count, dtype,
                        (hipStream_t)hip_stream);
}

int flex_alltoall_local(flex_comm_t* comm, const void* const* rank_bufs, void* out, size_t count, int dtype,
                        void* hip_stream) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_alltoall_local: comm is NULL");
    return comm->alltoall(rank_bufs, out, count, dtype, (hipStream_t)hip_stream);
}

int flex_set_split_paths(flex_comm_t* comm, int coll, int mode, const uint32_t* aux_units, int naux) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_set_split_paths: comm is NULL");
    if (coll < FLEX_ALLREDUCE || coll > FLEX_ALLTOALL)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_set_split_paths: unknown collective %d", coll);
    if (mode != FLEX_SPLIT_STATIC && mode != FLEX_SPLIT_ADAPTIVE)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_set_split_paths: unknown mode %d", mode);
    if (mode == FLEX_SPLIT_STATIC) {
        if (naux < 0 || naux > kMaxAux || (naux > 0 && !aux_units))
            return flex::fail(FLEX_ERR_INVALID_ARG, "flex_set_split_paths: bad share array");
        uint64_t sum = 0;
        for (int a = 0; a < naux; ++a) {
            if (aux_units[a] > comm->cfg.max_host_units)
                return flex::fail(FLEX_ERR_INVALID_ARG, "flex_set_split_paths: share %u exceeds max_host_units %u",
                                  aux_units[a], comm->cfg.max_host_units);
            if (aux_units[a] > 0 && a >= std::max(comm->naux, 1))
                return flex::fail(FLEX_ERR_INVALID_ARG,
                                  "flex_set_split_paths: the communicator has %d auxiliary path(s)", comm->naux);
            sum += aux_units[a];
        }
        if (sum > comm->cfg.balancer.share_total)
            return flex::fail(FLEX_ERR_INVALID_ARG, "flex_set_split_paths: shares exceed share_total");
        CollState& cs = comm->coll[coll];
        for (int p = 1; p < FLEX_MAX_PATHS; ++p) cs.static_units[p] = p - 1 < naux ? aux_units[p - 1] : 0;
    }
    comm->coll[coll].mode = (uint32_t)mode;
    return FLEX_OK;
}

int flex_set_split(flex_comm_t* comm, int coll, int mode, uint32_t host_units) {
    return flex_set_split_paths(comm, coll, mode, &host_units, 1);
}

// Balancer settings of this communicator: the configured ones, with the host
// paths' ceiling.
static flex_balancer_cfg_t balancer_cfg_of(const flex_comm* m) {
    flex_balancer_cfg_t bc = m->cfg.balancer;
    bc.aux_share_cap = m->cfg.max_host_units;
    return bc;
}

int flex_comm_tune(flex_comm_t* comm, int coll, const void* const* rank_bufs, void* out, size_t count,
                   int dtype, void* hip_stream, flex_tune_result_t* result) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_tune: comm is NULL");
    if (coll < FLEX_ALLREDUCE || coll > FLEX_ALLTOALL)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_tune: unknown collective %d", coll);
    int st = comm->validate("flex_comm_tune", rank_bufs, out, count, dtype);
    if (st) return st;
    if (count == 0) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_tune: empty message");
    hipStream_t stream = (hipStream_t)hip_stream;
    CollState& cs = comm->coll[coll];
    const size_t es = flex::dtype_size(dtype);
    const double msg_bytes = (double)count * es;
    const flex_config_t& cfg = comm->cfg;
    const flex_balancer_cfg_t bc = balancer_cfg_of(comm);
    const int np = std::max(comm->npaths(), 2);  // a communicator without peers still reports two paths
    flex_tune_result_t res;
    memset(&res, 0, sizeof res);

    struct Restore {
        CollState& cs;
        uint32_t mode;
        uint32_t units[FLEX_MAX_PATHS];
        ~Restore() {
            cs.mode = mode;
            memcpy(cs.static_units, units, sizeof units);
        }
    } restore{cs, cs.mode, {cs.static_units[0], cs.static_units[1], cs.static_units[2], cs.static_units[3]}};

    st = comm->poll(true);
    if (st) return st;

    // Rate of the device path carrying the whole message alone.
    std::vector<double> alone;
    st = comm->time_calls(coll, rank_bufs, out, count, dtype, stream, nullptr, cfg.tune_reps, true, &alone);
    if (st) return st;
    const double t_dev_alone = median_of(alone);
    res.path_bw[FLEX_PATH_DEVICE] = t_dev_alone > 0 ? msg_bytes / t_dev_alone : 0.0;

    // Rate of each host path, measured on a probe share of the message with the
    // other host path idle.
    double T[FLEX_MAX_PATHS] = {0, 0, 0, 0};
    const uint32_t probe = std::min(cfg.probe_units, cfg.max_host_units);
    for (int p = 1; p < comm->npaths() && probe > 0; ++p) {
        uint32_t units[FLEX_MAX_PATHS] = {0, 0, 0, 0};
        units[p] = probe;
        uint64_t start[FLEX_MAX_PATHS + 1];
        flex::partition_paths(count, units, comm->npaths(), bc.share_total, cfg.split_align_elems,
                              cfg.min_split_bytes / es, start);
        const uint64_t part = start[p + 1] - start[p];
        if (part == 0) continue;
        st = comm->measure_split(coll, rank_bufs, out, count, dtype, stream, units, T);
        if (st) return st;
        res.path_bw[p] = T[p] > 0 ? (double)part * es / T[p] : 0.0;
    }

    SizeClass sc;
    sc.tuned = true;
    if (!(res.path_bw[FLEX_PATH_DEVICE] > 0) || !sc.bal.init_from_bandwidth(np, res.path_bw, bc))
        return flex::fail(FLEX_ERR_STATE, "flex_comm_tune: could not measure the device path");
    {
        // a host path never starts above its ceiling: the excess goes to the device path
        uint32_t s0[FLEX_MAX_PATHS];
        bool trimmed = false;
        for (int p = 0; p < FLEX_MAX_PATHS; ++p) s0[p] = sc.bal.shares[p];
        for (int p = 1; p < np; ++p)
            if (s0[p] > cfg.max_host_units) {
                s0[0] += s0[p] - cfg.max_host_units;
                s0[p] = cfg.max_host_units;
                trimmed = true;
            }
        if (trimmed && !sc.bal.init_from_shares(np, s0, bc))
            return flex::fail(FLEX_ERR_STATE, "flex_comm_tune: could not set up the starting shares");
    }
    for (int p = 0; p < np; ++p) res.initial_shares[p] = sc.bal.shares[p];

    auto shares_of = [&](uint32_t* units) {
        for (int p = 0; p < FLEX_MAX_PATHS; ++p) units[p] = p < np ? sc.bal.shares[p] : 0;
    };

    // Algorithm 1 with real measurements.
    while (sc.bal.stage == FLEX_STAGE_TUNING) {
        flex_tune_round_t round;
        memset(&round, 0, sizeof round);
        uint32_t units[FLEX_MAX_PATHS];
        shares_of(units);
        memcpy(round.shares_before, units, sizeof units);
        st = comm->measure_split(coll, rank_bufs, out, count, dtype, stream, units, T);
        if (st) return st;
        if (!sc.bal.update(T))
            return flex::fail(FLEX_ERR_STATE, "flex_comm_tune: unusable path timings (%g s, %g s, %g s)", T[0],
                              T[1], T[2]);
        for (int p = 0; p < np; ++p)
            round.path_time_s[p] = (round.shares_before[p] > 0) ? T[p] : 0.0;
        shares_of(round.shares_after);
        round.step_after = sc.bal.step;
        round.active_after = sc.bal.active_mask;
        ++sc.rounds_run;
        if (sc.rounds.size() < kMaxTuneRounds) sc.rounds.push_back(round);
    }
    for (int p = 0; p < np; ++p) res.balanced_shares[p] = sc.bal.shares[p];

    // Acceptance check: the balanced split must beat the device path alone by
    // more than the noise.  Both are timed as whole calls on the caller's
    // stream, in turns, so that drift hits both alike.
    if (cfg.tune_accept_check && (sc.bal.active_mask & ~1u)) {
        uint32_t units[FLEX_MAX_PATHS];
        shares_of(units);
        std::vector<double> split_s, alone_s;
        for (uint32_t pair = 0; pair < cfg.accept_pairs; ++pair) {
            st = comm->time_calls(coll, rank_bufs, out, count, dtype, stream, units, cfg.tune_reps, pair == 0,
                                  &split_s);
            if (st) return st;
            st = comm->time_calls(coll, rank_bufs, out, count, dtype, stream, nullptr, cfg.tune_reps, pair == 0,
                                  &alone_s);
            if (st) return st;
        }
        res.combined_s = median_of(split_s);
        res.device_alone_s = median_of(alone_s);
        res.combined_mad_s = mad_of(split_s);
        res.device_alone_mad_s = mad_of(alone_s);
        res.accept_samples = (uint32_t)split_s.size();
        const double gain = res.device_alone_s - res.combined_s;
        if (!(gain > 3.0 * std::max(res.combined_mad_s, res.device_alone_mad_s))) {
            sc.bal.revert_to_primary();
            res.reverted = 1;
        }
    }

    // leave `out` holding a result computed after the last share change
    {
        uint32_t units[FLEX_MAX_PATHS];
        shares_of(units);
        memcpy(cs.static_units, units, sizeof units);
        cs.static_units[0] = 0;
        cs.mode = FLEX_SPLIT_STATIC;
    }
    st = comm->collective(coll, rank_bufs, out, count, dtype, stream);
    if (st) return st;
    HIP_TRY(hipStreamSynchronize(stream));
    st = comm->poll(true);
    if (st) return st;

    for (int p = 0; p < np; ++p) {
        res.shares[p] = sc.bal.shares[p];
        res.path_time_s[p] = T[p];
    }
    res.active_mask = sc.bal.active_mask;
    res.iterations = sc.bal.tune_iters;
    auto& slot = cs.classes[size_class_of(count * es)];
    const uint64_t gen = slot.generation + 1;
    slot = sc;
    slot.generation = gen;
    if (result) *result = res;
    return FLEX_OK;
}

int flex_comm_tune_trace(flex_comm_t* comm, int coll, size_t count, int dtype, flex_tune_round_t* rounds,
                         uint32_t max_rounds, uint32_t* nrounds) {
    if (!comm || !nrounds || (max_rounds > 0 && !rounds))
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_tune_trace: NULL argument");
    if (coll < FLEX_ALLREDUCE || coll > FLEX_ALLTOALL)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_tune_trace: unknown collective %d", coll);
    const size_t es = flex::dtype_size(dtype);
    if (es == 0) return flex::fail(FLEX_ERR_UNSUPPORTED, "flex_comm_tune_trace: unknown dtype %d", dtype);
    SizeClass* sc = comm->find_class(coll, size_class_of(count * es));
    if (!sc || !sc->tuned)
        return flex::fail(FLEX_ERR_STATE, "flex_comm_tune_trace: this size class was never tuned");
    *nrounds = sc->rounds_run;
    for (size_t k = 0; k < sc->rounds.size() && k < max_rounds; ++k) rounds[k] = sc->rounds[k];
    return FLEX_OK;
}

int flex_comm_set_shares(flex_comm_t* comm, int coll, size_t count, int dtype, const uint32_t* shares) {
    if (!comm || !shares) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_set_shares: NULL argument");
    if (coll < FLEX_ALLREDUCE || coll > FLEX_ALLTOALL)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_set_shares: unknown collective %d", coll);
    const size_t es = flex::dtype_size(dtype);
    if (es == 0) return flex::fail(FLEX_ERR_UNSUPPORTED, "flex_comm_set_shares: unknown dtype %d", dtype);
    const int np = std::max(comm->npaths(), 2);
    for (int p = 1; p < np; ++p)
        if (shares[p] > comm->cfg.max_host_units)
            return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_set_shares: share %u exceeds max_host_units %u",
                              shares[p], comm->cfg.max_host_units);
    SizeClass sc;
    sc.tuned = true;
    if (!sc.bal.init_from_shares(np, shares, balancer_cfg_of(comm)))
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_comm_set_shares: shares must sum to share_total");
    sc.bal.finish_tuning();
    auto& slot = comm->coll[coll].classes[size_class_of(count * es)];
    const uint64_t gen = slot.generation + 1;
    slot = sc;
    slot.generation = gen;
    return FLEX_OK;
}

int flex_evaluator_poll(flex_comm_t* comm) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_evaluator_poll: comm is NULL");
    return comm->poll(false);
}

int flex_evaluator_drain(flex_comm_t* comm) {
    if (!comm) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_evaluator_drain: comm is NULL");
    return comm->poll(true);
}

int flex_get_stats(flex_comm_t* comm, int coll, size_t count, int dtype, flex_stats_t* out) {
    if (!comm || !out) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_get_stats: NULL argument");
    if (coll < FLEX_ALLREDUCE || coll > FLEX_ALLTOALL)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_get_stats: unknown collective %d", coll);
    const size_t es = flex::dtype_size(dtype);
    if (es == 0) return flex::fail(FLEX_ERR_UNSUPPORTED, "flex_get_stats: unknown dtype %d", dtype);
    memset(out, 0, sizeof *out);
    const CollState& cs = comm->coll[coll];
    out->calls = cs.calls;
    out->split_calls = cs.split_calls;
    out->samples = cs.samples;
    out->blocking_reads = comm->ring.blocking_reads();
    out->last_count = cs.last_count;
    out->last_split = cs.last_start[1];
    out->mode = cs.mode;
    out->static_host_units = cs.static_units[1];
    out->npaths = (uint32_t)comm->npaths();
    for (int p = 0; p < FLEX_MAX_PATHS; ++p) {
        out->last_time_s[p] = cs.last_t[p];
        out->mean_time_s[p] = cs.samples ? cs.sum_t[p] / (double)cs.samples : 0.0;
        out->static_units[p] = cs.static_units[p];
        out->last_start[p] = cs.last_start[p];
    }
    if (SizeClass* sc = comm->find_class(coll, size_class_of(count * es))) sc->bal.get(&out->balancer);
    return FLEX_OK;
}

const char* flex_status_string(int status) {
    switch (status) {
        case FLEX_OK: return "ok";
        case FLEX_ERR_INVALID_ARG: return "invalid argument";
        case FLEX_ERR_UNSUPPORTED: return "unsupported dtype, op or collective";
        case FLEX_ERR_HIP: return "HIP runtime error";
        case FLEX_ERR_NOMEM: return "out of memory";
        case FLEX_ERR_STATE: return "invalid state";
        default: return "unknown status";
    }
}

const char* flex_last_error(void) { return flex::g_last_error; }

}  // extern "C"
