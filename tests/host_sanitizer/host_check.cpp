// Host-only check of the library's pure host logic under AddressSanitizer and
// UndefinedBehaviorSanitizer: the balancer (csrc/balancer.cpp, compiled into
// this program), the message partition, the pipeline step plan and the
// Evaluator's record ring driven by a scripted event layer instead of HIP.
// Test infrastructure: built and run by tests/test_host_sanitizer.py.
// Exit status 0 = every check passed.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <random>
#include <vector>

#include "evaluator_ring.h"
#include "flexlink_internal.h"

namespace flex {
// the library defines this next to its HIP code; the host-only build brings its own
static char g_msg[512];
int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_msg, sizeof g_msg, fmt, ap);
    va_end(ap);
    return status;
}
}  // namespace flex

static int g_failures = 0;
#define CHECK(cond)                                                       \
    do {                                                                  \
        if (!(cond)) {                                                    \
            printf("FAIL %s:%d: %s\n", __FILE__, __LINE__, #cond);        \
            ++g_failures;                                                 \
        }                                                                 \
    } while (0)

// ---- a scripted event layer: an event is an index into a table of completion times
struct FakeEvents {
    std::map<int, double> when;  // event id -> completion time; absent = never recorded
    double now = 0.0;
    int fail_query_of = -1;      // event whose query reports an error
    int queries = 0, waits = 0;
    int query(int e) {
        ++queries;
        if (e == fail_query_of) return 77;
        auto it = when.find(e);
        return (it != when.end() && it->second <= now) ? 0 : 1;
    }
    int wait(int e) {
        ++waits;
        if (e == fail_query_of) return 77;
        auto it = when.find(e);
        if (it == when.end()) return 78;  // waiting for an event nobody records
        if (it->second > now) now = it->second;
        return 0;
    }
    int elapsed(int a, int b, double* seconds) {
        if (!when.count(a) || !when.count(b)) return 79;
        *seconds = when[b] - when[a];
        return 0;
    }
};
using Ring = flex::EvaluatorRing<int, FakeEvents>;

struct Seen {
    int coll;
    uint64_t generation;
    double T[4];
};

static void check_ring() {
    const size_t cap = 4;
    Ring ring(cap);
    for (size_t i = 0; i < cap; ++i) {
        ring.records()[i].fork = (int)(10 * i);
        for (int p = 0; p < 4; ++p) ring.records()[i].done[p] = (int)(10 * i + 1 + p);
    }
    FakeEvents ev;
    std::vector<Seen> seen;
    auto sink = [&](const Ring::Record& r, const double* T) {
        Seen s{r.coll, r.generation, {T[0], T[1], T[2], T[3]}};
        seen.push_back(s);
    };
    // a call on paths 0 and 1: fork at t, device done at t+1, host done at t+3
    auto issue = [&](double t, int tag) {
        Ring::Record* r = nullptr;
        int st = ring.acquire(ev, sink, &r);
        if (st) return st;
        r->coll = tag;
        r->generation = (uint64_t)tag * 100;
        ev.when[r->fork] = t;
        ev.when[r->done[0]] = t + 1;
        ev.when[r->done[1]] = t + 3;
        r->used_mask = 3;
        return 0;
    };
    CHECK(issue(0, 1) == 0 && issue(1, 2) == 0 && ring.in_flight() == 2);
    // nothing has finished at time 0.5: a non-blocking poll pops nothing and does not wait
    ev.now = 0.5;
    CHECK(ring.poll(ev, sink, false) == 0 && seen.empty() && ev.waits == 0 && ring.in_flight() == 2);
    // at time 3.5 the first call is complete, the second (host path done at 4) is not
    ev.now = 3.5;
    CHECK(ring.poll(ev, sink, false) == 0 && seen.size() == 1 && ring.in_flight() == 1);
    CHECK(seen[0].coll == 1 && seen[0].T[0] == 1.0 && seen[0].T[1] == 3.0 && seen[0].T[2] == 0.0);
    // a blocking poll waits for the rest, oldest first
    CHECK(ring.poll(ev, sink, true) == 0 && seen.size() == 2 && ring.in_flight() == 0 && ev.now == 4.0);
    CHECK(seen[1].coll == 2 && seen[1].generation == 200);

    // a call that fails after taking its record gives it back: no sample, the slot is reused
    {
        Ring::Record* r = nullptr;
        CHECK(ring.acquire(ev, sink, &r) == 0 && ring.in_flight() == 1);
        r->coll = 99;
        r->used_mask = 1;            // one event "recorded", the rest of the call failed
        ring.abandon();
        CHECK(ring.in_flight() == 0);
        CHECK(ring.poll(ev, sink, true) == 0 && seen.size() == 2);   // nothing of it is ever consumed
        Ring::Record* again = nullptr;
        CHECK(ring.acquire(ev, sink, &again) == 0 && again == r && again->used_mask == 0);
        ring.abandon();
    }

    // ring full: acquiring waits for the oldest record and counts the blocking read
    seen.clear();
    for (int k = 0; k < (int)cap; ++k) CHECK(issue(10 + k, 10 + k) == 0);
    CHECK(ring.in_flight() == cap && ring.blocking_reads() == 0);
    ev.now = 10;
    CHECK(issue(20, 20) == 0);
    CHECK(ring.blocking_reads() == 1 && ring.in_flight() == cap && seen.size() == 1 && seen[0].coll == 10);
    CHECK(ring.poll(ev, sink, true) == 0 && seen.size() == cap + 1 && seen.back().coll == 20);
    for (size_t k = 1; k < seen.size(); ++k) CHECK(seen[k].coll > seen[k - 1].coll);   // oldest first, none twice

    // an error from the event layer is passed through and the record stays for a later poll
    CHECK(issue(30, 30) == 0);
    size_t before = seen.size();
    for (size_t i = 0; i < cap; ++i)
        if (ring.records()[i].coll == 30) ev.fail_query_of = ring.records()[i].done[1];
    ev.now = 100;
    CHECK(ring.poll(ev, sink, false) == 77 && seen.size() == before && ring.in_flight() == 1);
    ev.fail_query_of = -2;
    CHECK(ring.poll(ev, sink, false) == 0 && seen.size() == before + 1 && ring.in_flight() == 0);

    // random schedule: every issued call is consumed exactly once, in issue order
    std::mt19937 rng(12345);
    seen.clear();
    int issued = 0, abandoned = 0;
    double t = 200;
    for (int step = 0; step < 2000; ++step) {
        const int what = (int)(rng() % 4);
        if (what <= 1) {
            t += 1;
            ev.now = t - (double)(rng() % 6);
            if (issue(t, 1000 + issued) == 0) ++issued;
        } else if (what == 2) {
            ev.now = t + (double)(rng() % 5);
            CHECK(ring.poll(ev, sink, false) == 0);
        } else {
            Ring::Record* r = nullptr;
            ev.now = t + 10;         // everything issued so far has finished
            if (ring.acquire(ev, sink, &r) == 0) {
                ring.abandon();
                ++abandoned;
            }
        }
        CHECK(ring.in_flight() <= cap);
    }
    ev.now = t + 10;
    CHECK(ring.poll(ev, sink, true) == 0 && ring.in_flight() == 0);
    CHECK((int)seen.size() == issued && abandoned > 0);
    for (size_t k = 0; k < seen.size(); ++k) CHECK(seen[k].coll == 1000 + (int)k);
}

static void check_partition_and_plan() {
    std::mt19937_64 rng(99);
    for (int k = 0; k < 20000; ++k) {
        const uint64_t count = rng() % (k % 3 ? (1ull << 22) : (1ull << 40));
        const uint32_t total = 10000, align = (uint32_t[]){1, 64, 2048, 4096}[rng() % 4];
        uint32_t units[4] = {0, (uint32_t)(rng() % 3334), (uint32_t)(rng() % 3334), (uint32_t)(rng() % 3334)};
        const int np = 2 + (int)(rng() % 3);
        uint64_t start[5];
        flex::partition_paths(count, units, np, total, align, 32768, start);
        CHECK(start[0] == 0 && start[np] == count);
        for (int p = 0; p < np; ++p) CHECK(start[p] <= start[p + 1]);
        if (np == 2) CHECK(start[1] == flex::partition(count, units[1], total, align, 32768));
        const uint64_t bytes = rng() % (1ull << 31), chunk = 256ull << (rng() % 15), min_step = 1 + rng() % (8u << 20);
        if (chunk >= 4096) {
            uint64_t sum = 0;
            for (uint64_t n : flex::plan_steps(bytes, chunk, min_step)) {
                CHECK(n > 0 && n <= chunk);
                sum += n;
            }
            CHECK(sum == bytes);
        }
    }
}

static void check_balancer() {
    std::mt19937 rng(7);
    std::uniform_real_distribution<double> u(0.01, 10.0);
    for (int k = 0; k < 3000; ++k) {
        flex_balancer_cfg_t cfg;
        flex::balancer_cfg_default(&cfg);
        cfg.initial_step = 1 + rng() % 500;
        cfg.window = 1 + rng() % 12;
        cfg.aux_share_cap = (rng() % 2) ? 0 : 100 + rng() % 5000;
        const int np = 1 + (int)(rng() % 4);
        double bw[4] = {u(rng) * 100, u(rng), u(rng), (rng() % 4) ? u(rng) : 0.0};
        flex::Balancer b;
        CHECK(b.init_from_bandwidth(np, bw, cfg));
        for (int it = 0; it < 300; ++it) {
            double T[4] = {u(rng), u(rng), u(rng), u(rng)};
            if (rng() % 50 == 0) T[rng() % 4] = -1.0;   // bad sample: rejected unless that path is inactive
            uint32_t before[4];
            memcpy(before, b.shares, sizeof before);
            const bool ok = b.update(T);
            uint64_t sum = 0;
            for (int p = 0; p < 4; ++p) sum += b.shares[p];
            CHECK(sum == cfg.share_total);
            if (!ok) CHECK(memcmp(before, b.shares, sizeof before) == 0);
            for (int p = 1; p < np; ++p)
                if (cfg.aux_share_cap && b.shares[p] > before[p]) CHECK(b.shares[p] <= cfg.aux_share_cap);
            for (int p = 0; p < 4; ++p)
                if (!(b.active_mask & (1u << p))) CHECK(b.shares[p] == 0 || p == 0);
        }
        flex_balancer_state_t st;
        b.get(&st);
        CHECK(st.tune_iters <= cfg.max_tune_iters && st.step >= 1 && st.step <= cfg.initial_step);
        b.revert_to_primary();
        CHECK(b.shares[0] == cfg.share_total && b.active_mask == 1u);
    }
}

int main() {
    check_ring();
    check_partition_and_plan();
    check_balancer();
    printf(g_failures ? "host check FAILED (%d)\n" : "host check passed\n", g_failures);
    return g_failures ? 1 : 0;
}
