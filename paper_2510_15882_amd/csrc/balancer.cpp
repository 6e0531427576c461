// Two-stage load balancer: Algorithm 1 ("Initial Coarse-Grained Load Tuning")
// as a state machine fed one measurement at a time, followed by the runtime
// stage of Section "Stage 2: Runtime Fine-Grained Adjustment".  Host code only.
#include "flexlink_internal.h"

#include <algorithm>
#include <cmath>
#include <new>

namespace flex {

void balancer_cfg_default(flex_balancer_cfg_t* c) {
    c->share_total = 10000;
    c->initial_step = 16;
    c->stability_required = 3;
    c->max_tune_iters = 100;
    c->window = 10;
    c->runtime_step = 4;
    c->aux_share_cap = 0;
    c->reserved = 0;
    c->convergence_threshold = 0.05;
    c->runtime_threshold = 0.10;
}

static bool cfg_ok(const flex_balancer_cfg_t& c) {
    return c.share_total > 0 && c.initial_step > 0 && c.window > 0 && c.window <= 4096 &&
           c.runtime_step > 0 && std::isfinite(c.convergence_threshold) &&
           std::isfinite(c.runtime_threshold);
}

bool Balancer::init_from_shares(int np, const uint32_t* s, const flex_balancer_cfg_t& c) {
    if (np < 1 || np > FLEX_MAX_PATHS || !cfg_ok(c)) return false;
    uint64_t sum = 0;
    for (int p = 0; p < np; ++p) sum += s[p];
    if (sum != c.share_total) return false;
    cfg = c;
    npaths = np;
    active_mask = 0;
    for (int p = 0; p < FLEX_MAX_PATHS; ++p) shares[p] = 0;
    for (int p = 0; p < np; ++p) {
        shares[p] = s[p];
        if (s[p] > 0) active_mask |= 1u << p;
    }
    stage = FLEX_STAGE_TUNING;
    tune_iters = 0;
    step = c.initial_step;
    stability_count = 0;
    prev_slowest = -1;
    adjustments = 0;
    window.clear();
    end_tuning_if_done(false);
    return true;
}

bool Balancer::init_from_bandwidth(int np, const double* bw, const flex_balancer_cfg_t& c) {
    if (np < 1 || np > FLEX_MAX_PATHS || !cfg_ok(c)) return false;
    double rate[FLEX_MAX_PATHS];
    double denom = 0.0;
    for (int p = 0; p < np; ++p) {
        if (!std::isfinite(bw[p])) return false;
        rate[p] = bw[p] > 0 ? bw[p] : 0.0;
        denom = denom + rate[p];
    }
    if (!(rate[0] > 0)) return false;
    uint32_t s[FLEX_MAX_PATHS] = {0, 0, 0, 0};
    uint32_t used = 0;
    for (int p = 1; p < np; ++p) {
        s[p] = (uint32_t)std::floor((double)c.share_total * rate[p] / denom);
        used += s[p];
    }
    s[0] = c.share_total - used;
    return init_from_shares(np, s, c);
}

// The loop of Algorithm 1 stops before measuring when only the primary path is
// active, and after max_tune_iters measurements.
void Balancer::end_tuning_if_done(bool stable) {
    if (stage != FLEX_STAGE_TUNING) return;
    if (stable || active_mask == 1u || tune_iters >= cfg.max_tune_iters) {
        stage = FLEX_STAGE_RUNTIME;
        window.clear();
    }
}

void Balancer::slowest_fastest(const double* T, int* slow, int* fast) const {
    int s = -1, f = -1;
    for (int p = 0; p < npaths; ++p) {
        if (!(active_mask & (1u << p))) continue;
        if (s < 0 || T[p] > T[s]) s = p;   // ties: lowest index
        if (f < 0 || T[p] < T[f]) f = p;
    }
    *slow = s;
    *fast = f;
}

// One share transfer with the primary-first rule shared by both stages: the
// slowest path gives; the primary receives unless it is itself the slowest (or
// inactive), in which case the fastest path receives.  An auxiliary receiver
// is never filled beyond cfg.aux_share_cap (0 = no ceiling).
uint32_t Balancer::move_share(int slow, int fast, uint32_t amount) {
    int target = (slow != 0 && (active_mask & 1u)) ? 0 : fast;
    uint32_t m = std::min(amount, shares[slow]);
    if (target != 0 && cfg.aux_share_cap > 0) {
        uint32_t room = shares[target] < cfg.aux_share_cap ? cfg.aux_share_cap - shares[target] : 0;
        m = std::min(m, room);
    }
    shares[slow] -= m;
    shares[target] += m;
    if (shares[slow] == 0) active_mask &= ~(1u << slow);
    return m;
}

bool Balancer::times_ok(const double* T) const {
    for (int p = 0; p < npaths; ++p)
        if ((active_mask & (1u << p)) && !(std::isfinite(T[p]) && T[p] > 0)) return false;
    return true;
}

bool Balancer::update(const double* T) {
    if (!times_ok(T)) return false;
    if (stage == FLEX_STAGE_TUNING) {
        int slow, fast;
        slowest_fastest(T, &slow, &fast);
        double imbalance = (T[slow] - T[fast]) / T[fast];
        bool stable = false;
        ++tune_iters;
        if (imbalance < cfg.convergence_threshold) {
            ++stability_count;
            stable = stability_count >= cfg.stability_required;
        } else {
            const uint32_t calm_before = stability_count;
            stability_count = 0;
            if (prev_slowest >= 0 && slow != prev_slowest) step = std::max(step / 2, 1u);
            if (move_share(slow, fast, step) == 0) {
                // the receiver sits at its ceiling: nothing can change any more
                stability_count = calm_before + 1;
                stable = stability_count >= cfg.stability_required;
            }
            prev_slowest = slow;
        }
        end_tuning_if_done(stable);
        return true;
    }
    // Stage 2: Evaluator window, Load Balancer every cfg.window samples.
    Sample smp;
    for (int p = 0; p < FLEX_MAX_PATHS; ++p) smp.t[p] = p < npaths ? T[p] : 0.0;
    window.push_back(smp);
    if (window.size() < cfg.window) return true;
    double med[FLEX_MAX_PATHS] = {0, 0, 0, 0};
    int nactive = 0;
    std::vector<double> col(window.size());
    for (int p = 0; p < npaths; ++p) {
        if (!(active_mask & (1u << p))) continue;
        ++nactive;
        for (size_t k = 0; k < window.size(); ++k) col[k] = window[k].t[p];
        std::sort(col.begin(), col.end());
        size_t n = col.size();
        med[p] = (n & 1) ? col[n / 2] : (col[n / 2 - 1] + col[n / 2]) / 2.0;
    }
    window.clear();
    if (nactive < 2) return true;
    int slow, fast;
    slowest_fastest(med, &slow, &fast);
    double gap = (med[slow] - med[fast]) / med[fast];
    if (gap > cfg.runtime_threshold && move_share(slow, fast, cfg.runtime_step) > 0) ++adjustments;
    return true;
}

void Balancer::finish_tuning() {
    if (stage == FLEX_STAGE_TUNING) {
        stage = FLEX_STAGE_RUNTIME;
        window.clear();
    }
}

void Balancer::revert_to_primary() {
    for (int p = 1; p < npaths; ++p) {
        shares[0] += shares[p];
        shares[p] = 0;
    }
    active_mask = 1u;
    finish_tuning();
}

void Balancer::get(flex_balancer_state_t* o) const {
    o->npaths = (uint32_t)npaths;
    o->stage = stage;
    o->tune_iters = tune_iters;
    o->step = step;
    o->stability_count = stability_count;
    o->prev_slowest = prev_slowest;
    o->active_mask = active_mask;
    o->window_fill = (uint32_t)window.size();
    o->adjustments = adjustments;
    for (int p = 0; p < FLEX_MAX_PATHS; ++p) o->shares[p] = shares[p];
}

}  // namespace flex

struct flex_balancer {
    flex::Balancer impl;
};

extern "C" {

int flex_balancer_cfg_default(flex_balancer_cfg_t* cfg) {
    if (!cfg) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_balancer_cfg_default: cfg is NULL");
    flex::balancer_cfg_default(cfg);
    return FLEX_OK;
}

static int make_balancer(flex_balancer_t** b, const flex_balancer_cfg_t* cfg, flex_balancer_cfg_t* use) {
    if (!b) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_balancer_init: b is NULL");
    *b = nullptr;
    if (cfg)
        *use = *cfg;
    else
        flex::balancer_cfg_default(use);
    flex_balancer* o = new (std::nothrow) flex_balancer;
    if (!o) return flex::fail(FLEX_ERR_NOMEM, "flex_balancer_init: out of host memory");
    *b = o;
    return FLEX_OK;
}

int flex_balancer_init(flex_balancer_t** b, int npaths, const double* path_bw,
                       const flex_balancer_cfg_t* cfg) {
    if (!path_bw) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_balancer_init: path_bw is NULL");
    flex_balancer_cfg_t use;
    int st = make_balancer(b, cfg, &use);
    if (st) return st;
    if (!(*b)->impl.init_from_bandwidth(npaths, path_bw, use)) {
        delete *b;
        *b = nullptr;
        return flex::fail(FLEX_ERR_INVALID_ARG,
                          "flex_balancer_init: npaths, rates or configuration out of range");
    }
    return FLEX_OK;
}

int flex_balancer_init_shares(flex_balancer_t** b, int npaths, const uint32_t* shares,
                              const flex_balancer_cfg_t* cfg) {
    if (!shares) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_balancer_init_shares: shares is NULL");
    flex_balancer_cfg_t use;
    int st = make_balancer(b, cfg, &use);
    if (st) return st;
    if (npaths < 1 || npaths > FLEX_MAX_PATHS || !(*b)->impl.init_from_shares(npaths, shares, use)) {
        delete *b;
        *b = nullptr;
        return flex::fail(FLEX_ERR_INVALID_ARG,
                          "flex_balancer_init_shares: shares must sum to share_total; npaths in 1..4");
    }
    return FLEX_OK;
}

int flex_balancer_update(flex_balancer_t* b, const double* path_time_s, uint32_t* shares_out) {
    if (!b || !path_time_s) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_balancer_update: NULL argument");
    if (!b->impl.update(path_time_s))
        return flex::fail(FLEX_ERR_INVALID_ARG,
                          "flex_balancer_update: every active path needs a finite time > 0");
    if (shares_out)
        for (int p = 0; p < b->impl.npaths; ++p) shares_out[p] = b->impl.shares[p];
    return FLEX_OK;
}

int flex_balancer_finish_tuning(flex_balancer_t* b) {
    if (!b) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_balancer_finish_tuning: b is NULL");
    b->impl.finish_tuning();
    return FLEX_OK;
}

int flex_balancer_revert_to_primary(flex_balancer_t* b) {
    if (!b) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_balancer_revert_to_primary: b is NULL");
    b->impl.revert_to_primary();
    return FLEX_OK;
}

int flex_balancer_get(const flex_balancer_t* b, flex_balancer_state_t* out) {
    if (!b || !out) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_balancer_get: NULL argument");
    b->impl.get(out);
    return FLEX_OK;
}

int flex_balancer_destroy(flex_balancer_t* b) {
    delete b;
    return FLEX_OK;
}

int flex_struct_sizes(size_t* out) {
    if (!out) return flex::fail(FLEX_ERR_INVALID_ARG, "flex_struct_sizes: out is NULL");
    out[0] = sizeof(flex_balancer_cfg_t);
    out[1] = sizeof(flex_balancer_state_t);
    out[2] = sizeof(flex_config_t);
    out[3] = sizeof(flex_stats_t);
    out[4] = sizeof(flex_tune_result_t);
    out[5] = sizeof(flex_tune_round_t);
    return FLEX_OK;
}

int flex_partition(uint64_t count, uint32_t host_units, uint32_t share_total, uint32_t align_elems,
                   uint64_t min_count, uint64_t* split_out) {
    if (!split_out || share_total == 0 || align_elems == 0 || host_units > share_total)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_partition: argument out of range");
    *split_out = flex::partition(count, host_units, share_total, align_elems, min_count);
    return FLEX_OK;
}

int flex_partition_paths(uint64_t count, const uint32_t* units, int npaths, uint32_t share_total,
                         uint32_t align_elems, uint64_t min_count, uint64_t* start_out) {
    if (!units || !start_out || npaths < 1 || npaths > FLEX_MAX_PATHS || share_total == 0 || align_elems == 0)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_partition_paths: argument out of range");
    uint64_t sum = 0;
    for (int p = 1; p < npaths; ++p) sum += units[p];
    if (sum > share_total)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_partition_paths: shares exceed share_total");
    flex::partition_paths(count, units, npaths, share_total, align_elems, min_count, start_out);
    return FLEX_OK;
}

int flex_pipeline_plan(uint64_t bytes, uint64_t chunk_bytes, uint64_t min_step_bytes, uint64_t* steps,
                       uint32_t max_steps, uint32_t* nsteps) {
    if (!nsteps || chunk_bytes < 512 || chunk_bytes % 256 || min_step_bytes == 0)
        return flex::fail(FLEX_ERR_INVALID_ARG, "flex_pipeline_plan: argument out of range");
    const std::vector<uint64_t> plan = flex::plan_steps(bytes, chunk_bytes, min_step_bytes);
    *nsteps = (uint32_t)plan.size();
    for (size_t k = 0; steps && k < plan.size() && k < max_steps; ++k) steps[k] = plan[k];
    return FLEX_OK;
}

}  // extern "C"
