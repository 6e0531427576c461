// Internal declarations shared by the translation units of libflexlink.
#ifndef FLEXLINK_INTERNAL_H
#define FLEXLINK_INTERNAL_H

#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <vector>

#include "flexlink.h"

namespace flex {

// Records a message for flex_last_error() and returns `status`.
int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

void balancer_cfg_default(flex_balancer_cfg_t* c);

// Cut between the device part [0, split) and the host part [split, count).
inline uint64_t partition(uint64_t count, uint32_t host_units, uint32_t share_total, uint32_t align,
                          uint64_t min_count) {
    if (host_units == 0 || count < min_count || count < align) return count;
    if (host_units >= share_total) return 0;
    uint64_t owed = (uint64_t)(((unsigned __int128)count * host_units) / share_total);
    uint64_t split = ((count - owed) / align) * align;
    if (split == count) split = count - align;
    return split;
}

// The same cut for several auxiliary paths.  Path p carries elements
// [start[p], start[p+1]); start[0] = 0 and start[npaths] = count.  The last
// path takes the end of the message, the one before it the piece in front of
// that, and so on; what is left at the front is the primary path's.  Each
// auxiliary path p >= 1 is owed floor(count * units[p] / share_total) elements,
// its start is rounded down to a multiple of `align` (never below 0), and a
// non-zero share never yields an empty piece.  units[0] is ignored.
inline void partition_paths(uint64_t count, const uint32_t* units, int npaths, uint32_t share_total,
                            uint32_t align, uint64_t min_count, uint64_t* start) {
    uint64_t end = count;
    start[npaths] = count;
    for (int p = npaths - 1; p >= 1; --p) {
        uint64_t s = end;
        if (units[p] > 0 && count >= min_count && count >= align) {
            uint64_t owed = (uint64_t)(((unsigned __int128)count * units[p]) / share_total);
            s = end > owed ? ((end - owed) / align) * align : 0;
            if (s == end) s = end >= align ? ((end - 1) / align) * align : 0;
        }
        start[p] = s;
        end = s;
    }
    start[0] = 0;
}

// Algorithm 1 as a state machine plus the Stage-2 window logic.
struct Balancer {
    struct Sample {
        double t[FLEX_MAX_PATHS];
    };
    flex_balancer_cfg_t cfg;
    int npaths = 0;
    uint32_t shares[FLEX_MAX_PATHS] = {0, 0, 0, 0};
    uint32_t active_mask = 0;
    uint32_t stage = FLEX_STAGE_TUNING;
    uint32_t tune_iters = 0;
    uint32_t step = 0;
    uint32_t stability_count = 0;
    int32_t prev_slowest = -1;
    uint64_t adjustments = 0;
    std::vector<Sample> window;

    bool init_from_bandwidth(int np, const double* bw, const flex_balancer_cfg_t& c);
    bool init_from_shares(int np, const uint32_t* s, const flex_balancer_cfg_t& c);
    bool update(const double* T);  // false: bad times, state unchanged
    void finish_tuning();
    void revert_to_primary();
    void get(flex_balancer_state_t* o) const;

   private:
    void end_tuning_if_done(bool stable);
    void slowest_fastest(const double* T, int* slow, int* fast) const;
    uint32_t move_share(int slow, int fast, uint32_t amount);  // units moved
    bool times_ok(const double* T) const;
};

// Step sizes of a host part of `bytes` bytes per peer (see flex_pipeline_plan):
// min_step, 2 min_step, ... up to chunk, chunk ..., and back down, every step a
// multiple of 256 bytes, the last one also taking the left-over bytes.
inline std::vector<uint64_t> plan_steps(uint64_t bytes, uint64_t chunk, uint64_t min_step) {
    std::vector<uint64_t> steps;
    if (bytes == 0) return steps;
    min_step = std::max<uint64_t>((min_step + 255) / 256 * 256, 256);
    if (min_step > chunk) min_step = chunk;
    const uint64_t whole = bytes / 256 * 256, loose = bytes - whole;
    // the ramp: sizes below chunk, doubling
    std::vector<uint64_t> ramp;
    for (uint64_t s = min_step; s < chunk; s *= 2) ramp.push_back(s);
    size_t levels = 0;
    uint64_t in_ramps = 0;
    while (levels < ramp.size() && in_ramps + 2 * ramp[levels] <= whole) in_ramps += 2 * ramp[levels++];
    for (size_t k = 0; k < levels; ++k) steps.push_back(ramp[k]);
    // what the two ramps leave, in even pieces of at most chunk bytes
    const uint64_t middle = whole - in_ramps;
    if (middle > 0) {
        const uint64_t pieces = (middle + chunk - 1) / chunk;
        const uint64_t each = ((middle + pieces - 1) / pieces + 255) / 256 * 256;
        for (uint64_t done = 0; done < middle; done += each) steps.push_back(std::min(each, middle - done));
    }
    for (size_t k = levels; k-- > 0;) steps.push_back(ramp[k]);
    if (loose > 0) {
        if (!steps.empty() && steps.back() + loose <= chunk)
            steps.back() += loose;
        else
            steps.push_back(loose);
    }
    return steps;
}

// ---- device path launchers (defined in reduce_n.hip / gather_copy.hip) ----

struct LaunchShape {
    uint32_t threads;       // workgroup size: 64 (one tile of 1 KiB per workgroup) or 256
    uint32_t unroll;        // copy kernel: 16-byte vectors in flight per thread (1, 2, 4 or 6)
    uint32_t nontemporal;   // bit 0: loads, bit 1: stores
    uint32_t num_cus;       // compute units of the device
    uint32_t max_blocks;    // 0 = one workgroup per tile; else the grid is this many workgroups striding over the tiles
    // The grid is made 2^block_shift times larger and only every 2^block_shift-th
    // workgroup works: 3 keeps the working workgroups on one of the 8 dies.
    uint32_t block_shift = 0;
    // Reduce kernel: a launch of at least this many wavefront tiles (1 KiB per
    // input) and at least serial_min_inputs inputs keeps one load in flight per
    // wavefront instead of all of a tile's loads (0 tiles = never).
    uint32_t serial_min_tiles = 0;
    uint32_t serial_min_inputs = 1;
    // Bytes of LDS reserved per workgroup.  The kernels use no LDS: the reservation
    // only caps how many workgroups a compute unit holds at once (160 KiB / lds_bytes).
    uint32_t lds_bytes = 0;
    // Reduce kernel: the reservation used instead when a launch takes the serial
    // load schedule, has at least cap_min_inputs inputs and reads (inputs + output)
    // at least cap_min_tiles_per_cu wavefront tiles of 1 KiB per compute unit.
    uint32_t serial_lds_bytes = 0;
    uint32_t cap_min_tiles_per_cu = 2048;  // 8 inputs: 57 MiB of bf16 per rank on 256 compute units
    uint32_t cap_min_inputs = 4;
};

// Enqueue out[i] = sum over r (rank order) of in[r][i], i in [0, count), on
// `stream`.  Pointers are device pointers with no alignment requirement.
// Returns a hipError_t value as int (0 = success).
int launch_reduce_n(const void* const* in, int n, void* out, size_t count, int dtype,
                    const LaunchShape& shape, void* stream);

// Enqueue, for r in [0, n): copy bytes[r] bytes from src[r] to dst[r] on
// `stream`; pairs with src[r] == dst[r] or bytes[r] == 0 are skipped.
int launch_gather_copy(const void* const* src, void* const* dst, const uint64_t* bytes, int n,
                       const LaunchShape& shape, void* stream);

inline size_t dtype_size(int dtype) {
    return dtype == FLEX_F32 ? 4 : (dtype == FLEX_BF16 || dtype == FLEX_F16) ? 2 : 0;
}

}  // namespace flex

#endif
