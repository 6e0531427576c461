/*
 * flexlink.h - C ABI of the MI355X-native local share of FlexLink's collectives.
 *
 * FlexLink (arXiv 2510.15882) splits every AllReduce / AllGather message over
 * several heterogeneous paths in proportion to a share vector and keeps that
 * vector balanced with a two-stage load balancer (paper: Design; Section
 * "Communicator"; Section "Two-Stage Load Balancing Strategy"; Algorithm 1).
 *
 * This library builds the part of that which one GPU can show.  The N ranks'
 * contributions are N buffers resident in one GPU's HBM.  Two paths exist:
 *
 *   FLEX_PATH_DEVICE  the on-device path (HIP kernels reading the rank buffers
 *                     straight from HBM); it plays the role the paper gives to
 *                     NVLink, i.e. it is the primary path the balancer favours;
 *   FLEX_PATH_HOST    the host-staged path of Section "Communicator": peer
 *                     data goes device -> pinned host buffer -> device through
 *                     a double-buffered pipeline on side streams.
 *   FLEX_PATH_HOST2   optional (num_aux_paths = 2): a second host-staged path
 *                     with its own pinned ring and streams, driven by the other
 *                     engine (copy kernels vs DMA engines).  It shares the PCIe
 *                     link with FLEX_PATH_HOST the way the paper's RDMA NIC
 *                     shares the PCIe switch with its PCIe path (Section
 *                     "Observation: Inefficiency of Intra-node PCIe
 *                     Communication"), and gives the balancer three paths.
 *
 * General conventions
 *   - Every function returns a flex_status code (0 = FLEX_OK) unless stated
 *     otherwise, never throws and never aborts.  After a non-zero return,
 *     flex_last_error() gives a message for the calling thread.
 *   - "device pointer" = address in the HBM of the current HIP device;
 *     "host pointer" = ordinary process memory.  Each argument says which.
 *   - The caller owns every buffer it passes in.  The library owns what a
 *     flex_comm_t holds: pinned transit buffers, device scratch, side streams,
 *     events, balancer state.
 *   - Collective calls are asynchronous: they enqueue work on the caller's HIP
 *     stream (side streams fork from it and join back into it by events) and
 *     return.  Stream order is the only synchronisation the caller sees; any
 *     number of calls may be queued back to back on one stream.
 *   - Stream capture: a collective call whose whole message takes the device
 *     path (host share 0, or a message too short to split) only launches one
 *     kernel on the caller's stream and may be captured into a HIP graph.  A
 *     call that would use a host path returns FLEX_ERR_STATE on a capturing
 *     stream and enqueues nothing (its timing events are read back by the
 *     host, which a graph replay cannot serve).
 *   - A flex_comm_t is bound to the HIP device that was current at creation
 *     and is not thread-safe; use one per thread/stream.
 *   - Structs are plain C with fixed-width fields; obtain defaults with the
 *     *_default() call and then change fields.
 */
#ifndef FLEXLINK_H
#define FLEXLINK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FLEX_MAX_RANKS 8
#define FLEX_MAX_PATHS 4

typedef struct flex_comm flex_comm_t;         /* opaque; device-bound */
typedef struct flex_balancer flex_balancer_t; /* opaque; pure host state */

enum flex_status {
    FLEX_OK = 0,
    FLEX_ERR_INVALID_ARG = 1, /* null pointer, size or index out of range; nothing was enqueued */
    FLEX_ERR_UNSUPPORTED = 2, /* unknown dtype / op / collective; nothing was enqueued */
    FLEX_ERR_HIP = 3,         /* a HIP runtime call failed; see flex_last_error() */
    FLEX_ERR_NOMEM = 4,       /* host or device allocation failed */
    FLEX_ERR_STATE = 5        /* call not valid in the object's current state */
};

enum flex_dtype { FLEX_F32 = 0, FLEX_BF16 = 1, FLEX_F16 = 2 };
enum flex_op { FLEX_SUM = 0 };
enum flex_coll { FLEX_ALLREDUCE = 0, FLEX_ALLGATHER = 1, FLEX_REDUCESCATTER = 2, FLEX_ALLTOALL = 3 };
enum flex_path { FLEX_PATH_DEVICE = 0, FLEX_PATH_HOST = 1, FLEX_PATH_HOST2 = 2 };
enum flex_split_mode { FLEX_SPLIT_STATIC = 0, FLEX_SPLIT_ADAPTIVE = 1 };
enum flex_balancer_stage { FLEX_STAGE_TUNING = 1, FLEX_STAGE_RUNTIME = 2 };

/* ------------------------------------------------------------------------
 * Load balancer (paper: Section "Two-Stage Load Balancing Strategy",
 * Algorithm 1 for Stage 1, Section "Stage 2: Runtime Fine-Grained Adjustment"
 * for Stage 2).  Pure host code: no HIP call is made by any flex_balancer_*
 * function, so they work on a machine without a GPU.
 *
 * Shares are non-negative integers summing to share_total.  Path 0 is the
 * primary path (NVLink in the paper, the device path here).
 * ---------------------------------------------------------------------- */
typedef struct flex_balancer_cfg {
    uint32_t share_total;          /* units the message is divided into (default 10000) */
    uint32_t initial_step;         /* Algorithm 1 INITIAL_ADJUSTMENT_STEP, in units (default 16: on one GPU the
                                      balanced host share is 30-90 units, a coarser step drains it in one move) */
    uint32_t stability_required;   /* Algorithm 1 STABILITY_REQUIRED (default 3) */
    uint32_t max_tune_iters;       /* Algorithm 1 loop bound (paper: 100) */
    uint32_t window;               /* Stage 2: calls per Evaluator window = Load Balancer period (default 10) */
    uint32_t runtime_step;         /* Stage 2: fixed share moved per adjustment, in units (default 4) */
    uint32_t aux_share_cap;        /* 0 = none (the paper's method unchanged); else no auxiliary path is ever
                                      filled beyond this many units: a transfer is trimmed to the room left,
                                      and a transfer trimmed to nothing leaves the shares alone (Stage 1 counts
                                      such an iteration as a stable one) */
    uint32_t reserved;
    double convergence_threshold;  /* Algorithm 1 CONVERGENCE_THRESHOLD on (Tslow-Tfast)/Tfast (default 0.05) */
    double runtime_threshold;      /* Stage 2 threshold on the same ratio of window medians (default 0.10) */
} flex_balancer_cfg_t;

typedef struct flex_balancer_state {
    uint32_t npaths;
    uint32_t stage;                /* flex_balancer_stage */
    uint32_t tune_iters;           /* Algorithm 1 iterations measured so far */
    uint32_t step;                 /* current Algorithm 1 step */
    uint32_t stability_count;
    int32_t prev_slowest;          /* -1 = none yet */
    uint32_t active_mask;          /* bit p set = path p active */
    uint32_t window_fill;          /* Stage 2 samples held in the current window */
    uint64_t adjustments;          /* Stage 2 moves made so far */
    uint32_t shares[FLEX_MAX_PATHS];
} flex_balancer_state_t;

/* Fill *cfg (host pointer) with the defaults listed above. */
int flex_balancer_cfg_default(flex_balancer_cfg_t* cfg);

/* Create a balancer in Stage 1 with bandwidth-proportional starting shares
 * (Algorithm 1's InitializeShares step: the primary path starts with the
 * largest share).
 *   b        host pointer; receives the new object (caller destroys it).
 *   npaths   1..FLEX_MAX_PATHS.
 *   path_bw  host array of npaths rates, same unit for all: how fast path p
 *            moves a whole message on its own; <= 0 marks a path unavailable.
 *            Every path p >= 1 gets floor(total * bw[p] / sum(bw)) units, path 0
 *            the rest; a path with 0 units starts inactive.
 *   cfg      host pointer or NULL for defaults.
 * Errors: INVALID_ARG (null b/path_bw, npaths out of range, bw[0] <= 0,
 * non-finite rates, zero share_total/window/initial_step), NOMEM. */
int flex_balancer_init(flex_balancer_t** b, int npaths, const double* path_bw,
                       const flex_balancer_cfg_t* cfg);

/* Same, but start from explicit shares (host array of npaths units that must
 * sum to cfg->share_total). */
int flex_balancer_init_shares(flex_balancer_t** b, int npaths, const uint32_t* shares,
                              const flex_balancer_cfg_t* cfg);

/* Feed one measurement of per-path completion times and get the shares to use
 * next.
 *   path_time_s  host array of npaths seconds; entries of inactive paths are
 *                ignored; every active path must report a finite time > 0.
 *   shares_out   host array of npaths units, may be NULL.
 * In Stage 1 one call is one iteration of Algorithm 1's loop body (find slowest
 * and fastest active path, test the imbalance, move `step` units from the
 * slowest path to the primary path, or from a bottlenecked primary path to the
 * fastest one, halve the step when the bottleneck moved, deactivate a drained
 * path).  When the loop's exit condition holds (stable for stability_required
 * iterations, only the primary path left, or max_tune_iters reached) the
 * balancer moves to Stage 2.  In Stage 2 each call adds a sample to the
 * Evaluator window; the call that fills the window compares the window medians
 * and moves at most runtime_step units by the same source/target rule.
 * Errors: INVALID_ARG (null, bad time for an active path): state unchanged. */
int flex_balancer_update(flex_balancer_t* b, const double* path_time_s, uint32_t* shares_out);

/* End Stage 1 now (no-op in Stage 2): later updates are Stage-2 samples. */
int flex_balancer_finish_tuning(flex_balancer_t* b);

/* Give every auxiliary path's share back to the primary path, deactivate them
 * and end Stage 1: the state Algorithm 1 itself ends in once the primary path
 * is the only active one.  Used when the split, however balanced, is no faster
 * than the primary path alone (paper, Section "Two-Stage Load Balancing
 * Strategy": the system then falls back to the primary-only baseline). */
int flex_balancer_revert_to_primary(flex_balancer_t* b);

/* Copy the balancer's state to *out (host pointer). */
int flex_balancer_get(const flex_balancer_t* b, flex_balancer_state_t* out);

/* Free the object.  NULL is accepted. */
int flex_balancer_destroy(flex_balancer_t* b);

/* ------------------------------------------------------------------------
 * Message partition (paper: Design - the Communicator divides each payload
 * over the paths according to the shares and runs them concurrently).
 *
 * Computes the cut between the device part [0, split) and the host part
 * [split, count) of a message of `count` elements for a host share of
 * host_units / share_total:  the host part is owed floor(count*host_units/
 * share_total) elements; the cut is rounded down to a multiple of align_elems
 * (so the host part only grows by rounding, and the ragged end of the message
 * belongs to it); host_units == 0, count < min_count or count < align_elems
 * gives split == count; host_units == share_total gives split == 0; a non-zero
 * share never yields an empty host part.  Pure host arithmetic.
 * Errors: INVALID_ARG (null split_out, host_units > share_total, zero
 * share_total or align_elems). */
int flex_partition(uint64_t count, uint32_t host_units, uint32_t share_total,
                   uint32_t align_elems, uint64_t min_count, uint64_t* split_out);

/* The same partition for npaths paths (1..FLEX_MAX_PATHS).
 *   units      host array of npaths shares; units[0] (the primary path) is
 *              ignored: the primary path gets what the others leave.
 *   start_out  host array of npaths + 1 element offsets: path p carries
 *              [start_out[p], start_out[p+1]); start_out[0] = 0,
 *              start_out[npaths] = count.
 * The last path takes the end of the message, the one before it the piece in
 * front of that, and so on, each by the rule of flex_partition (owed
 * floor(count * units[p] / share_total), start rounded down to align_elems,
 * never empty for a non-zero share).  With npaths = 2 it gives flex_partition's
 * cut.  Errors: INVALID_ARG (null, npaths out of range, shares above
 * share_total, zero share_total or align_elems). */
int flex_partition_paths(uint64_t count, const uint32_t* units, int npaths, uint32_t share_total,
                         uint32_t align_elems, uint64_t min_count, uint64_t* start_out);

/* ------------------------------------------------------------------------
 * Communicator (paper: Section "Communicator").
 * ---------------------------------------------------------------------- */
enum flex_host_engine {
    FLEX_ENGINE_KERNEL = 0, /* default: both stages are small HIP kernels that write to / read from the pinned
                               buffer over PCIe; for AllReduce the second stage is the reduce kernel itself,
                               reading the peers straight from pinned memory.  Lowest latency (about 55 us
                               for the first byte) and, with the workgroup counts below, the steadiest rate
                               in both directions at once on MI355X */
    FLEX_ENGINE_HYBRID = 1, /* producer stage: the same copy kernel; consumer stage: one hipMemcpyAsync (DMA
                               engine) brings the slot back into a device staging buffer, and a kernel reduces
                               from there (AllReduce) or places the pieces (AllGather).  Holds no compute
                               units while the data comes back; about 180 us for the first byte, and its
                               rate varies from box to box and drops when calls are queued back to back */
    FLEX_ENGINE_SDMA = 2    /* both stages are hipMemcpyAsync copies (DMA engines), one per peer and step;
                               AllReduce then reduces once from a device scratch buffer.  A DMA engine
                               writes host memory at half the rate of a copy kernel on MI355X */
};

enum flex_slot_sync {
    FLEX_SYNC_EVENTS = 0,   /* slot hand-over by HIP events (default) */
    FLEX_SYNC_COUNTERS = 1  /* slot hand-over by the paper's monotonically increasing counters and
                               stream memory operations (Section "Communicator"): for use i of a slot
                               the producer waits semEmpty >= i, fills the slot, writes semFull = i+1;
                               the consumer waits semFull >= i+1, drains it, writes semEmpty = i+1 */
};

enum flex_launch_shape {
    FLEX_SHAPE_WAVE = 0,    /* default: one wavefront (64 threads) per workgroup, one workgroup per 1 KiB
                               tile of each input; best or within 2 % at every size measured on MI355X */
    FLEX_SHAPE_BLOCK = 1    /* 256-thread workgroups, one per 4 KiB tile: the one alternate that wins
                               anywhere (about 10 % on AllReduce messages around 2 MiB per rank) */
};

typedef struct flex_config {
    uint32_t struct_size;        /* sizeof(flex_config_t) as the caller's header declares it.
                                    flex_config_default() fills it in; flex_comm_create() refuses any other
                                    value, so a caller built against another layout fails loudly */
    uint32_t num_slots;          /* transit slots in the ring; 2 (default) = the paper's double buffering */
    uint64_t chunk_bytes;        /* transit buffer bytes per peer and pipeline step (paper: 4 MB; default
                                    4 MiB); one pinned slot holds (nranks-1) * chunk_bytes */
    uint64_t min_split_bytes;    /* messages shorter than this per rank are never split (default 64 KiB) */
    uint32_t max_host_units;     /* largest share one host path may carry (default 2500 = 25 %); sizes the
                                    FLEX_ENGINE_SDMA scratch and is the balancers' aux_share_cap */
    uint32_t split_align_elems;  /* alignment of the cut, elements (default 2048) */
    uint32_t tune_reps;          /* collective calls per MeasurePathTimings in flex_comm_tune (default 5) */
    uint32_t probe_units;        /* host share used to measure the host path's rate (default 200) */
    uint32_t tune_accept_check;  /* 1 (default): flex_comm_tune keeps the tuned split only if it is faster
                                    than the device path alone by a margin the noise cannot explain */
    uint32_t accept_pairs;       /* acceptance check: interleaved (split, device-only) measurement pairs of
                                    tune_reps calls each (default 3, at least 1) */
    uint32_t launch_shape;       /* flex_launch_shape of the two device-path kernels */
    uint32_t reduce_serial_loads;/* device-path reduce kernel.  2 = a wavefront keeps one load in flight and asks
                                    for input r+1 only when input r has arrived; 0 = all N loads of a tile are
                                    issued before the first add; 1 (default) = the first for launches of at
                                    least 16 tiles per compute unit (4 MiB of bf16 per rank on MI355X) with
                                    three or more ranks, the second for shorter ones and for two ranks */
    uint32_t reduce_nontemporal; /* streaming hints of the reduce kernel: 0 none, 1 non-temporal loads,
                                    3 (default) non-temporal loads and stores.  Plain stores let a reused
                                    output stay in the 256 MB memory-side cache (an nccl-tests style loop) */
    uint32_t copy_nontemporal;   /* same for the copy kernel */
    uint32_t reduce_lds_reserve; /* bytes of LDS reserved per workgroup of the device-path reduce kernel when it
                                    takes the one-load-in-flight schedule on a long launch (four or more
                                    ranks, at least 2 MiB read per compute unit: 57 MiB of bf16 per rank with
                                    8 ranks).  Default 5632; 0 = none.  The kernel uses no LDS: the reservation
                                    caps the wavefronts a compute unit holds at 160 KiB / reserve = 29 instead
                                    of 32, which on MI355X makes such launches 2-4 % faster (any value from
                                    5200 to 6400 does; short launches, two and three ranks, the all-in-flight
                                    schedule and the copy kernel lose with it and are launched without) */
    uint32_t reserved;
    uint32_t host_engine;        /* flex_host_engine of the first host path (default FLEX_ENGINE_KERNEL; the
                                    engine with hipMemcpyAsync in both directions is FLEX_ENGINE_SDMA) */
    uint32_t host_blocks;        /* workgroups (of 256 threads) of the producer-stage copy kernel, which writes
                                    pinned memory (default 8: two already fill the link) */
    uint32_t host_die_shift;     /* 0 = host-path workgroups spread over all 8 accelerator dies; 1..3 = their
                                    grids are 2^shift times larger and only every 2^shift-th workgroup works,
                                    which keeps them on 4, 2 (default) or 1 of the dies and disturbs the device
                                    path less */
    uint32_t min_step_bytes;     /* shortest pipeline step per peer (default 256 KiB): a host part starts and
                                    ends with steps of this size, doubling up to chunk_bytes in between, so
                                    that little of it travels with only one of the two stages busy */
    uint32_t slot_sync;          /* flex_slot_sync (default FLEX_SYNC_EVENTS) */
    uint32_t num_aux_paths;      /* host-staged paths: 1 (default) = FLEX_PATH_HOST with host_engine;
                                    2 = also FLEX_PATH_HOST2 on FLEX_ENGINE_SDMA (on FLEX_ENGINE_KERNEL if the
                                    first one is FLEX_ENGINE_SDMA) */
    uint32_t host_down_blocks;   /* FLEX_ENGINE_KERNEL: workgroups of the consumer-stage reduce kernel, which reads
                                    pinned memory (default 6; measured on MI355X next to 8 producer workgroups:
                                    4 give 34.7, 6 give 41.9, 8 give 38.2, 16 give 31 GB/s each way) */
    uint32_t sample_every;       /* the Evaluator times every sample_every-th split call (default 1: every call, the
                                    window holds consecutive calls as in the paper); the other split calls fork and
                                    join with ordering-only events, which saves about 5 us of the 16 us a split call
                                    costs on top of its kernels.  flex_comm_tune always times every call */
    flex_balancer_cfg_t balancer;
} flex_config_t;

typedef struct flex_stats {
    uint64_t calls;              /* collective calls of this kind since creation */
    uint64_t split_calls;        /* of which used both paths */
    uint64_t samples;            /* per-path timings the Evaluator has read back */
    uint64_t blocking_reads;     /* times the Evaluator had to wait for an old call because its record
                                    ring was full (0 in normal operation) */
    uint64_t last_count;         /* elements per rank of the last call */
    uint64_t last_split;         /* its cut: device part [0,split), host part [split,count) */
    uint32_t mode;               /* flex_split_mode */
    uint32_t static_host_units;
    double last_time_s[FLEX_MAX_PATHS]; /* latest per-path completion times read back (0 = none) */
    double mean_time_s[FLEX_MAX_PATHS]; /* mean over all samples */
    uint32_t npaths;                    /* 1 + number of host-staged paths of this communicator */
    uint32_t static_units[FLEX_MAX_PATHS]; /* static shares per path ([0] unused) */
    uint32_t reserved;
    uint64_t last_start[FLEX_MAX_PATHS];   /* last call: first element of each path's piece */
    flex_balancer_state_t balancer;     /* state for the size class of the queried message
                                           (npaths == 0 if that class has none) */
} flex_stats_t;

typedef struct flex_tune_result {
    double path_bw[FLEX_MAX_PATHS];         /* measured rates, message bytes per second */
    uint32_t initial_shares[FLEX_MAX_PATHS];/* InitializeShares' result */
    uint32_t shares[FLEX_MAX_PATHS];        /* shares after Algorithm 1 and the acceptance check */
    uint32_t active_mask;
    uint32_t iterations;                    /* Algorithm 1 iterations measured */
    double path_time_s[FLEX_MAX_PATHS];     /* last measured per-path times */
    uint32_t balanced_shares[FLEX_MAX_PATHS]; /* shares Algorithm 1 ended with, before the acceptance check */
    /* acceptance check (all 0 if it did not run): whole-call times, events around the call on the
       caller's stream, accept_pairs * tune_reps samples of each kind taken in turns */
    double device_alone_s;                  /* median, whole message on the device path */
    double combined_s;                      /* median, call split at balanced_shares */
    double device_alone_mad_s;              /* median absolute deviation of the device-only samples */
    double combined_mad_s;                  /* same for the split samples */
    uint32_t accept_samples;                /* samples of each kind */
    uint32_t reverted;                      /* 1 = not faster by more than 3 * max(MAD): reverted to device-only */
} flex_tune_result_t;

/* One iteration of Algorithm 1 as flex_comm_tune ran it. */
typedef struct flex_tune_round {
    double path_time_s[FLEX_MAX_PATHS];      /* MeasurePathTimings' result (0 for inactive paths) */
    uint32_t shares_before[FLEX_MAX_PATHS];  /* shares the measurement was taken at */
    uint32_t shares_after[FLEX_MAX_PATHS];   /* shares after the iteration's move */
    uint32_t step_after;
    uint32_t active_after;                   /* bit p = path p still active */
} flex_tune_round_t;

/* Fill *cfg (host pointer) with defaults. */
int flex_config_default(flex_config_t* cfg);

/* Create a communicator on the current HIP device.
 *   comm                host pointer; receives the object.
 *   nranks              simulated ranks, 1..FLEX_MAX_RANKS.
 *   rank                which rank this GPU plays, 0..nranks-1: that rank's
 *                       buffer is local and never takes the host path.
 *   max_bytes_per_rank  largest per-rank message any later call will pass.
 *   cfg                 host pointer or NULL for defaults.
 * Allocates, once, per host path: num_slots pinned slots of (nranks-1) *
 * chunk_bytes, two side streams at default priority (FLEX_ENGINE_HYBRID: one
 * per slot, or three with FLEX_SYNC_COUNTERS), slot events and, by engine,
 * device memory: FLEX_ENGINE_HYBRID num_slots staging buffers of the
 * slot size; FLEX_ENGINE_SDMA a scratch of (nranks-1) * ceil(max_bytes_per_rank
 * * max_host_units / share_total) bytes (rounded up); FLEX_ENGINE_KERNEL none.
 * Plus one ring of timing events.  Nothing is allocated per call afterwards.
 * Errors: INVALID_ARG (also cfg->struct_size != sizeof(flex_config_t)), NOMEM,
 * HIP. */
int flex_comm_create(flex_comm_t** comm, int nranks, int rank, size_t max_bytes_per_rank,
                     const flex_config_t* cfg);

/* Wait for all work this communicator enqueued on its side streams, then free
 * everything it owns.  NULL is accepted. */
int flex_comm_destroy(flex_comm_t* comm);

/* AllReduce(sum), local share (paper: Evaluation, "End-to-End Performance" -
 * ring AllReduce = reduce-scatter with a reduce-sum, then all-gather; the
 * abstract's "lossless": the result is the same whatever the split).
 *   rank_bufs  host array of nranks device pointers; rank_bufs[r] holds rank
 *              r's `count` contiguous elements.  The array itself is only read
 *              during the call.
 *   out        device pointer to `count` elements.
 *   count      elements per rank (0 is allowed: nothing is enqueued).
 *   dtype      FLEX_F32, FLEX_BF16 or FLEX_F16.   op: FLEX_SUM.
 *   hip_stream the caller's hipStream_t (NULL = the default stream).
 * Result, for every i:  out[i] = round(((b0[i] + b1[i]) + b2[i]) + ... ) with
 * the additions done in IEEE binary32, round-to-nearest-even, strictly in rank
 * order starting from rank 0's value, and one final rounding to dtype
 * (bfloat16 and binary16: round-to-nearest-even, subnormals kept; a NaN result
 * is some NaN).  The bits
 * of out do not depend on the split, the chunk size, `rank` or the launch
 * shape.  Elements [0, split) are reduced by the device path on hip_stream;
 * peers' elements [split, count) travel through the pinned transit buffers on
 * the side streams and are reduced there, in the same rank order, together
 * with the local rank's elements read in place.
 * Pointers need element alignment only; fastest when every pointer has the
 * same offset within 16 bytes (any common offset runs at the aligned rate,
 * differing offsets cost 10-25 %).  out may be the same buffer as rank_bufs[rank]; any other overlap
 * between out and an input is undefined.
 * Errors: INVALID_ARG (null comm/rank_bufs/out/any rank pointer with count > 0,
 * count * size > max_bytes_per_rank), UNSUPPORTED (dtype, op), HIP. */
int flex_allreduce_local(flex_comm_t* comm, const void* const* rank_bufs, void* out, size_t count,
                         int dtype, int op, void* hip_stream);

/* ReduceScatter(sum), local share: the strict one-rank view of the first half of
 * the paper's ring AllReduce (Evaluation, "End-to-End Performance": N-1
 * reduce-scatter steps, after which rank r owns the fully reduced slice r).
 *   rank_bufs   host array of nranks device pointers; rank_bufs[r] holds rank r's
 *               nranks * recv_count contiguous elements (slice s at offset
 *               s * recv_count).
 *   out         device pointer to recv_count elements.
 * Result: out[j] = sum over r, in rank order, of rank_bufs[r][rank*recv_count + j],
 * with exactly the arithmetic, split, engines and error behaviour of
 * flex_allreduce_local (it is that reduction applied to the local rank's slice;
 * HBM traffic (nranks+1) * recv_count elements).  nranks * recv_count * size
 * must not exceed max_bytes_per_rank.  Followed by flex_allgather_local over the
 * nranks reduced slices it gives the AllReduce a real rank performs. */
int flex_reducescatter_local(flex_comm_t* comm, const void* const* rank_bufs, void* out, size_t recv_count,
                             int dtype, int op, void* hip_stream);

/* AllGather, local share (paper: same section; N-1 ring steps that place every
 * rank's slice at its rank offset).
 *   rank_slices  host array of nranks device pointers to slice_count elements.
 *   out          device pointer to nranks * slice_count elements.
 * Result: out[r * slice_count + j] = rank_slices[r][j], bit for bit.  The
 * device path copies the head [0, split) of every slice on hip_stream; the tail
 * [split, slice_count) of every peer slice goes through the transit buffers
 * straight to its place in out (the local slice is copied whole by the device
 * path).  rank_slices[rank] may already be out + rank * slice_count (in-place
 * convention): it is then not copied.  Errors as for flex_allreduce_local. */
int flex_allgather_local(flex_comm_t* comm, const void* const* rank_slices, void* out,
                         size_t slice_count, int dtype, void* hip_stream);

/* AllReduce(sum), local share, for callers that cannot allocate: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  No
 * communicator is needed and the call allocates nothing, on the host or on the
 * device, and creates no stream or event.
 *   rank_bufs, out, count, dtype, op, hip_stream  as for flex_allreduce_local;
 *   nranks, rank   as for flex_comm_create;
 *   staged_units   share of the message, in units of 1/10000, whose peer parts
 *                  are staged through a transit buffer before they are reduced
 *                  (0 = none: one kernel launch).
 * The message is cut as flex_allreduce_local cuts it at its default settings;
 * the head is reduced straight from the rank buffers, the tail's peer parts are
 * first copied into a transit buffer and reduced from there in the same rank
 * order, with the local rank's part read in place.  The result has the bits of
 * flex_allreduce_local.  Everything is enqueued on hip_stream, so a call may be
 * captured into a graph (make the first call on each device outside a capture:
 * it looks the transit buffer's address up once per device).
 * The transit buffer is a 32 MiB array built into the library's device code;
 * each GPU the library runs on holds it until the process ends.  The staged
 * part, rounded up to 256 bytes, times (nranks - 1) must fit into it
 * (4 MiB per peer with 8 ranks); a larger one is refused with INVALID_ARG and
 * nothing is enqueued.  All calls on one GPU share the buffer: calls that may
 * run at the same time on different streams of one GPU race on it.  Nothing in
 * it needs clearing between calls (a call reads only what it has just written).
 * Errors: INVALID_ARG, UNSUPPORTED (dtype, op, device index above 63), HIP. */
int flex_allreduce_staged_noalloc(const void* const* rank_bufs, int nranks, int rank, void* out, size_t count,
                                  int dtype, int op, uint32_t staged_units, void* hip_stream);

/* AllToAll, local share: the primitive the paper names as its next one
 * (Limitations and Future Work).
 *   rank_bufs  host array of nranks device pointers; rank_bufs[r] holds rank r's
 *              nranks * count contiguous elements, piece d (count elements at
 *              offset d * count) being addressed to rank d.
 *   out        device pointer to nranks * count elements.
 * Result: out[r * count + j] = rank_bufs[r][rank * count + j], bit for bit: the
 * local rank's receive buffer.  It is flex_allgather_local applied to the pieces
 * addressed to the local rank (same split, engines and error behaviour; the
 * local rank's own piece is copied by the device path).  nranks * count * size
 * must not exceed max_bytes_per_rank. */
int flex_alltoall_local(flex_comm_t* comm, const void* const* rank_bufs, void* out, size_t count, int dtype,
                        void* hip_stream);

/* Choose how later calls of collective `coll` are split.
 *   FLEX_SPLIT_STATIC    every call uses host_units (0 = device path only).
 *   FLEX_SPLIT_ADAPTIVE  calls use the share vector of the balancer that
 *                        belongs to the message's size class (messages are
 *                        classed by floor(log2(bytes per rank))); the Evaluator
 *                        feeds per-path times of finished calls back into it
 *                        (Stage 2).  A size class that was never tuned borrows
 *                        the shares of the nearest tuned class of the same
 *                        collective; with none tuned, calls stay device-only.
 * Errors: INVALID_ARG (coll, mode, host_units > max_host_units). */
int flex_set_split(flex_comm_t* comm, int coll, int mode, uint32_t host_units);

/* The same for communicators with two host-staged paths.
 *   aux_units  host array of naux (0..FLEX_MAX_PATHS-1) shares, aux_units[a] for
 *              path 1 + a; paths beyond naux get 0.  Read only in static mode.
 * Errors: INVALID_ARG (as flex_set_split; a non-zero share for a path the
 * communicator does not have; shares summing above share_total). */
int flex_set_split_paths(flex_comm_t* comm, int coll, int mode, const uint32_t* aux_units, int naux);

/* Stage 1 on the real hardware (paper: Section "Stage 1: Initial
 * Coarse-Grained Tuning").  Blocking.  Runs collective `coll` on the given
 * buffers repeatedly: first to measure each path's rate (device path alone;
 * each host path at probe_units with the other idle), then Algorithm 1 with MeasurePathTimings = median
 * of tune_reps calls, until the balancer leaves Stage 1.  Then, unless
 * tune_accept_check is 0 or the host path was already drained, the balanced
 * split is timed against the device path alone, accept_pairs times in turns
 * (split, device-only, split, ...), and kept only if its median is lower by
 * more than three times the larger median absolute deviation; otherwise the
 * class reverts to device-only (the two paths share the GPU's memory system,
 * so a balanced split can be slower than no split).  The resulting
 * balancer is stored for the message's size class (replacing an older one).
 * Arguments as for the collective itself; `out` is overwritten with the
 * collective's (correct) result.  result may be NULL.
 * Errors: as the collective, plus STATE if timings cannot be read. */
int flex_comm_tune(flex_comm_t* comm, int coll, const void* const* rank_bufs, void* out, size_t count,
                   int dtype, void* hip_stream, flex_tune_result_t* result);

/* Install explicit shares for the size class of a message of `count` elements of
 * `dtype` (for example shares saved from an earlier flex_comm_tune): the class
 * gets a balancer in Stage 2 holding them, marked as tuned.
 *   shares  host array of one share per path of the communicator ({device,
 *           host}, or {device, host, host2} with num_aux_paths = 2) summing to
 *           share_total; a path given 0 units is inactive.
 * Errors: INVALID_ARG (null, unknown collective, sum != share_total, host share
 * above max_host_units), UNSUPPORTED (dtype). */
int flex_comm_set_shares(flex_comm_t* comm, int coll, size_t count, int dtype, const uint32_t* shares);

/* Evaluator: read back the timing records of finished calls without blocking
 * (also done at the start of every collective call). */
int flex_evaluator_poll(flex_comm_t* comm);

/* Evaluator: wait until every call issued so far has finished and read all
 * records back. */
int flex_evaluator_drain(flex_comm_t* comm);

/* Statistics for collective `coll` and for the size class of a message of
 * `count` elements of `dtype`.  out: host pointer. */
int flex_get_stats(flex_comm_t* comm, int coll, size_t count, int dtype, flex_stats_t* out);

/* The iterations of the last flex_comm_tune for the size class of a message of
 * `count` elements of `dtype`, oldest first: up to max_rounds entries are
 * written to rounds (host array), *nrounds receives how many the tuning ran
 * (it may exceed max_rounds; at most 128 are kept).
 * Errors: INVALID_ARG (null, unknown collective), UNSUPPORTED (dtype),
 * STATE (that class was never tuned). */
int flex_comm_tune_trace(flex_comm_t* comm, int coll, size_t count, int dtype, flex_tune_round_t* rounds,
                         uint32_t max_rounds, uint32_t* nrounds);

/* How a host part of `bytes` bytes per peer is cut into pipeline steps (paper:
 * Section "Communicator", the double-buffered PD2H / H2CD pipeline): step sizes
 * start at min_step_bytes, double up to chunk_bytes, stay there, and halve back
 * down to min_step_bytes at the end, so that the stretch at either end of the
 * transfer where only one of the two stages is busy is short.  Every step is a
 * multiple of 256 bytes except that the last one also takes what is left over;
 * no step exceeds chunk_bytes.  Pure host arithmetic.
 *   steps   host array receiving up to max_steps sizes (may be NULL to count);
 *   nsteps  receives the number of steps of the plan.
 * Errors: INVALID_ARG (null nsteps, chunk_bytes < 512 or not a multiple of 256,
 * min_step_bytes == 0). */
int flex_pipeline_plan(uint64_t bytes, uint64_t chunk_bytes, uint64_t min_step_bytes, uint64_t* steps,
                       uint32_t max_steps, uint32_t* nsteps);

/* sizeof() of the structs of this header as the library was compiled, for
 * bindings that mirror them: out[0..5] = flex_balancer_cfg_t,
 * flex_balancer_state_t, flex_config_t, flex_stats_t, flex_tune_result_t,
 * flex_tune_round_t.  out: host array of 6.  Errors: INVALID_ARG (null). */
int flex_struct_sizes(size_t* out);

/* Static strings; never NULL. */
const char* flex_status_string(int status);
const char* flex_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FLEXLINK_H */
