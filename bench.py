#!/usr/bin/env python3
"""Benchmark of the local-share hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
an AllReduce of the 8 x 256 MiB bf16 message (configuration 2) followed by an
AllGather of 8 x 32 MiB bf16 slices into 256 MiB (configuration 1), both through
the C ABI with the two-path split chosen by the tuned, adaptive balancer
(partition -> device path + host-staged path -> join -> evaluate/rebalance).
Inputs are resident in HBM before the timed region starts.

Successive steps rotate over --buffer-sets independent sets of input and output
buffers (default 3, about 8 GiB in all), so that every byte a step touches was
last touched several GiB of traffic earlier: the 256 MB memory-side cache cannot
keep an output buffer resident from one call to the next and the HBM traffic
equals the algorithmic bytes.  The same-buffers-every-call figures (what
nccl-tests style loops measure) are reported under extras.warm_same_buffers*.

Prints ONE JSON line.  `value` is algorithmic HBM bytes per second over the
timed steps (AllReduce (N+1)*S, AllGather 2*N*slice); `roofline` prices the
dominant kernel (the N-way reduce) against the 8 TB/s HBM3E peak from per-launch
HIP-event timings taken inside the timed region (two events around the
AllReduce call of every 4th step, sample count and p10 / p90 reported: each
event is a packet of its own on the stream and costs about 2 us of stream time,
so bracketing every call of every step would cost 2 % of `value`; the AllGather
call is timed in an untimed leg right after, call by call and in batches of ten
that share one pair of events); `host_path` gives configuration 2's static 5 / 12 /
22 % splits with the PCIe rate per direction against 64 GB/s; `extras.ceilings`
is what plain probe kernels reach on this very box (bench_ceilings.hip);
`cpu_baseline` is the CPU oracle timed on this machine's host cores.
"""
import argparse
import ctypes
import hashlib
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PCIE_PEAK_GBS = 64.0
METRIC = "AllReduce/AllGather local-share GB/s at 256MB (8 sim ranks); % HBM peak"
N = 8

CEILINGS_SRC = os.path.join(ROOT, "bench_ceilings.hip")
CEILINGS_LIB = os.path.join(ROOT, "libflex_ceilings.so")
CEILINGS_EXE = os.path.join(ROOT, "bench_ceilings")
PMC_SUMMARY = os.path.join("profiles", "reduce_n_allreduce_bf16_256MiB_pmc.txt")
KERNEL_SOURCES = [os.path.join("paper_2510_15882_amd", "csrc", f)
                  for f in ("reduce_n.hip", "gather_copy.hip", "flexlink_internal.h")]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def median(v):
    v = sorted(v)
    n = len(v)
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def percentile(v, q):
    v = sorted(v)
    return v[min(len(v) - 1, max(0, int(round(q * (len(v) - 1)))))]


def build_ceilings():
    """Compile bench_ceilings.hip for gfx950: a shared library this script loads
    and a stand-alone program for rocprofv3."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    common = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
              "-packed-fp32-ops", "-Wall", "-Wextra", CEILINGS_SRC]
    for extra, target in ((["-shared", "-fPIC"], CEILINGS_LIB), (["-DCEILINGS_MAIN"], CEILINGS_EXE)):
        tmp = target + ".tmp.%d" % os.getpid()
        subprocess.check_call(common + extra + ["-o", tmp])
        os.replace(tmp, target)


def measure_ceilings(what=3, reps=6):
    """HBM and PCIe ceilings of this machine from the probe kernels, or a note why not."""
    if not os.path.exists(CEILINGS_LIB):
        return {"note": "libflex_ceilings.so is not built (python -c 'import bench; bench.build_ceilings()')"}
    lib = ctypes.CDLL(CEILINGS_LIB)
    lib.flex_ceilings_run.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int]
    buf = ctypes.create_string_buffer(1 << 16)
    rc = lib.flex_ceilings_run(buf, len(buf), what, reps)
    text = buf.value.decode()
    return json.loads(text) if rc == 0 else {"error": text}


def kernel_sources_hash():
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_from_profiles():
    """HBM bytes per launch of the reduce kernel from the committed rocprofv3
    counter summary (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel
    calibration).  The summary names the kernel sources it was measured on; if
    they have changed since, the figure is stale and None is returned."""
    note = {"source": PMC_SUMMARY, "kernel_sources": kernel_sources_hash()}
    try:
        fields = {}
        for line in open(os.path.join(ROOT, PMC_SUMMARY)):
            if ":" in line and not line.startswith(" "):
                k, v = line.split(":", 1)
                fields[k.strip()] = v.strip()
        measured_on = fields.get("kernel_sources_sha256", "")
        note["measured_on_kernel_sources"] = measured_on
        if measured_on == note["kernel_sources"]:
            return float(fields["traffic_bytes_per_launch"]), note
        note["stale"] = True
    except (OSError, KeyError, ValueError):
        note["missing"] = True
    return None, note


def cpu_baseline(oc, ar_host, ag_host, ar_bytes, ag_bytes, budget_s=10.0):
    threads = oc.get_threads()
    oc.allreduce(ar_host)          # warm pass (page faults, thread pool)
    oc.allgather(ag_host)
    times = []
    t_start = time.perf_counter()
    while not times or (time.perf_counter() - t_start < budget_s and len(times) < 200):
        t0 = time.perf_counter()
        oc.allreduce(ar_host)
        oc.allgather(ag_host)
        times.append(time.perf_counter() - t0)
    med = median(times)
    # the same step on one thread, best of 3 (a few seconds)
    oc.set_threads(1)
    single = []
    for _ in range(3):
        t0 = time.perf_counter()
        oc.allreduce(ar_host)
        oc.allgather(ag_host)
        single.append(time.perf_counter() - t0)
    oc.set_threads(threads)
    # the single collectives, all cores, best of 5 (algorithmic bytes / time): configuration 2's AllReduce,
    # configuration 1's AllGather, configuration 0's shape (1 MiB of f32 per rank, in cache) and a 64 MiB-per-rank
    # slice standing in for the larger messages of configurations 3 and 4
    def best(fn, n=5):
        out = []
        for _ in range(n):
            t0 = time.perf_counter()
            fn()
            out.append(time.perf_counter() - t0)
        return min(out)
    import numpy as np
    small = [np.linspace(-1.0, 1.0, 262144, dtype=np.float32) * (r + 1) / 8 for r in range(N)]
    slice64 = [a[:32 << 20] for a in ar_host]
    per_collective = {
        "cfg2_allreduce_bf16_256MiB_GBs": ar_bytes / best(lambda: oc.allreduce(ar_host)) / 1e9,
        "cfg1_allgather_bf16_32MiB_GBs": ag_bytes / best(lambda: oc.allgather(ag_host)) / 1e9,
        "cfg0_allreduce_f32_1MiB_GBs": 9 * (1 << 20) / best(lambda: oc.allreduce(small), 20) / 1e9,
        "allreduce_bf16_64MiB_per_rank_GBs": 9 * (64 << 20) / best(lambda: oc.allreduce(slice64)) / 1e9,
        "allgather_bf16_64MiB_per_rank_GBs": 16 * (64 << 20) / best(lambda: oc.allgather(slice64)) / 1e9,
    }
    return {"value": (ar_bytes + ag_bytes) / med / 1e9, "unit": "GB/s", "cores": threads,
            "per_collective": per_collective,
            "single_thread": {"value": (ar_bytes + ag_bytes) / min(single) / 1e9, "unit": "GB/s",
                              "seconds_per_step": min(single), "passes": 3, "statistic": "best"},
            "kind": "oracle", "seconds_per_step": med, "best_seconds_per_step": min(times), "passes": len(times),
            "sample": "the full step (configuration 2 AllReduce + configuration 1 AllGather), same bytes as "
                      "buffer set 0 of the GPU run; median of %d passes (about %.0f s of wall time, %d OpenMP "
                      "threads) after one warm pass" % (len(times), time.perf_counter() - t_start, threads)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--mode", default="adaptive",
                    help="adaptive (tuned balancer) | device (host share 0) | static:UNITS (of 10000)")
    ap.add_argument("--buffer-sets", type=int, default=3, help="independent buffer sets the steps rotate over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="only launch a plain copy of known size (1-rank AllGather of 1 GiB, 10 launches): the "
                         "reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--no-extras", action="store_true", help="skip the untimed warm / static-split / ceilings legs")
    ap.add_argument("--event-every", type=int, default=0,
                    help="bracket the AllReduce call of every K-th timed step with HIP events (per-launch times for the "
                         "roofline); 0 = every 4th step")
    ap.add_argument("--launch-shape", type=int, default=-1, help="0: 64-thread workgroups, 1: 256-thread workgroups")
    ap.add_argument("--reduce-nt", type=int, default=-1)
    ap.add_argument("--copy-nt", type=int, default=-1)
    ap.add_argument("--reduce-serial", type=int, default=-1,
                    help="2: one load in flight per wavefront; 0: all of a tile; 1: by message size")
    ap.add_argument("--host-engine", type=int, default=-1, help="0 copy kernels, 1 hybrid (copy kernel up, DMA down), 2 DMA engines")
    ap.add_argument("--host-blocks", type=int, default=0)
    ap.add_argument("--reduce-lds", type=int, default=-1, help="LDS bytes reserved per reduce workgroup (occupancy cap)")
    ap.add_argument("--max-host-units", type=int, default=0,
                    help="largest host share the communicator accepts (default 2500; 10000 to time the host path alone "
                         "with --mode static:10000)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is the single-GPU local share; it runs on exactly one GPU "
                 "(--gpus 1). No figure at several GPUs exists.")

    import torch
    from paper_2510_15882_amd import binding as fx
    from paper_2510_15882_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    fx.lib()
    torch.cuda.set_device(0)
    dev = "cuda:0"
    if args.pmc_calibration:
        n = 1 << 29                                   # 512 Mi bf16 = 1 GiB
        src = torch.empty(n, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty(n, dtype=torch.bfloat16, device=dev)
        comm = fx.flex_comm_create(1, 0, 2 * n)
        for _ in range(10):
            fx.flex_allgather_local(comm, [src], dst)
        torch.cuda.synchronize()
        assert torch.equal(src.view(torch.int16), dst.view(torch.int16))
        fx.flex_comm_destroy(comm)
        print(json.dumps({"calibration": "gather_copy_kernel, 1 rank, 10 launches",
                          "read_bytes_per_launch": 2 * n, "write_bytes_per_launch": 2 * n,
                          "kernel_sources_sha256": kernel_sources_hash()}))
        return

    w_ar, w_ag = wl.config(2), wl.config(1)
    nsets = max(1, args.buffer_sets)
    log("generating %d buffer set(s) on the GPU ..." % nsets)
    sets = []
    for k in range(nsets):
        ar_bufs = wl.make_rank_buffers(w_ar, dev)        # every set holds the same seeded values
        ag_slices = wl.make_rank_buffers(w_ag, dev)
        sets.append((ar_bufs, torch.empty(w_ar.count, dtype=w_ar.dtype, device=dev),
                     ag_slices, torch.empty(N * w_ag.count, dtype=w_ag.dtype, device=dev)))
    ar_bytes = (N + 1) * w_ar.bytes_per_rank
    ag_bytes = 2 * N * w_ag.bytes_per_rank

    cfg = fx.flex_config_default()
    if args.host_blocks:
        cfg.host_blocks = args.host_blocks
    if args.max_host_units:
        cfg.max_host_units = args.max_host_units
    for key, val in (("reduce_nontemporal", args.reduce_nt), ("copy_nontemporal", args.copy_nt),
                     ("host_engine", args.host_engine), ("reduce_serial_loads", args.reduce_serial),
                     ("launch_shape", args.launch_shape), ("reduce_lds_reserve", args.reduce_lds)):
        if val >= 0:
            setattr(cfg, key, val)
    effective = {key: getattr(cfg, key) for key in (
        "launch_shape", "reduce_serial_loads", "reduce_nontemporal", "reduce_lds_reserve", "copy_nontemporal",
        "host_engine", "host_blocks", "host_down_blocks",
        "host_die_shift", "chunk_bytes", "min_step_bytes", "num_slots")}
    comm = fx.flex_comm_create(N, 0, w_ar.bytes_per_rank, cfg)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()

    def ar(k=0):
        s = sets[k % nsets]
        fx.flex_allreduce_local(comm, s[0], s[1], stream=stream)

    def ag(k=0):
        s = sets[k % nsets]
        fx.flex_allgather_local(comm, s[2], s[3], stream=stream)

    def timed_calls(fn, n, rotate):
        """Per-call milliseconds of n calls, HIP events on the launch stream."""
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        with torch.cuda.stream(stream):
            for k, (a, b) in enumerate(evs):
                a.record(stream)
                fn(k if rotate else 0)
                b.record(stream)
        stream.synchronize()
        return [a.elapsed_time(b) for a, b in evs]

    def stats(coll, w):
        return fx.flex_get_stats(comm, coll, w.count, w.dtype)

    tune = {}
    with torch.cuda.stream(stream):
        # ---- untimed: Stage 1 of the balancer, or a fixed split ----------
        if args.mode == "adaptive":
            for coll, bufs, out, name in ((fx.FLEX_ALLREDUCE, sets[0][0], sets[0][1], "allreduce"),
                                          (fx.FLEX_ALLGATHER, sets[0][2], sets[0][3], "allgather")):
                res = fx.flex_comm_tune(comm, coll, bufs, out, stream=stream)
                tune[name] = {"path_rate_GBs_of_message": [res.path_bw[0] / 1e9, res.path_bw[1] / 1e9],
                              "initial_shares": list(res.initial_shares)[:2],
                              "balanced_shares": list(res.balanced_shares)[:2],
                              "balanced_split_ms": res.combined_s * 1e3, "device_alone_ms": res.device_alone_s * 1e3,
                              "balanced_split_mad_ms": res.combined_mad_s * 1e3,
                              "device_alone_mad_ms": res.device_alone_mad_s * 1e3,
                              "acceptance_samples_each": res.accept_samples,
                              "reverted_to_device_only": bool(res.reverted),
                              "shares": list(res.shares)[:2], "iterations": res.iterations}
                log("tuned", name, tune[name])
                fx.flex_set_split(comm, coll, fx.FLEX_SPLIT_ADAPTIVE)
        elif args.mode == "device":
            pass
        elif args.mode.startswith("static:"):
            units = int(args.mode.split(":")[1])
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
            fx.flex_set_split(comm, fx.FLEX_ALLGATHER, fx.FLEX_SPLIT_STATIC, units)
        else:
            sys.exit("unknown --mode")

        for k in range(args.warmup):
            ar(k)
            ag(k)
    stream.synchronize()
    fx.flex_evaluator_drain(comm)
    s_ar0 = stats(fx.FLEX_ALLREDUCE, w_ar)

    # ---- timed region: exactly --steps steps --------------------------------
    every = args.event_every if args.event_every > 0 else 4
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(0, args.steps, every)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        for k in range(args.steps):
            if k % every == 0:
                e = ev[k // every]
                e[0].record(stream)
                ar(k)
                e[1].record(stream)
            else:
                ar(k)
            ag(k)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    fx.flex_evaluator_drain(comm)
    s_ar1 = stats(fx.FLEX_ALLREDUCE, w_ar)
    s_ag1 = stats(fx.FLEX_ALLGATHER, w_ag)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = (ar_bytes + ag_bytes) / (ms_per_step * 1e-3) / 1e9
    ar_ms = [e[0].elapsed_time(e[1]) for e in ev]
    # untimed: the AllGather call by call, in the same AR -> AG sequence over the same rotating buffers
    ev_ag = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(40)]
    with torch.cuda.stream(stream):
        for k, e in enumerate(ev_ag):
            ar(k)
            e[0].record(stream)
            ag(k)
            e[1].record(stream)
    torch.cuda.synchronize()
    fx.flex_evaluator_drain(comm)
    ag_ms = [e[0].elapsed_time(e[1]) for e in ev_ag]
    # ... and in batches of ten calls between one pair of events (the events' own stream time amortised)
    ev_batch = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(6)]
    with torch.cuda.stream(stream):
        for b, e in enumerate(ev_batch):
            e[0].record(stream)
            for k in range(10):
                ag(10 * b + k)
            e[1].record(stream)
    torch.cuda.synchronize()
    ag_batch_ms = median([e[0].elapsed_time(e[1]) / 10 for e in ev_batch])

    # Dominant kernel: the N-way reduce of the device part.  When the call was
    # split, its launch is bracketed by the Evaluator's own events (fork ->
    # device path done) on the same stream; otherwise by the events above.
    split_samples = s_ar1.samples - s_ar0.samples
    dev_elems = s_ar1.last_split if s_ar1.last_count == w_ar.count else w_ar.count
    if split_samples > 0:
        total_dev_s = s_ar1.mean_time_s[0] * s_ar1.samples - s_ar0.mean_time_s[0] * s_ar0.samples
        kern_ms = total_dev_s / split_samples * 1e3
        spread = {}
        how = "Evaluator events fork->device-path-done, mean of %d split calls" % split_samples
        nlaunch = int(split_samples)
    else:
        kern_ms = sum(ar_ms) / len(ar_ms)
        spread = {"launch_ms_p10": percentile(ar_ms, 0.1), "launch_ms_p90": percentile(ar_ms, 0.9)}
        how = ("HIP events on the launch stream around every %slaunch of the timed region, mean of %d launches"
               % ("" if every == 1 else "%d-th " % every, len(ar_ms)))
        nlaunch = len(ar_ms)
    bytes_per_elem = (N + 1) * 2
    achieved = bytes_per_elem * dev_elems / (kern_ms * 1e-3) / 1e9 if dev_elems > 0 and kern_ms > 0 else 0.0
    host_timed = None
    if split_samples > 0:
        # the host path of the timed AllReduce calls: fork -> host path done, 7 peers' parts each way
        host_s = (s_ar1.mean_time_s[1] * s_ar1.samples - s_ar0.mean_time_s[1] * s_ar0.samples) / split_samples
        host_elems = s_ar1.last_count - s_ar1.last_split
        pcie = (N - 1) * host_elems * 2 / host_s / 1e9 if host_s > 0 else 0.0
        host_timed = {"allreduce_host_share_pct": 100.0 * host_elems / s_ar1.last_count, "host_path_ms": host_s * 1e3,
                      "pcie_GBs_per_direction": pcie, "pcie_frac_of_64GBs": pcie / PCIE_PEAK_GBS,
                      "split_calls": int(split_samples)}
    traffic, traffic_note = traffic_from_profiles()
    roofline = {"bound": "hbm", "kernel": "reduce_n_kernel<8, bf16>", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "traffic_from_profiles": traffic_note,
                "launch_ms": kern_ms, "launches_timed": nlaunch, "elements_per_launch": int(dev_elems),
                "bytes_per_element": bytes_per_elem,
                "algorithmic_bytes_per_launch": int(bytes_per_elem * dev_elems), "timing": how}
    roofline.update(spread)

    def host_units(st):
        return int(st.balancer.shares[1]) if args.mode == "adaptive" else int(st.static_host_units)

    result = {
        "metric": METRIC, "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[2] AllReduce bf16 8 ranks x 256 MiB (fp32 accumulate) + configs[1] "
                               "AllGather bf16 8 x 32 MiB -> 256 MiB, one call each per step",
                   "mode": args.mode, "nranks": N, "buffer_sets": nsets,
                   "algorithmic_bytes_per_step": ar_bytes + ag_bytes, "library": effective},
        "pct_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        "roofline": roofline,
        "allreduce": {"ms_median": median(ar_ms), "ms_p10": percentile(ar_ms, 0.1), "ms_p90": percentile(ar_ms, 0.9),
                      "calls_timed": len(ar_ms),
                      "hbm_GBs": ar_bytes / (median(ar_ms) * 1e-3) / 1e9,
                      "algbw_GBs": w_ar.bytes_per_rank / (median(ar_ms) * 1e-3) / 1e9,
                      "host_units": host_units(s_ar1), "split_calls_timed": int(split_samples)},
        "allgather": {"ms_median": median(ag_ms), "ms_p10": percentile(ag_ms, 0.1), "ms_p90": percentile(ag_ms, 0.9),
                      "calls_timed": len(ag_ms), "timing": "untimed leg after the timed region, same call sequence",
                      "ms_per_call_in_batches_of_10": ag_batch_ms,
                      "hbm_GBs_in_batches_of_10": ag_bytes / (ag_batch_ms * 1e-3) / 1e9,
                      "hbm_GBs": ag_bytes / (median(ag_ms) * 1e-3) / 1e9,
                      "algbw_GBs": N * w_ag.bytes_per_rank / (median(ag_ms) * 1e-3) / 1e9,
                      "host_units": host_units(s_ag1)},
    }
    if tune:
        result["tune"] = tune
    if host_timed:
        result["host_path_timed"] = host_timed

    # ---- untimed extras ------------------------------------------------------
    if not args.no_extras:
        extras = {}
        for coll in (fx.FLEX_ALLREDUCE, fx.FLEX_ALLGATHER):
            fx.flex_set_split(comm, coll, fx.FLEX_SPLIT_STATIC, 0)
        for name, rotate in (("device_only_rotating_buffers", True), ("warm_same_buffers", False)):
            d_ar = median(timed_calls(ar, 60, rotate))
            d_ag = median(timed_calls(ag, 60, rotate))
            extras[name] = {"allreduce_ms": d_ar, "allreduce_hbm_GBs": ar_bytes / d_ar / 1e6,
                            "allgather_ms": d_ag, "allgather_hbm_GBs": ag_bytes / d_ag / 1e6}
        extras["warm_same_buffers"]["note"] = ("same buffers every call, library defaults (non-temporal stores "
                                               "do not linger in the memory-side cache, so this is close to cold)")
        # plain (write-back) stores let a reused 256 MiB output stay resident in the 256 MB memory-side cache:
        # HBM then sees fewer bytes than the algorithm moves
        cfg2 = fx.flex_config_default()
        cfg2.reduce_nontemporal = 1
        comm2 = fx.flex_comm_create(N, 0, w_ar.bytes_per_rank, cfg2)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(60)]
        with torch.cuda.stream(stream):
            for a, b in evs:
                a.record(stream)
                fx.flex_allreduce_local(comm2, sets[0][0], sets[0][1], stream=stream)
                b.record(stream)
        stream.synchronize()
        fx.flex_comm_destroy(comm2)
        d = median([a.elapsed_time(b) for a, b in evs])
        extras["warm_same_buffers_plain_stores"] = {
            "allreduce_ms": d, "allreduce_hbm_GBs": ar_bytes / d / 1e6,
            "note": "reduce_nontemporal = 1: the reused output stays in the memory-side cache, its stores never reach HBM"}
        # the reduce kernel's occupancy cap on this machine: the library as configured against the same
        # library without the LDS reservation, alternating blocks of 10 launches over the rotating buffers
        cfg3 = fx.flex_config_default()
        cfg3.reduce_lds_reserve = 0
        comm3 = fx.flex_comm_create(N, 0, w_ar.bytes_per_rank, cfg3)
        ab = {"as_configured": [], "without_reservation": []}
        for block in range(4):
            ab["as_configured"] += timed_calls(ar, 10, True)
            ab["without_reservation"] += timed_calls(
                lambda k: fx.flex_allreduce_local(comm3, sets[k % nsets][0], sets[k % nsets][1], stream=stream), 10, True)
        fx.flex_comm_destroy(comm3)
        extras["reduce_occupancy_cap"] = {
            "reduce_lds_reserve": int(cfg.reduce_lds_reserve),
            "allreduce_ms": {k: median(v) for k, v in ab.items()},
            "allreduce_hbm_GBs": {k: ar_bytes / median(v) / 1e6 for k, v in ab.items()},
            "launches_each": len(ab["as_configured"])}
        # configuration 2's static split sweep: device-only vs 5 / 12 / 22 % through pinned host memory
        sweep = {}
        for units in (0, 100, 500, 1200, 2200):
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
            timed_calls(ar, 2, True)
            fx.flex_evaluator_drain(comm)
            b = stats(fx.FLEX_ALLREDUCE, w_ar)
            ms = median(timed_calls(ar, 10, True))
            fx.flex_evaluator_drain(comm)
            a = stats(fx.FLEX_ALLREDUCE, w_ar)
            row = {"allreduce_ms": ms, "hbm_GBs": ar_bytes / ms / 1e6, "algbw_GBs": w_ar.bytes_per_rank / ms / 1e6}
            n = a.samples - b.samples
            if n > 0:
                t_dev = (a.mean_time_s[0] * a.samples - b.mean_time_s[0] * b.samples) / n
                t_host = (a.mean_time_s[1] * a.samples - b.mean_time_s[1] * b.samples) / n
                host_elems = a.last_count - a.last_split
                pcie = (N - 1) * host_elems * 2 / t_host / 1e9
                row.update({"host_share_pct": 100.0 * host_elems / a.last_count, "device_path_ms": t_dev * 1e3,
                            "host_path_ms": t_host * 1e3, "pcie_GBs_per_direction": pcie,
                            "pcie_frac_of_64GBs": pcie / PCIE_PEAK_GBS})
            sweep[str(units)] = row
        fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, 0)
        extras["allreduce_static_split"] = sweep
        result["host_path"] = {
            "workload": "configs[2]: 8 x 256 MiB bf16 AllReduce, static host share, 7 peers' parts each way",
            "peak_GBs_per_direction": PCIE_PEAK_GBS, "engine": int(cfg.host_engine),
            "pcie_GBs_per_direction": {"%g%%" % (u / 100.0): sweep[str(u)].get("pcie_GBs_per_direction")
                                       for u in (500, 1200, 2200)},
            "allreduce_ms": {"%g%%" % (u / 100.0): sweep[str(u)]["allreduce_ms"] for u in (0, 500, 1200, 2200)}}
        torch.cuda.synchronize()
        log("measuring this box's ceilings ...")
        extras["ceilings"] = measure_ceilings()
        result["extras"] = extras

    if not args.no_cpu_baseline:
        from oracle import collectives as oc
        log("timing the CPU oracle ...")
        ar_host = [wl.to_numpy_bits(b) for b in sets[0][0]]
        ag_host = [wl.to_numpy_bits(b) for b in sets[0][2]]
        result["cpu_baseline"] = cpu_baseline(oc, ar_host, ag_host, ar_bytes, ag_bytes)

    torch.cuda.synchronize()
    fx.flex_comm_destroy(comm)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
