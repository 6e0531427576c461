#!/usr/bin/env python3
"""Configurations 0, 3 and 4 on one MI355X: message-size sweep with the
two-stage balancer, the tensor-parallel prefill shape, and the small
launch-bound message.  Prints one JSON line per case; --summary FILE also
writes the figures as a plain-text table.

    python sweep.py --config 3      # 1..1024 MiB per rank, AR and AG
    python sweep.py --config 3 --dtype f32   # same byte sizes in binary32 (or f16)
    python sweep.py --config 4      # 65536 x 5120 bf16 AllReduce, 50 calls
    python sweep.py --config 0      # 1 MiB fp32 AllReduce: latency
    python sweep.py --config 5      # the paper's evaluation grid: 2 / 4 / 8 ranks x 32..256 MiB, AR and AG

Per case: Stage 1 on the hardware (rates of both paths, bandwidth-proportional
initial shares, Algorithm 1, acceptance check), then adaptive calls (Stage 2),
then the same number of device-only calls interleaved block by block for an A/B
comparison.  For messages of 640 MiB per rank and more the host path is also
forced live (the shares Algorithm 1 balanced at, before the acceptance check)
and compared with the device path alone the same way: the only sizes where what
PCIe can carry during one call exceeds what a split call costs.
"""
import argparse
import json
import sys
import time

import torch

from paper_2510_15882_amd import binding as fx
from paper_2510_15882_amd import workloads as wl

def median(v):
    v = sorted(v)
    n = len(v)
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def mad(v):
    m = median(v)
    return median([abs(x - m) for x in v])


def pct(v, q):
    v = sorted(v)
    return v[min(len(v) - 1, max(0, int(round(q * (len(v) - 1)))))]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Case:
    def __init__(self, w, dev="cuda:0", cfg=None):
        self.w = w
        self.bufs = wl.make_rank_buffers(w, dev)
        es = self.bufs[0].element_size()
        self.is_ar = w.collective == "allreduce"
        self.coll = fx.FLEX_ALLREDUCE if self.is_ar else fx.FLEX_ALLGATHER
        n = w.nranks
        self.out = torch.empty(w.count if self.is_ar else n * w.count, dtype=w.dtype, device=dev)
        self.hbm_bytes = (n + 1) * w.count * es if self.is_ar else 2 * n * w.count * es
        self.alg_bytes = w.count * es if self.is_ar else n * w.count * es
        self.comm = fx.flex_comm_create(n, 0, w.count * es, cfg)
        self.stream = torch.cuda.Stream()
        torch.cuda.synchronize()

    def call(self):
        if self.is_ar:
            fx.flex_allreduce_local(self.comm, self.bufs, self.out, stream=self.stream)
        else:
            fx.flex_allgather_local(self.comm, self.bufs, self.out, stream=self.stream)

    def timed(self, n):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        with torch.cuda.stream(self.stream):
            for a, b in evs:
                a.record(self.stream)
                self.call()
                b.record(self.stream)
        self.stream.synchronize()
        return [a.elapsed_time(b) for a, b in evs]

    def close(self):
        torch.cuda.synchronize()
        fx.flex_comm_destroy(self.comm)


def live_ab(c, w, units, blocks=12, per_block=10):
    """Host path forced live at `units` against the device path alone, in
    alternating blocks of calls; Stage 2 keeps running in the live blocks."""
    fx.flex_comm_set_shares(c.comm, c.coll, w.count, w.dtype, [10000 - units, units])
    live_ms, device_ms = [], []
    for _ in range(blocks):
        fx.flex_set_split(c.comm, c.coll, fx.FLEX_SPLIT_ADAPTIVE)
        live_ms += c.timed(per_block)
        fx.flex_evaluator_drain(c.comm)
        fx.flex_set_split(c.comm, c.coll, fx.FLEX_SPLIT_STATIC, 0)
        device_ms += c.timed(per_block)
    st = fx.flex_get_stats(c.comm, c.coll, w.count, w.dtype)
    a, d = median(live_ms), median(device_ms)
    noise = 3 * max(mad(live_ms), mad(device_ms))
    # what PCIe could carry while the device path handles the rest, at 45 GB/s each way
    pcie_share = (d * 1e-3) * 45e9 / ((w.nranks - 1) * w.count * c.bufs[0].element_size())
    return {"host_share_units_start": units, "host_share_units_end": int(st.balancer.shares[1]),
            "live_ms": a, "device_only_ms": d, "mad_ms": [mad(live_ms), mad(device_ms)], "calls_each": len(live_ms),
            "gain_ms": d - a, "three_mad_ms": noise, "live_faster": bool(d - a > noise),
            "live_slower": bool(a - d > noise), "last_path_times_ms": [t * 1e3 for t in list(st.last_time_s)[:2]],
            "ideal_host_share_pct_at_45GBs": 100.0 * pcie_share,
            "ideal_gain_ms": d * pcie_share / (1.0 + pcie_share)}


def run_case(w, windows=20, cfg=None):
    c = Case(w, cfg=cfg)
    bc = fx.flex_config_default().balancer
    calls = windows * bc.window
    with torch.cuda.stream(c.stream):
        res = fx.flex_comm_tune(c.comm, c.coll, c.bufs, c.out, stream=c.stream)
    trajectory = []
    adaptive_ms, device_ms = [], []
    for _ in range(windows):
        fx.flex_set_split(c.comm, c.coll, fx.FLEX_SPLIT_ADAPTIVE)
        adaptive_ms += c.timed(bc.window)
        fx.flex_evaluator_drain(c.comm)
        st = fx.flex_get_stats(c.comm, c.coll, w.count, w.dtype)
        trajectory.append(int(st.balancer.shares[1]))
        fx.flex_set_split(c.comm, c.coll, fx.FLEX_SPLIT_STATIC, 0)
        device_ms += c.timed(bc.window)
    st = fx.flex_get_stats(c.comm, c.coll, w.count, w.dtype)
    a, d = median(adaptive_ms), median(device_ms)
    out = {
        "config": w.index, "case": w.name, "MiB_per_rank": w.bytes_per_rank / wl.MIB,
        "path_rate_GBs": [res.path_bw[0] / 1e9, res.path_bw[1] / 1e9],
        "initial_host_share_pct": res.initial_shares[1] / 100.0,
        "balanced_host_share_pct": res.balanced_shares[1] / 100.0, "stage1_iterations": res.iterations,
        "balanced_split_ms": res.combined_s * 1e3, "device_alone_ms": res.device_alone_s * 1e3,
        "acceptance_mad_ms": [res.combined_mad_s * 1e3, res.device_alone_mad_s * 1e3],
        "reverted_to_device_only": bool(res.reverted), "stage1_host_share_pct": res.shares[1] / 100.0,
        "host_active_after_stage1": bool(res.active_mask & 2),
        "stage2_windows": windows, "stage2_adjustments": int(st.balancer.adjustments),
        "converged_host_share_pct": trajectory[-1] / 100.0, "host_share_trajectory_units": trajectory,
        "adaptive_ms": a, "adaptive_hbm_GBs": c.hbm_bytes / a / 1e6, "adaptive_algbw_GBs": c.alg_bytes / a / 1e6,
        "device_only_ms": d, "device_only_hbm_GBs": c.hbm_bytes / d / 1e6,
        "gain_pct": 100.0 * (d / a - 1.0), "mad_ms": [mad(adaptive_ms), mad(device_ms)],
        "adaptive_ms_p10_p90": [pct(adaptive_ms, 0.1), pct(adaptive_ms, 0.9)],
        "device_only_ms_p10_p90": [pct(device_ms, 0.1), pct(device_ms, 0.9)],
        "combined_faster": bool(d - a > 3 * max(mad(adaptive_ms), mad(device_ms))),
        "calls_each": calls,
    }
    if w.bytes_per_rank >= 640 * wl.MIB:
        units = res.balanced_shares[1] or res.initial_shares[1] or 20
        out["host_path_forced_live"] = live_ab(c, w, units)
    c.close()
    return out


def run_grid_case(w, windows=5):
    """One point of the paper's evaluation grid: the sweep's protocol with fewer
    windows, plus the device path over rotating buffer sets (small messages
    would otherwise be served by the memory-side cache)."""
    out = run_case(w, windows=windows)
    out["nranks"] = w.nranks
    c = Case(w)
    per_set = c.hbm_bytes
    nsets = min(12, max(2, -(-(3 << 29) // per_set)))
    sets = [(c.bufs, c.out)] + [(wl.make_rank_buffers(w, "cuda:0"), torch.empty_like(c.out)) for _ in range(nsets - 1)]
    call = fx.flex_allreduce_local if c.is_ar else fx.flex_allgather_local
    fx.flex_set_split(c.comm, c.coll, fx.FLEX_SPLIT_STATIC, 0)
    reps = 5 * nsets
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    with torch.cuda.stream(c.stream):
        for k in range(nsets):
            call(c.comm, sets[k][0], sets[k][1], stream=c.stream)
        for k, (a, b) in enumerate(evs):
            bufs, dst = sets[k % nsets]
            a.record(c.stream)
            call(c.comm, bufs, dst, stream=c.stream)
            b.record(c.stream)
        # the same calls with one event pair around all of them: events around a call of
        # 15-50 us add 2-3 us to it
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(c.stream)
        for k in range(reps):
            call(c.comm, sets[k % nsets][0], sets[k % nsets][1], stream=c.stream)
        e1.record(c.stream)
    c.stream.synchronize()
    ms = [a.elapsed_time(b) for a, b in evs]
    batch = e0.elapsed_time(e1) / reps
    out["rotating_buffer_sets"] = nsets
    out["rotating_ms"] = median(ms)
    out["rotating_hbm_GBs"] = c.hbm_bytes / median(ms) / 1e6
    out["rotating_algbw_GBs"] = c.alg_bytes / median(ms) / 1e6
    out["rotating_batch_ms_per_call"] = batch
    out["rotating_batch_hbm_GBs"] = c.hbm_bytes / batch / 1e6
    out["rotating_batch_algbw_GBs"] = c.alg_bytes / batch / 1e6
    out["rotating_batch_calls"] = reps
    c.close()
    del sets
    return out


def run_prefill(calls=50):
    w = wl.config(4)
    c = Case(w)
    with torch.cuda.stream(c.stream):
        res = fx.flex_comm_tune(c.comm, c.coll, c.bufs, c.out, stream=c.stream)
    out = {"config": 4, "case": w.name, "MiB_per_rank": w.bytes_per_rank / wl.MIB,
           "path_rate_GBs": [res.path_bw[0] / 1e9, res.path_bw[1] / 1e9],
           "initial_host_share_pct": res.initial_shares[1] / 100.0,
           "balanced_host_share_pct": res.balanced_shares[1] / 100.0, "balanced_split_ms": res.combined_s * 1e3,
           "device_alone_ms": res.device_alone_s * 1e3, "reverted_to_device_only": bool(res.reverted),
           "stage1_host_share_pct": res.shares[1] / 100.0, "stage1_iterations": res.iterations}
    for mode, name in ((fx.FLEX_SPLIT_ADAPTIVE, "adaptive"), (fx.FLEX_SPLIT_STATIC, "device_only")):
        fx.flex_set_split(c.comm, c.coll, mode, 0)
        c.timed(5)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(c.stream):
            for _ in range(calls):            # back to back on one stream, no host sync
                c.call()
        c.stream.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / calls
        out[name + "_ms_per_call"] = ms
        out[name + "_hbm_GBs"] = c.hbm_bytes / ms / 1e6
        out[name + "_algbw_GBs"] = c.alg_bytes / ms / 1e6
    fx.flex_evaluator_drain(c.comm)
    st = fx.flex_get_stats(c.comm, c.coll, w.count, w.dtype)
    out["host_share_pct_after"] = st.balancer.shares[1] / 100.0
    out["blocking_reads"] = int(st.blocking_reads)
    units = res.balanced_shares[1] or res.initial_shares[1] or 20
    out["host_path_forced_live"] = live_ab(c, w, units)
    c.close()
    return out


def run_small():
    w = wl.config(0)
    c = Case(w)
    c.timed(20)
    single = c.timed(200)
    # back-to-back launches amortise the launch gap
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(c.stream):
        e0.record(c.stream)
        for _ in range(1000):
            c.call()
        e1.record(c.stream)
    c.stream.synchronize()
    per = e0.elapsed_time(e1) / 1000
    # the same 1000 calls as 10 replays of a captured graph of 100
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=c.stream):
        for _ in range(100):
            c.call()
    torch.cuda.synchronize()
    graph.replay()
    with torch.cuda.stream(c.stream):
        e0.record(c.stream)
        for _ in range(10):
            graph.replay()
        e1.record(c.stream)
    c.stream.synchronize()
    per_graph = e0.elapsed_time(e1) / 1000
    want = [t.clone() for t in [c.out]]
    c.out.zero_()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(c.out, want[0]), "graph replay changed the result"
    del graph
    # cold: rotate over distinct buffer sets larger than the caches
    sets = [(wl.make_rank_buffers(w, "cuda:0"), torch.empty_like(c.out)) for _ in range(64)]
    torch.cuda.synchronize()
    with torch.cuda.stream(c.stream):
        e0.record(c.stream)
        for k in range(640):
            bufs, out = sets[k % 64]
            fx.flex_allreduce_local(c.comm, bufs, out, stream=c.stream)
        e1.record(c.stream)
    c.stream.synchronize()
    cold = e0.elapsed_time(e1) / 640
    out = {"config": 0, "case": w.name, "event_bracketed_single_call_us": median(single) * 1e3,
           "back_to_back_us_per_call": per * 1e3, "back_to_back_hbm_GBs": c.hbm_bytes / per / 1e6,
           "graph_replay_us_per_call": per_graph * 1e3, "graph_replay_hbm_GBs": c.hbm_bytes / per_graph / 1e6,
           "rotating_64_buffer_sets_us_per_call": cold * 1e3, "rotating_hbm_GBs": c.hbm_bytes / cold / 1e6,
           "note": "9 MiB of traffic per call: launch-bound; the warm figure is served by L2 and the memory-side cache"}
    c.close()
    return out


def summary_lines(r):
    """One case as a few lines of plain text."""
    if r["config"] == 0:
        return ["cfg0 %s: event-bracketed single call %.2f us; back to back %.2f us per call (%.0f GB/s); graph "
                "replay %.2f us per call (%.0f GB/s); rotating over 64 cold buffer sets %.2f us per call (%.0f GB/s)"
                % (r["case"], r["event_bracketed_single_call_us"], r["back_to_back_us_per_call"],
                   r["back_to_back_hbm_GBs"], r["graph_replay_us_per_call"], r["graph_replay_hbm_GBs"],
                   r["rotating_64_buffer_sets_us_per_call"], r["rotating_hbm_GBs"])]
    lines = ["%s %s (%g MiB per rank)" % ("grid" if r["config"] == 5 else "cfg%d" % r["config"], r["case"],
                                          r["MiB_per_rank"]),
             "  path rates (message GB/s) device %.1f, host %.2f; InitializeShares host %.2f %%; Algorithm 1: %s "
             "iterations, balanced host share %.2f %%"
             % (r["path_rate_GBs"][0], r["path_rate_GBs"][1], r["initial_host_share_pct"],
                r.get("stage1_iterations", "?"), r["balanced_host_share_pct"]),
             "  acceptance check: balanced split %.4f ms vs device alone %.4f ms -> %s; host share after Stage 1 %.2f %%"
             % (r["balanced_split_ms"], r["device_alone_ms"],
                "reverted to device-only" if r["reverted_to_device_only"] else "kept", r["stage1_host_share_pct"])]
    if "adaptive_ms" in r:
        lines.append("  %d Stage-2 windows: converged host share %.2f %%, %d adjustments; adaptive %.4f ms (MAD %.4f) vs "
                     "device-only %.4f ms (MAD %.4f), %d calls each, interleaved -> combined faster: %s"
                     % (r["stage2_windows"], r["converged_host_share_pct"], r["stage2_adjustments"], r["adaptive_ms"],
                        r["mad_ms"][0], r["device_only_ms"], r["mad_ms"][1], r["calls_each"], r["combined_faster"]))
        lines.append("  adaptive: HBM %.0f GB/s, algbw %.1f GB/s; device-only: HBM %.0f GB/s"
                     % (r["adaptive_hbm_GBs"], r["adaptive_algbw_GBs"], r["device_only_hbm_GBs"]))
    else:
        lines.append("  50 calls back to back on one stream: adaptive %.4f ms per call (HBM %.0f GB/s, algbw %.1f GB/s), "
                     "device-only %.4f ms per call (HBM %.0f GB/s); host share afterwards %.2f %%; blocking reads %d"
                     % (r["adaptive_ms_per_call"], r["adaptive_hbm_GBs"], r["adaptive_algbw_GBs"],
                        r["device_only_ms_per_call"], r["device_only_hbm_GBs"], r["host_share_pct_after"],
                        r["blocking_reads"]))
    if "rotating_ms" in r:
        lines.append("  device path over %d rotating buffer sets: events around each call %.4f ms, HBM %.0f GB/s, algbw "
                     "%.1f GB/s; %d calls between one pair of events %.4f ms per call, HBM %.0f GB/s, algbw %.1f GB/s"
                     % (r["rotating_buffer_sets"], r["rotating_ms"], r["rotating_hbm_GBs"], r["rotating_algbw_GBs"],
                        r["rotating_batch_calls"], r["rotating_batch_ms_per_call"], r["rotating_batch_hbm_GBs"],
                        r["rotating_batch_algbw_GBs"]))
    live = r.get("host_path_forced_live")
    if live:
        lines.append("  host path forced live at %d units (ends at %d): %.4f ms (MAD %.4f) vs device-only %.4f ms (MAD %.4f), "
                     "%d calls each in alternating blocks; gain %.4f ms against 3 x MAD %.4f ms -> %s; PCIe at 45 GB/s "
                     "could carry %.2f %% in that time (ideal gain %.4f ms)"
                     % (live["host_share_units_start"], live["host_share_units_end"], live["live_ms"], live["mad_ms"][0],
                        live["device_only_ms"], live["mad_ms"][1], live["calls_each"], live["gain_ms"],
                        live["three_mad_ms"], "faster" if live["live_faster"] else
                        ("slower" if live["live_slower"] else "no difference beyond the noise"),
                        live["ideal_host_share_pct_at_45GBs"], live["ideal_gain_ms"]))
    return lines


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True, choices=[0, 3, 4, 5],
                    help="0, 3, 4: the configurations; 5: the paper's evaluation grid (2 / 4 / 8 ranks x 32..256 MiB)")
    ap.add_argument("--summary", default=None, help="append the cases as plain text to this file")
    ap.add_argument("--windows", type=int, default=20)
    ap.add_argument("--max-mib", type=int, default=1024)
    ap.add_argument("--dtype", default="bf16", choices=sorted(wl.DTYPE_NAMES),
                    help="element type of the configuration 3 sweep (same byte sizes)")
    args = ap.parse_args()
    assert torch.cuda.is_available(), "needs the GPU"
    fx.lib()
    torch.cuda.set_device(0)
    def emit(r):
        print(json.dumps(r), flush=True)
        if args.summary:
            with open(args.summary, "a") as f:
                f.write("\n".join(summary_lines(r)) + "\n")

    if args.config == 0:
        emit(run_small())
    elif args.config == 4:
        emit(run_prefill())
    elif args.config == 5:
        for w in wl.evaluation_grid_workloads():
            log("case", w.name)
            emit(run_grid_case(w, windows=min(args.windows, 5)))
            torch.cuda.empty_cache()
    else:
        for w in wl.sweep_workloads(args.dtype):
            if w.bytes_per_rank > args.max_mib * wl.MIB:
                continue
            log("case", w.name)
            emit(run_case(w, windows=args.windows))
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
