"""CPU-side tests of the library: it loads and exports every declared symbol,
and its host logic (balancer, partition) follows the oracle step for step.
No GPU call is made here."""
import os
import random
import re

import pytest
from hypothesis import given, settings, strategies as st

from oracle import balancer as ob
from oracle import partition as op
from paper_2510_15882_amd import binding as fx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "flexlink.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flex_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 20
    L = fx.lib()
    for n in names:
        assert hasattr(L, n), n


def test_struct_layout_defaults_come_through():
    c = fx.flex_config_default()
    import ctypes
    assert c.struct_size == ctypes.sizeof(fx.Config)
    assert c.chunk_bytes == 4 << 20 and c.num_slots == 2 and c.max_host_units == 2500
    assert c.split_align_elems == 2048 and c.min_split_bytes == 64 << 10
    assert c.tune_reps == 5 and c.probe_units == 200 and c.reduce_nontemporal == 3 and c.copy_nontemporal == 3
    assert (c.host_engine, c.host_blocks, c.host_down_blocks, c.min_step_bytes) == (fx.FLEX_ENGINE_KERNEL, 8, 6, 256 << 10)
    assert c.sample_every == 1 and c.reduce_lds_reserve == 5632
    assert c.tune_accept_check == 1 and c.accept_pairs == 3 and c.launch_shape == fx.FLEX_SHAPE_WAVE
    assert c.slot_sync == 0 and c.num_aux_paths == 1 and c.host_die_shift == 2 and c.reduce_serial_loads == 1
    b = c.balancer
    assert (b.share_total, b.initial_step, b.stability_required, b.max_tune_iters, b.window,
            b.runtime_step, b.aux_share_cap) == (10000, 16, 3, 100, 10, 4, 0)
    assert b.convergence_threshold == 0.05 and b.runtime_threshold == 0.10
    assert fx.flex_status_string(0) == "ok" and fx.flex_status_string(1) == "invalid argument"


def cfg(**kw):
    c = fx.flex_balancer_cfg_default()
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def run_library_tune(S0, measure, c):
    """Drive the library's state machine with the oracle's measure() callback."""
    b = fx.flex_balancer_init_shares(S0, c)
    traj = []
    try:
        while True:
            s = fx.flex_balancer_get(b)
            if s.stage != fx.FLEX_STAGE_TUNING:
                break
            active = {p for p in range(len(S0)) if s.active_mask >> p & 1}
            T = measure(list(s.shares)[:len(S0)], active)
            shares = fx.flex_balancer_update(b, T)
            s2 = fx.flex_balancer_get(b)
            traj.append(dict(S=shares, step=s2.step, stability_count=s2.stability_count,
                             active=sorted(p for p in range(len(S0)) if s2.active_mask >> p & 1)))
        return traj, fx.flex_balancer_get(b)
    finally:
        fx.flex_balancer_destroy(b)


def test_library_follows_hand_trace():
    measure = lambda S, A: [S[0] / 9.0, S[1] / 1.0]
    traj, final = run_library_tune([80, 20], measure, cfg(share_total=100, initial_step=8, stability_required=2))
    assert [t["S"] for t in traj] == [[88, 12], [96, 4], [92, 8], [88, 12], [90, 10], [90, 10], [90, 10]]
    assert [t["step"] for t in traj] == [8, 8, 4, 4, 2, 2, 2]
    assert final.stage == fx.FLEX_STAGE_RUNTIME and final.tune_iters == 7


@given(seed=st.integers(0, 10 ** 6), npaths=st.integers(2, 4), step0=st.sampled_from([1, 16, 64, 500]),
       thr=st.sampled_from([0.01, 0.05, 0.3]), stab=st.integers(1, 4), cap=st.sampled_from([0, 0, 2500, 4000]))
@settings(max_examples=400, deadline=None)
def test_library_stage1_equals_oracle_step_for_step(seed, npaths, step0, thr, stab, cap):
    # cap: ceiling on every auxiliary path's share (0 = the paper's method unchanged)
    rnd = random.Random(seed)
    total = 10000
    cuts = sorted(rnd.randint(0, total) for _ in range(npaths - 1))
    S0 = [b - a for a, b in zip([0] + cuts, cuts + [total])]
    lat = [rnd.uniform(0, 3) for _ in range(npaths)]
    rate = [rnd.uniform(0.5, 50) for _ in range(npaths)]
    noise = [rnd.uniform(0.95, 1.05) for _ in range(400)]

    def make_measure():
        k = [0]

        def measure(S, A):
            k[0] += 1
            return [(lat[p] + S[p] / rate[p]) * noise[(k[0] * 7 + p) % 400] + 1e-6 if p in A else 0.0
                    for p in range(npaths)]
        return measure

    trace = []
    S_or, A_or = ob.initial_tune(S0, make_measure(), step0=step0, threshold=thr, stability_required=stab,
                                 trace=trace, cap=[None] + [cap] * (npaths - 1) if cap else None)
    traj, final = run_library_tune(S0, make_measure(),
                                   cfg(initial_step=step0, convergence_threshold=thr, stability_required=stab,
                                       aux_share_cap=cap))
    assert len(traj) == len(trace)
    for a, b in zip(traj, trace):
        assert a["S"] == b["S"] and a["step"] == b["step"] and a["active"] == b["active"]
        assert a["stability_count"] == b["stability_count"]
    assert list(final.shares)[:npaths] == S_or
    assert {p for p in range(npaths) if final.active_mask >> p & 1} == A_or


@given(bw=st.lists(st.floats(0.0, 1e13), min_size=1, max_size=4), total=st.sampled_from([100, 10000, 65536]))
@settings(max_examples=300, deadline=None)
def test_library_initialize_shares_equals_oracle(bw, total):
    if not bw[0] > 0:
        bw[0] = 1.0
    want = ob.initialize_shares(bw, total)
    b = fx.flex_balancer_init(bw, cfg(share_total=total))
    try:
        s = fx.flex_balancer_get(b)
        assert list(s.shares)[:len(bw)] == want
        assert s.active_mask == sum(1 << p for p in range(len(bw)) if want[p] > 0)
    finally:
        fx.flex_balancer_destroy(b)


@given(seed=st.integers(0, 10 ** 6), npaths=st.integers(2, 4), window=st.sampled_from([1, 2, 5, 10]),
       step=st.sampled_from([1, 4, 50]), cap=st.sampled_from([0, 0, 120, 400]))
@settings(max_examples=300, deadline=None)
def test_library_stage2_equals_oracle(seed, npaths, window, step, cap):
    rnd = random.Random(seed)
    total = 10000
    cuts = sorted(rnd.randint(0, 300) for _ in range(npaths - 1))
    S0 = [cuts[0]] + [b - a for a, b in zip(cuts, cuts[1:])] if npaths > 1 else []
    S0 = [total - sum(S0)] + S0
    c = cfg(window=window, runtime_step=step, runtime_threshold=0.10, aux_share_cap=cap)
    b = fx.flex_balancer_init_shares(S0, c)
    fx.flex_balancer_finish_tuning(b)
    r = ob.RuntimeAdjuster(S0, {p for p in range(npaths) if S0[p] > 0}, window=window, threshold=0.10, step=step,
                           cap=[None] + [cap] * (npaths - 1) if cap else None)
    try:
        for _ in range(120):
            T = [rnd.choice([1.0, 1.05, 1.2, 3.0, 0.5]) * rnd.uniform(0.9, 1.1) for _ in range(npaths)]
            got = fx.flex_balancer_update(b, T)
            r.observe(T)
            assert got == r.S
        s = fx.flex_balancer_get(b)
        assert s.adjustments == r.adjustments
        assert {p for p in range(npaths) if s.active_mask >> p & 1} == r.C_active
    finally:
        fx.flex_balancer_destroy(b)


def test_library_balancer_rejects_bad_input():
    with pytest.raises(fx.FlexError) as e:
        fx.flex_balancer_init([0.0, 1.0])
    assert e.value.status == fx.FLEX_ERR_INVALID_ARG
    with pytest.raises(fx.FlexError):
        fx.flex_balancer_init([1.0] * 5)
    with pytest.raises(fx.FlexError):
        fx.flex_balancer_init_shares([50, 40], cfg(share_total=100))
    b = fx.flex_balancer_init_shares([90, 10], cfg(share_total=100))
    before = fx.flex_balancer_get(b).as_dict()
    for bad in ([1.0, 0.0], [1.0, -1.0], [float("nan"), 1.0], [float("inf"), 1.0]):
        with pytest.raises(fx.FlexError):
            fx.flex_balancer_update(b, bad)
    assert fx.flex_balancer_get(b).as_dict() == before       # state unchanged by rejected updates
    assert "time" in fx.flex_last_error()
    fx.flex_balancer_destroy(b)


def test_library_only_primary_skips_tuning():
    b = fx.flex_balancer_init([5.0, 0.0])
    s = fx.flex_balancer_get(b)
    assert s.stage == fx.FLEX_STAGE_RUNTIME and list(s.shares)[:2] == [10000, 0] and s.active_mask == 1
    # host time is ignored once the path is inactive
    assert fx.flex_balancer_update(b, [1.0, 0.0]) == [10000, 0]
    fx.flex_balancer_destroy(b)


@given(count=st.integers(0, 1 << 36), units=st.integers(0, 10000), align=st.sampled_from([1, 64, 2048, 4096]),
       min_count=st.sampled_from([0, 1, 32768, 1 << 20]))
@settings(max_examples=500, deadline=None)
def test_library_partition_equals_oracle(count, units, align, min_count):
    assert fx.flex_partition(count, units, 10000, align, min_count) == op.partition(count, units, 10000, align, min_count)


def test_library_partition_rejects_bad_input():
    with pytest.raises(fx.FlexError):
        fx.flex_partition(100, 10001)
    with pytest.raises(fx.FlexError):
        fx.flex_partition(100, 1, align_elems=0)


def test_library_revert_to_primary():
    b = fx.flex_balancer_init_shares([9000, 600, 400], cfg())
    fx.flex_balancer_revert_to_primary(b)
    s = fx.flex_balancer_get(b)
    assert list(s.shares)[:3] == [10000, 0, 0] and s.active_mask == 1 and s.stage == fx.FLEX_STAGE_RUNTIME
    for _ in range(25):      # drained paths never come back
        assert fx.flex_balancer_update(b, [5.0, 0.0, 0.0]) == [10000, 0, 0]
    fx.flex_balancer_destroy(b)


@given(count=st.integers(0, 1 << 36), units=st.lists(st.integers(0, 3333), min_size=1, max_size=3),
       align=st.sampled_from([1, 64, 2048]), min_count=st.sampled_from([0, 32768, 1 << 20]))
@settings(max_examples=500, deadline=None)
def test_library_partition_paths_equals_oracle(count, units, align, min_count):
    u = [0] + units
    assert fx.flex_partition_paths(count, u, 10000, align, min_count) == op.partition_paths(count, u, 10000, align, min_count)
    if len(u) == 2:
        assert fx.flex_partition_paths(count, u, 10000, align, min_count)[1] == fx.flex_partition(count, u[1], 10000, align, min_count)


def test_library_partition_paths_rejects_bad_input():
    with pytest.raises(fx.FlexError):
        fx.flex_partition_paths(100, [0, 6000, 6000])
    with pytest.raises(fx.FlexError):
        fx.flex_partition_paths(100, [0, 1, 1, 1, 1])


def test_binding_structs_have_the_library_layout():
    import ctypes
    want = [ctypes.sizeof(t) for t in (fx.BalancerCfg, fx.BalancerState, fx.Config, fx.Stats, fx.TuneResult,
                                       fx.TuneRound)]
    assert fx.flex_struct_sizes() == want


def test_header_is_plain_c_and_its_structs_have_the_library_layout(tmp_path):
    # the boundary is a C ABI: the header must compile as strict C99 and as C++
    # with no other header, and a C compiler must lay the structs out as the
    # library does
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text(
        '#include "flexlink.h"\n#include <stdio.h>\n'
        'int main(void) { printf("%zu %zu %zu %zu %zu %zu\\n", sizeof(flex_balancer_cfg_t), '
        'sizeof(flex_balancer_state_t), sizeof(flex_config_t), sizeof(flex_stats_t), sizeof(flex_tune_result_t), '
        'sizeof(flex_tune_round_t)); '
        'return (FLEX_MAX_RANKS == 8 && FLEX_MAX_PATHS == 4 && FLEX_ALLTOALL == 3) ? 0 : 1; }\n')
    exe = tmp_path / "sizes"
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, str(src), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(x) for x in out] == fx.flex_struct_sizes()
    cpp = tmp_path / "only_header.cpp"
    cpp.write_text('#include "flexlink.h"\nint main() { return sizeof(flex_config_t) ? 0 : 1; }\n')
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(cpp)], check=True)


@given(nbytes=st.integers(0, 1 << 33), chunk=st.sampled_from([4096, 64 << 10, 1 << 20, 4 << 20]),
       min_step=st.sampled_from([1, 256, 4096, 256 << 10, 8 << 20]), es=st.sampled_from([1, 2, 4]))
@settings(max_examples=400, deadline=None)
def test_pipeline_plan_properties(nbytes, chunk, min_step, es):
    nbytes -= nbytes % es
    steps = fx.flex_pipeline_plan(nbytes, chunk, min_step)
    assert sum(steps) == nbytes and all(0 < n <= chunk for n in steps)
    assert all(n % 256 == 0 for n in steps[:-1])          # only the last step is ragged ...
    assert all(n % es == 0 for n in steps)                # ... and every step holds whole elements
    if nbytes >= 256:
        floor = min(max((min_step + 255) // 256 * 256, 256), chunk)
        # first and last steps are short (one min_step, give or take the left-overs), the middle ones long
        if nbytes >= 4 * floor and floor < chunk:
            assert steps[0] == floor and steps[-1] < 2 * floor + 256
        assert len(steps) <= nbytes // chunk + 2 * 16 + 2
    # the ramps mirror each other: as many doubling steps at the front as halving steps at the back
    up = 0
    while up + 1 < len(steps) and steps[up + 1] == 2 * steps[up] and steps[up + 1] < chunk:
        up += 1
    if up:
        back = steps[::-1]
        back[0] -= back[0] % 256 if back[0] >= 256 else 0       # the last step also carries the left-over bytes
        assert back[:up] == steps[:up]


def test_pipeline_plan_hand_values_and_errors():
    K = 1 << 10
    assert fx.flex_pipeline_plan(0) == []
    assert fx.flex_pipeline_plan(100) == [100]
    assert fx.flex_pipeline_plan(1 << 20) == [256 * K, 512 * K, 256 * K]
    assert fx.flex_pipeline_plan(10 << 20) == [x * K for x in (256, 512, 1024, 2048, 2560, 2048, 1024, 512, 256)]
    assert fx.flex_pipeline_plan((1 << 20) + 6) == [256 * K, 512 * K, 256 * K + 6]
    assert fx.flex_pipeline_plan(9 << 20, 4 << 20, 4 << 20) == [3 << 20] * 3     # no ramp: even steps
    with pytest.raises(fx.FlexError):
        fx.flex_pipeline_plan(1 << 20, 1000, 256)
    with pytest.raises(fx.FlexError):
        fx.flex_pipeline_plan(1 << 20, 4096, 0)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2510_15882_amd import build
    monkeypatch.setattr(fx, "_lib", None)
    monkeypatch.setattr(build, "LIB", str(tmp_path / "libflexlink.so"))
    with pytest.raises(RuntimeError, match="not built"):
        fx.flex_config_default()


def test_binding_refuses_counts_beyond_a_tensor():
    # the C ABI takes plain pointers: the binding is where a count that runs past a
    # tensor's end can still be caught before a kernel reads or writes outside it
    import torch
    n = 4
    bufs = [torch.zeros(4 * 100) for _ in range(n)]
    small, big = torch.zeros(100), torch.zeros(4 * 100)
    fx._marshal(fx.FLEX_ALLREDUCE, bufs, big, 400, require_device=False)
    fx._marshal(fx.FLEX_REDUCESCATTER, bufs, small, 100, require_device=False)
    fx._marshal(fx.FLEX_ALLGATHER, [small] * n, big, 100, require_device=False)
    arr = fx._marshal(fx.FLEX_ALLTOALL, bufs, big, 100, require_device=False)
    assert [arr[r] for r in range(n)] == [b.data_ptr() for b in bufs]
    for coll, tensors, out, count in ((fx.FLEX_ALLREDUCE, bufs, big, 401), (fx.FLEX_ALLREDUCE, bufs, small, 400),
                                      (fx.FLEX_REDUCESCATTER, bufs, small, 101), (fx.FLEX_ALLGATHER, [small] * n, big, 101),
                                      (fx.FLEX_ALLGATHER, bufs, small, 100), (fx.FLEX_ALLTOALL, bufs, big, 101),
                                      (fx.FLEX_ALLTOALL, bufs, small, 100), (fx.FLEX_ALLREDUCE, bufs[:3] + [small], big, 400)):
        with pytest.raises(ValueError):
            fx._marshal(coll, tensors, out, count, require_device=False)
    with pytest.raises(ValueError):
        fx._marshal(fx.FLEX_ALLREDUCE, bufs, big, 400)                     # host tensors
    with pytest.raises(ValueError):
        fx._marshal(fx.FLEX_ALLREDUCE, bufs, big.double(), 400, require_device=False)
