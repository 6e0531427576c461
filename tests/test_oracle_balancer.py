"""Pins for the balancer oracle (Algorithm 1 and the Stage-2 prose) and for the
partition oracle: hand-executed trajectories, the closed-form balance point of a
pure-bandwidth timing model, and the properties the paper states in prose."""
import os

import pytest
from hypothesis import given, settings, strategies as st

from oracle import balancer as ob
from oracle import partition as op

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_trace(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def bandwidth_model(rate, latency=None):
    latency = latency or [0.0] * len(rate)

    def measure(S, C_active):
        return [latency[p] + S[p] / rate[p] if p in C_active else 0.0 for p in range(len(S))]
    return measure


# ---------------------------------------------------------------- Stage 1

def test_alg1_two_path_hand_trace():
    trace = []
    S, active = ob.initial_tune([80, 20], bandwidth_model([9.0, 1.0]), primary=0, step0=8,
                                threshold=0.05, stability_required=2, trace=trace)
    rows = read_trace("alg1_two_path_trace.txt")
    assert len(trace) == len(rows)
    for t, row in zip(trace, rows):
        i, slow, step, stab, s0, s1 = map(int, row)
        assert (t["i"], t["slow"], t["step"], t["stability_count"], t["S"]) == (i, slow, step, stab, [s0, s1])
    assert S == [90, 10] and active == {0, 1}


def test_alg1_three_path_hand_trace():
    trace = []
    S, active = ob.initial_tune([70, 20, 10], bandwidth_model([10.0, 2.0, 0.1]), primary=0, step0=16,
                                threshold=0.1, stability_required=1, trace=trace)
    rows = read_trace("alg1_three_path_trace.txt")
    assert len(trace) == len(rows)
    for t, row in zip(trace, rows):
        i, slow, step, stab, s0, s1, s2 = map(int, row[:7])
        act = [int(x) for x in row[7].split(",")]
        assert (t["i"], t["slow"], t["step"], t["stability_count"], t["S"], t["active"]) == \
            (i, slow, step, stab, [s0, s1, s2], act)
    assert S == [84, 16, 0] and active == {0, 1}


def test_alg1_bottlenecked_primary_sheds_to_fastest_path():
    # primary slowest, two auxiliaries: the move goes to the faster of the two
    trace = []
    ob.initial_tune([90, 5, 5], bandwidth_model([1.0, 1.0, 2.0]), step0=4, max_iters=1, trace=trace)
    assert trace[0]["slow"] == 0 and trace[0]["fast"] == 2 and trace[0]["S"] == [86, 5, 9]


def test_alg1_slow_auxiliary_gives_to_primary_even_if_other_aux_is_faster():
    # path 1 slowest, path 2 fastest, but the primary is the target (primary-first rule)
    trace = []
    ob.initial_tune([50, 40, 10], bandwidth_model([1.0, 0.1, 10.0]), step0=4, max_iters=1, trace=trace)
    assert trace[0]["slow"] == 1 and trace[0]["fast"] == 2 and trace[0]["S"] == [54, 36, 10]


def test_alg1_only_primary_measures_nothing():
    calls = []

    def measure(S, A):
        calls.append(1)
        return [1.0, 1.0]
    S, active = ob.initial_tune([100, 0], measure)
    assert S == [100, 0] and active == {0} and not calls


def test_alg1_hopeless_auxiliary_path_is_deactivated():
    # host path has a latency 1000x the device's whole-message time: every
    # measurement finds it slowest, so its share drains to zero and the loop
    # ends with only the primary active.
    total = 10000
    S0 = ob.initialize_shares([1.0, 0.01], total)
    measure = bandwidth_model([total / 1.0, total / 100.0], latency=[0.0, 1000.0])
    trace = []
    S, active = ob.initial_tune(S0, measure, step0=64, trace=trace)
    assert S == [total, 0] and active == {0}
    assert all(t["slow"] == 1 for t in trace)
    assert len(trace) == -(-S0[1] // 64)        # one full step per iteration, no halving


def test_alg1_stops_after_100_measurements():
    # a model that flips the bottleneck every time never converges
    flip = [0]

    def measure(S, A):
        flip[0] ^= 1
        return [2.0, 1.0] if flip[0] else [1.0, 2.0]
    trace = []
    ob.initial_tune([5000, 5000], measure, step0=64, trace=trace)
    assert len(trace) == 100
    assert trace[-1]["step"] == 1


@given(rate0=st.floats(1.0, 1000.0), ratio=st.floats(0.001, 0.5), step0=st.sampled_from([16, 64, 256]),
       start=st.integers(1, 5000))
@settings(max_examples=200, deadline=None)
def test_alg1_pure_bandwidth_model_reaches_closed_form_balance(rate0, ratio, step0, start):
    # T_p = S_p / rate_p  =>  both paths finish together at
    # S_1* = total * rate_1 / (rate_0 + rate_1).
    total = 10000
    rate = [rate0, rate0 * ratio]
    trace = []
    S, active = ob.initial_tune([total - start, start], bandwidth_model(rate), step0=step0,
                                threshold=0.05, stability_required=3, trace=trace)
    star = total * rate[1] / (rate[0] + rate[1])
    assert sum(S) == total and min(S) >= 0
    last = trace[-1]
    if active == {0}:
        # share drained: only possible when the balance point is within a step of zero
        assert star <= step0
    elif len(trace) < 100:
        assert last["imbalance"] < 0.05 and last["stability_count"] == 3
        # imbalance < 5 % bounds the distance to the balance point
        assert abs(S[1] - star) <= 0.06 * star + 1
    elif last["step"] == step0:
        # 100 measurements spent without ever crossing the balance point:
        # every one of them moved a full step towards it
        moves = sum(1 for t in trace if t["imbalance"] >= 0.05)
        assert moves >= 97 and abs(S[1] - start) == moves * step0
        assert abs(S[1] - star) < abs(start - star)
    else:
        assert abs(S[1] - star) <= 2 * last["step"] + 0.06 * star + 1


@given(seed=st.integers(0, 10 ** 6), npaths=st.integers(2, 4))
@settings(max_examples=200, deadline=None)
def test_alg1_invariants_under_arbitrary_timings(seed, npaths):
    import random
    rnd = random.Random(seed)
    total = 10000
    cuts = sorted(rnd.randint(0, total) for _ in range(npaths - 1))
    S0 = [b - a for a, b in zip([0] + cuts, cuts + [total])]
    lat = [rnd.uniform(0, 5) for _ in range(npaths)]
    rate = [rnd.uniform(0.1, 100) for _ in range(npaths)]
    noise = lambda: rnd.uniform(0.9, 1.1)

    def measure(S, A):
        return [(lat[p] + S[p] / rate[p]) * noise() + 1e-9 if p in A else 0.0 for p in range(npaths)]
    trace = []
    S, active = ob.initial_tune(S0, measure, step0=64, trace=trace)
    assert sum(S) == total and min(S) >= 0 and len(trace) <= 100
    prev_step, prev_active, prev_S = 64, {p for p in range(npaths) if S0[p] > 0}, S0
    for t in trace:
        assert 1 <= t["step"] <= prev_step                     # step never grows
        assert set(t["active"]) <= prev_active                 # a path never comes back
        assert sum(t["S"]) == total
        moved = sum(abs(a - b) for a, b in zip(t["S"], prev_S))
        assert moved <= 2 * t["step"]                          # at most one move of <= step
        for p in range(npaths):
            if p not in prev_active:
                assert t["S"][p] == prev_S[p] == 0 or p == 0   # inactive paths keep share 0
        prev_step, prev_active, prev_S = t["step"], set(t["active"]), t["S"]
    assert all(S[p] == 0 for p in range(1, npaths) if p not in active)


def test_share_ceiling_trims_a_transfer_and_an_empty_transfer_counts_as_calm():
    # hand-executed: three paths, primary slowest every round, path 2 fastest, ceiling 8 on both
    # auxiliaries, step 4, two calm rounds end the tuning.
    # r1: 0 -> 2 wants 4, room 8-5 = 3: S = [87, 5, 8]          calm 0
    # r2: 0 -> 2 wants 4, room 0: nothing moves                  calm 1
    # r3: the same                                               calm 2 -> stop
    trace = []
    S, live = ob.initial_tune([90, 5, 5], lambda S, A: [3.0, 2.0, 1.0], step0=4, stability_required=2,
                              cap=[None, 8, 8], trace=trace)
    assert [t["S"] for t in trace] == [[87, 5, 8], [87, 5, 8], [87, 5, 8]]
    assert [t["stability_count"] for t in trace] == [0, 1, 2] and S == [87, 5, 8] and live == {0, 1, 2}
    # without the ceiling the same timings keep draining the primary path
    S, live = ob.initial_tune([90, 5, 5], lambda S, A: [3.0, 2.0, 1.0], step0=4, stability_required=2, max_iters=5)
    assert S == [70, 5, 25]
    # the primary path has no ceiling: a slow auxiliary still hands everything back
    S, live = ob.initial_tune([90, 5, 5], lambda S, A: [1.0, 9.0, 2.0], step0=4, cap=[None, 8, 8], max_iters=2)
    assert S == [95, 0, 5] and live == {0, 2}
    # Stage 2: a trimmed move is a move, an empty one is not
    r = ob.RuntimeAdjuster([9900, 98, 2], {0, 1, 2}, window=1, threshold=0.10, step=4, cap=[None, 100, 100])
    assert r.observe([3.0, 1.0, 2.0]) and r.S == [9898, 100, 2] and r.adjustments == 1
    assert not r.observe([3.0, 1.0, 2.0]) and r.S == [9898, 100, 2] and r.adjustments == 1


# ----------------------------------------------------- InitializeShares

def test_initialize_shares_is_bandwidth_proportional():
    assert ob.initialize_shares([99.0, 1.0], 10000) == [9900, 100]
    assert ob.initialize_shares([6000.0, 55.0], 10000) == [10000 - 90, 90]      # floor(90.83)
    assert ob.initialize_shares([3.0, 1.0, 1.0], 100) == [60, 20, 20]
    assert ob.initialize_shares([5.0, 0.0], 10000) == [10000, 0]
    assert ob.initialize_shares([5.0, -1.0, 5.0], 10) == [5, 0, 5]


# ---------------------------------------------------------------- Stage 2

def test_stage2_no_move_inside_threshold():
    r = ob.RuntimeAdjuster([9900, 100], {0, 1}, window=10, threshold=0.10, step=4)
    for _ in range(50):
        assert not r.observe([1.00, 1.09])
    assert r.S == [9900, 100] and r.adjustments == 0


def test_stage2_moves_one_fixed_step_per_window_towards_primary():
    r = ob.RuntimeAdjuster([9900, 100], {0, 1}, window=10, threshold=0.10, step=4)
    moved = [r.observe([1.0, 2.0]) for _ in range(30)]
    assert moved == ([False] * 9 + [True]) * 3
    assert r.S == [9912, 88]


def test_stage2_bottlenecked_primary_sheds_to_fastest():
    r = ob.RuntimeAdjuster([9900, 60, 40], {0, 1, 2}, window=4, threshold=0.10, step=4)
    for _ in range(4):
        r.observe([3.0, 2.0, 1.0])
    assert r.S == [9896, 60, 44]


def test_stage2_single_spike_in_window_is_ignored():
    r = ob.RuntimeAdjuster([9900, 100], {0, 1}, window=10, threshold=0.10, step=4)
    for k in range(10):
        r.observe([1.0, 50.0 if k == 3 else 1.0])
    assert r.S == [9900, 100]


def test_stage2_drains_and_deactivates_and_never_reactivates():
    r = ob.RuntimeAdjuster([9994, 6], {0, 1}, window=2, threshold=0.10, step=4)
    for _ in range(2):
        r.observe([1.0, 9.0])
    assert r.S == [9998, 2] and r.C_active == {0, 1}
    for _ in range(2):
        r.observe([1.0, 9.0])
    assert r.S == [10000, 0] and r.C_active == {0}
    for _ in range(20):
        assert not r.observe([9.0, 0.0])
    assert r.S == [10000, 0]


def test_stage2_window_median_even_length():
    assert ob.median([4.0, 1.0, 3.0, 2.0]) == 2.5
    assert ob.median([5.0, 1.0, 3.0]) == 3.0


# -------------------------------------------------------------- partition

def test_partition_edges():
    assert op.partition(1 << 20, 0) == 1 << 20
    assert op.partition(1 << 20, 10000) == 0
    assert op.partition(1000, 5000) == 1000                  # below min_count: not split
    assert op.partition(1 << 20, 5000) == 1 << 19
    # 1 unit of 2^20 elements owes 104 elements -> rounds to one quantum
    assert op.partition(1 << 20, 1) == (1 << 20) - 2048
    # ragged tail goes to the host part: 1_000_003 * 0.05 = 50000 owed;
    # 950003 rounded down to 2048 -> 948224
    assert op.partition(1000003, 500) == 948224


@given(count=st.integers(0, 1 << 34), units=st.integers(0, 10000))
@settings(max_examples=500, deadline=None)
def test_partition_properties(count, units):
    s = op.partition(count, units)
    assert 0 <= s <= count
    if units == 0 or count < 32768:
        assert s == count
        return
    assert s % 2048 == 0
    host = count - s
    owed = count * units // 10000
    assert host >= owed and host > 0
    assert host - owed <= 2048 + 2048          # rounding adds less than two quanta


def test_partition_paths_reduces_to_the_two_path_cut():
    for count in (0, 5, 40000, 1 << 20, 1000003, (1 << 27) + 17):
        for u in (0, 1, 37, 500, 2200, 9999, 10000):
            assert op.partition_paths(count, [0, u]) == [0, op.partition(count, u), count]


def test_partition_paths_hand_values():
    # 2^20 elements, 5 % and 12 %: owed 52428 and 125829.  The last path's piece
    # starts at floor((1048576 - 125829) / 2048) * 2048 = 921600; the middle one
    # at floor((921600 - 52428) / 2048) * 2048 = 868352.
    assert op.partition_paths(1 << 20, [0, 500, 1200]) == [0, 868352, 921600, 1 << 20]
    # a path with share 0 gets nothing; everything to the last path
    assert op.partition_paths(1 << 20, [0, 0, 10000]) == [0, 0, 0, 1 << 20]
    assert op.partition_paths(1 << 20, [0, 10000, 0]) == [0, 0, 1 << 20, 1 << 20]
    # tiny shares still get one quantum each
    assert op.partition_paths(1 << 20, [0, 1, 1]) == [0, (1 << 20) - 4096, (1 << 20) - 2048, 1 << 20]
    assert op.partition_paths(1000, [0, 5000, 5000]) == [0, 1000, 1000, 1000]      # too short to split


@given(count=st.integers(0, 1 << 34), u1=st.integers(0, 5000), u2=st.integers(0, 5000), u3=st.integers(0, 0))
@settings(max_examples=500, deadline=None)
def test_partition_paths_properties(count, u1, u2, u3):
    start = op.partition_paths(count, [0, u1, u2])
    assert start[0] == 0 and start[3] == count and start == sorted(start)
    if count < 32768:
        assert start[1] == start[2] == count
        return
    for p, u in ((1, u1), (2, u2)):
        piece = start[p + 1] - start[p]
        owed = count * u // 10000
        if u == 0:
            assert piece == 0
        else:
            assert piece > 0 or start[p + 1] == 0
            assert start[p] % 2048 == 0
            if start[p] > 0:
                assert owed <= piece < owed + 2 * 2048
