"""Parity of the HIP path against the CPU oracle, through the C ABI, on a real
MI355X.  Integer/byte work (AllGather) and, because the summation order is
fixed, the floating-point AllReduce too must match bit for bit: tolerance 0 ULP
wherever the oracle's result is not a NaN; a NaN must come out as a NaN."""
import sys

import numpy as np
import pytest
import torch

from oracle import balancer as ob
from oracle import collectives as oc
from oracle import partition as op
from paper_2510_15882_amd import binding as fx
from paper_2510_15882_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    fx.lib()
    torch.cuda.set_device(0)
    yield
    torch.cuda.synchronize()


class Comm:
    def __init__(self, nranks=8, rank=0, max_bytes=64 << 20, **cfg_fields):
        cfg = fx.flex_config_default()
        for k, v in cfg_fields.items():
            setattr(cfg, k, v)
        self.h = fx.flex_comm_create(nranks, rank, max_bytes, cfg)

    def __enter__(self):
        return self.h

    def __exit__(self, *a):
        torch.cuda.synchronize()
        fx.flex_comm_destroy(self.h)


def assert_same_bits(got: torch.Tensor, want_bits: np.ndarray, what=""):
    got_bits = wl.to_numpy_bits(got)
    if got.dtype == torch.float32:
        g, w = got_bits.view(np.uint32), want_bits.view(np.uint32)
        nan, got_nan = np.isnan(want_bits), np.isnan(got_bits)
    elif got.dtype == torch.float16:
        g, w = got_bits.view(np.uint16), want_bits.view(np.uint16)
        nan, got_nan = np.isnan(want_bits), np.isnan(got_bits)
    else:
        g, w = got_bits, want_bits
        nan = ((w & 0x7F80) == 0x7F80) & ((w & 0x7F) != 0)
        got_nan = ((g & 0x7F80) == 0x7F80) & ((g & 0x7F) != 0)
    assert g.shape == w.shape, what
    bad = (g != w) & ~nan
    if bad.any():
        i = int(np.flatnonzero(bad)[0])
        raise AssertionError("%s: %d of %d elements differ, first at %d: got 0x%x want 0x%x"
                             % (what, int(bad.sum()), g.size, i, int(g[i]), int(w[i])))
    assert np.array_equal(nan, got_nan), what + ": NaN positions differ"


def oracle_allreduce(bufs):
    return oc.allreduce([wl.to_numpy_bits(b) for b in bufs])


def oracle_allgather(slices):
    return oc.allgather([wl.to_numpy_bits(b) for b in slices])


COUNTS = [0, 1, 7, 8, 9, 2047, 2048, 2049, 65536, (1 << 20) + 3]


# ---- the balancer on hardware, replayed through the oracle ----------------
#
# The library's Stage 1 and Stage 2 run on times measured on the GPU.  The same
# times are fed to oracle/balancer.py, which must then take the same decisions:
# same shares after every Algorithm-1 iteration and after every adaptive call.

def live_set(mask, npaths):
    return {p for p in range(npaths) if mask >> p & 1}


def ceiling(cfg, npaths):
    return [None] + [cfg.max_host_units] * (npaths - 1)


def check_stage1_against_oracle(comm, coll, count, dtype, res, cfg, npaths=2):
    bc = cfg.balancer
    # InitializeShares: bandwidth-proportional, a host path never above its ceiling
    want0 = ob.initialize_shares(list(res.path_bw)[:npaths], bc.share_total)
    for p in range(1, npaths):
        excess = max(want0[p] - cfg.max_host_units, 0)
        want0[p] -= excess
        want0[0] += excess
    assert list(res.initial_shares)[:npaths] == want0
    rounds, nrounds = fx.flex_comm_tune_trace(comm, coll, count, dtype)
    assert nrounds == res.iterations == len(rounds)
    pending = list(rounds)

    def replay(S, live):
        r = pending.pop(0)
        assert list(r.shares_before)[:npaths] == S, "the library measured at other shares than the oracle holds"
        return list(r.path_time_s)[:npaths]
    trace = []
    S, live = ob.initial_tune(want0, replay, step0=bc.initial_step, threshold=bc.convergence_threshold,
                              stability_required=bc.stability_required, max_iters=bc.max_tune_iters, trace=trace,
                              cap=ceiling(cfg, npaths))
    assert not pending, "the library ran more Algorithm-1 iterations than the oracle"
    assert len(trace) == nrounds
    for t, r in zip(trace, rounds):
        assert t["S"] == list(r.shares_after)[:npaths] and t["step"] == r.step_after
        assert set(t["active"]) == live_set(r.active_after, npaths)
    assert S == list(res.balanced_shares)[:npaths]
    if not res.reverted:
        assert S == list(res.shares)[:npaths] and live == live_set(res.active_mask, npaths)
    return trace


class Stage2Twin:
    """oracle.balancer.RuntimeAdjuster fed with the times the library's Evaluator read back."""

    def __init__(self, comm, coll, count, dtype, cfg, npaths=2):
        self.args = (comm, coll, count, dtype)
        self.npaths = npaths
        st = fx.flex_get_stats(*self.args)
        assert st.balancer.stage == fx.FLEX_STAGE_RUNTIME and st.balancer.window_fill == 0
        bc = cfg.balancer
        self.twin = ob.RuntimeAdjuster(list(st.balancer.shares)[:npaths], live_set(st.balancer.active_mask, npaths),
                                       window=bc.window, threshold=bc.runtime_threshold, step=bc.runtime_step,
                                       cap=ceiling(cfg, npaths))
        self.samples = st.samples
        self.moves = []

    def after_call(self):
        """Call after every adaptive collective call: drains the Evaluator and compares."""
        torch.cuda.synchronize()
        fx.flex_evaluator_drain(self.args[0])
        st = fx.flex_get_stats(*self.args)
        assert st.samples - self.samples in (0, 1)
        if st.samples > self.samples:                 # the call was split: one sample per call
            self.samples = st.samples
            before = list(self.twin.S)
            if self.twin.observe(list(st.last_time_s)[:self.npaths]):
                self.moves.append([b - a for a, b in zip(before, self.twin.S)])
        assert list(st.balancer.shares)[:self.npaths] == self.twin.S, "library and oracle shares differ"
        assert live_set(st.balancer.active_mask, self.npaths) == self.twin.C_active
        assert st.balancer.adjustments == self.twin.adjustments
        return st


# ------------------------------------------------------------ device path

@pytest.mark.parametrize("serial", [2, 0])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("nranks", [1, 2, 3, 8])
def test_allreduce_device_path_all_counts(dtype, nranks, serial):
    # serial 2: one load in flight per wavefront at every size; 0: every load of a tile at once
    # (the default, 1, picks between the two by message size)
    with Comm(nranks=nranks, reduce_serial_loads=serial) as comm:
        for count in COUNTS:
            say("allreduce device", dtype, nranks, count, "serial", serial)
            bufs = [wl.random_bits(count, dtype, 11 * r + count % 97, DEV, finite_only=True) for r in range(nranks)]
            # keep exponents within reach of each other so that roundings matter
            bufs = [torch.ldexp(torch.frexp(b.float())[0], torch.tensor(r % 3, device=DEV)).to(dtype) for r, b in enumerate(bufs)]
            out = torch.full((count + 8,), 7.0, dtype=dtype, device=DEV)
            fx.flex_allreduce_local(comm, bufs, out, count=count)
            torch.cuda.synchronize()
            assert_same_bits(out[:count], oracle_allreduce(bufs), "count %d" % count)
            assert torch.all(out[count:] == 7.0), "wrote past the end"


@pytest.mark.parametrize("serial", [2, 0])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
def test_allreduce_raw_bit_patterns_and_specials(dtype, serial):
    count = 300007
    with Comm(reduce_serial_loads=serial) as comm:
        bufs = [wl.random_bits(count, dtype, 500 + r, DEV) for r in range(8)]   # NaN, inf, denormals included
        out = torch.empty(count, dtype=dtype, device=DEV)
        fx.flex_allreduce_local(comm, bufs, out)
        torch.cuda.synchronize()
        assert_same_bits(out, oracle_allreduce(bufs), "raw bits")
        # denormal inputs and sums stay denormal (no flushing)
        tiny = torch.full((4099,), 1e-40 if dtype != torch.float16 else 6e-8, dtype=torch.float32, device=DEV).to(dtype)
        bufs = [tiny * (r + 1) for r in range(8)]
        out = torch.empty(4099, dtype=dtype, device=DEV)
        fx.flex_allreduce_local(comm, bufs, out)
        torch.cuda.synchronize()
        want = oracle_allreduce(bufs)
        assert want.view(np.uint32 if dtype == torch.float32 else np.uint16)[0] != 0
        assert_same_bits(out, want, "denormals")
        if dtype == torch.float16:
            # sums that land on the overflow threshold and in the subnormal range
            edge = torch.tensor([65504.0, 8190.0, 2.0 ** -24, 2.0 ** -14, 0.33], device=DEV).repeat(800).to(dtype)
            fx.flex_allreduce_local(comm, [edge] * 8, out[:4000], count=4000)
            torch.cuda.synchronize()
            assert_same_bits(out[:4000], oracle_allreduce([edge] * 8), "f16 edges")
        # signed zero: starts from rank 0's value
        neg0 = torch.full((1000,), -0.0, dtype=dtype, device=DEV)
        fx.flex_allreduce_local(comm, [neg0] * 8, out[:1000], count=1000)
        torch.cuda.synchronize()
        assert_same_bits(out[:1000], oracle_allreduce([neg0] * 8), "-0")


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
def test_allreduce_of_two_ranks_on_every_pair_of_bit_patterns(dtype):
    # N = 2 and all 2^32 ordered pairs (a, b) of 16-bit patterns: every accumulator a
    # single binary32 add of two widened inputs can produce goes through the kernel's
    # widening, add and narrowing (for binary16 the hardware converters) and through
    # the oracle's integer routines; the bits must agree wherever the sum is not a NaN.
    # Random patterns cannot cover this: the ties and the subnormal / overflow edges
    # of the narrowing are measure-zero sets.
    slab_bits = 27                                   # 2^27 pairs per slab, 32 slabs
    n = 1 << slab_bits
    a_per_slab = n >> 16
    idx = torch.arange(n, dtype=torch.int32, device=DEV)
    b_dev = (idx & 0xFFFF).to(torch.int16).view(dtype)           # b runs through all patterns, fastest
    hi_dev = (idx >> 16).to(torch.int32)
    del idx
    idx_np = np.arange(n, dtype=np.uint32)
    b_np = (idx_np & 0xFFFF).astype(np.uint16)
    hi_np = (idx_np >> 16).astype(np.uint16)
    del idx_np
    view = (lambda x: x) if dtype == torch.bfloat16 else (lambda x: x.view(np.float16))
    out = torch.empty(n, dtype=dtype, device=DEV)
    with Comm(nranks=2, max_bytes=2 * n) as comm:
        for slab in range(1 << (32 - slab_bits)):
            base = slab * a_per_slab
            a_dev = (hi_dev + base).to(torch.int16).view(dtype)
            fx.flex_allreduce_local(comm, [a_dev, b_dev], out)
            want = oc.allreduce([view(hi_np + np.uint16(base)), view(b_np)])
            torch.cuda.synchronize()
            assert_same_bits(out, want, "a = 0x%04x.., all b" % base)
            if slab % 8 == 0:
                say("pairs", dtype, "slab", slab, "ok")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_allreduce_misaligned_pointers_and_in_place(dtype):
    count = 100003
    with Comm() as comm:
        base = wl.make_rank_buffers(wl.config(0 if dtype == torch.float32 else 1), DEV, count=count + 64)
        # same misalignment everywhere (vector body with a scalar head)
        for off in (1, 3, 5):
            bufs = [b[off:off + count] for b in base]
            out_full = torch.zeros(count + 64, dtype=dtype, device=DEV)
            out = out_full[off:off + count]
            fx.flex_allreduce_local(comm, bufs, out)
            torch.cuda.synchronize()
            assert_same_bits(out, oracle_allreduce(bufs), "offset %d" % off)
            assert out_full[:off].abs().sum() == 0 and out_full[off + count:].abs().sum() == 0
        # different misalignment per rank (element-wise path)
        bufs = [b[r:r + count] for r, b in enumerate(base)]
        out = torch.zeros(count + 2, dtype=dtype, device=DEV)[2:]
        fx.flex_allreduce_local(comm, bufs, out)
        torch.cuda.synchronize()
        assert_same_bits(out, oracle_allreduce(bufs), "mixed offsets")
        # in place: out is rank 3's buffer
    with Comm(rank=3, max_host_units=10000) as comm:
        for units in (0, 1200):
            bufs = [b[:count].clone() for b in base]
            want = oracle_allreduce(bufs)
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
            fx.flex_allreduce_local(comm, bufs, bufs[3])
            torch.cuda.synchronize()
            assert_same_bits(bufs[3], want, "in place units %d" % units)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("nranks", [1, 2, 8])
def test_allgather_device_path_all_counts(dtype, nranks):
    with Comm(nranks=nranks) as comm:
        for count in COUNTS:
            say("allgather device", dtype, nranks, count)
            slices = [wl.random_bits(count, dtype, 31 * r + count % 89, DEV) for r in range(nranks)]
            out = torch.full((nranks * count + 8,), 7.0, dtype=dtype, device=DEV)
            fx.flex_allgather_local(comm, slices, out, slice_count=count)
            torch.cuda.synchronize()
            want = oracle_allgather(slices)
            assert wl.to_numpy_bits(out[:nranks * count]).tobytes() == want.tobytes(), count
            assert torch.all(out[nranks * count:] == 7.0)


def test_allgather_misaligned_and_in_place():
    dtype = torch.bfloat16
    count = 70001                       # odd: every destination slice lands on a different alignment
    with Comm(rank=2, max_host_units=10000) as comm:
        base = [wl.random_bits(count + 16, dtype, 700 + r, DEV) for r in range(8)]
        slices = [b[r % 5:r % 5 + count] for r, b in enumerate(base)]
        want = oracle_allgather(slices)
        for units in (0, 700):
            fx.flex_set_split(comm, fx.FLEX_ALLGATHER, fx.FLEX_SPLIT_STATIC, units)
            out = torch.zeros(8 * count + 3, dtype=dtype, device=DEV)[3:]
            fx.flex_allgather_local(comm, slices, out)
            torch.cuda.synchronize()
            assert wl.to_numpy_bits(out).tobytes() == want.tobytes(), units
            # in place: rank 2's slice already sits at its offset
            out2 = torch.zeros(8 * count, dtype=dtype, device=DEV)
            out2[2 * count:3 * count] = slices[2]
            sl = list(slices)
            sl[2] = out2[2 * count:3 * count]
            fx.flex_allgather_local(comm, sl, out2)
            torch.cuda.synchronize()
            assert wl.to_numpy_bits(out2).tobytes() == want.tobytes(), ("in place", units)


@pytest.mark.parametrize("shape", [fx.FLEX_SHAPE_WAVE, fx.FLEX_SHAPE_BLOCK])
@pytest.mark.parametrize("nt", [0, 1, 3])
def test_every_launch_shape_gives_the_same_bits(shape, nt):
    count = (1 << 21) + 12345
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    want_ar = oracle_allreduce(bufs)
    want_ag = oracle_allgather(bufs)
    for serial in (0, 1, 2):
        with Comm(launch_shape=shape, reduce_serial_loads=serial, reduce_nontemporal=nt, copy_nontemporal=nt) as comm:
            out = torch.empty(count, dtype=torch.bfloat16, device=DEV)
            fx.flex_allreduce_local(comm, bufs, out)
            out2 = torch.empty(8 * count, dtype=torch.bfloat16, device=DEV)
            fx.flex_allgather_local(comm, bufs, out2)
            torch.cuda.synchronize()
            assert_same_bits(out, want_ar, "allreduce, serial %d" % serial)
            assert wl.to_numpy_bits(out2).tobytes() == want_ag.tobytes()
    for bad in (dict(reduce_nontemporal=2), dict(copy_nontemporal=4), dict(launch_shape=2)):
        with pytest.raises(fx.FlexError):
            Comm(**bad).__enter__()


@pytest.mark.parametrize("reserve", [0, 5632, 40000])
def test_occupancy_cap_of_long_reduce_launches_does_not_change_the_bits(reserve):
    # long launches of the one-load-in-flight schedule reserve LDS they never use, only to
    # hold fewer wavefronts per compute unit; 96 MiB per rank with 8 and with 4 ranks takes
    # that path (3 and 2 ranks never do; 2 ranks keep both loads in flight)
    count = 48 * wl.MIB + 2048 + 3
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    for nranks in (8, 4, 3, 2):
        want = oracle_allreduce(bufs[:nranks])
        with Comm(nranks=nranks, max_bytes=count * 2, reduce_lds_reserve=reserve) as comm:
            out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
            fx.flex_allreduce_local(comm, bufs[:nranks], out)
            torch.cuda.synchronize()
            assert_same_bits(out, want, "reserve %d, %d ranks" % (reserve, nranks))
    with pytest.raises(fx.FlexError):
        Comm(reduce_lds_reserve=70000).__enter__()


# ---------------------------------------------------------- ReduceScatter

@pytest.mark.parametrize("engine", [0, 1, 2])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
def test_reducescatter_is_the_rank_slice_and_composes_to_allreduce(dtype, engine):
    n = 8
    for rc in (0, 1, 2049, 65536 + 7, (1 << 18) + 2048):
        total = n * rc
        w = wl.config(0) if dtype == torch.float32 else wl.config(2)
        bufs = [b.to(dtype) for b in wl.make_rank_buffers(w, DEV, count=total)]
        if dtype == torch.float16:
            bufs = [b * 50 for b in bufs]
        host = [wl.to_numpy_bits(b) for b in bufs]
        want_full = oc.allreduce(host) if total else None
        reduced = []
        for rank in range(n):
            with Comm(rank=rank, max_host_units=10000, host_engine=engine) as comm:
                units = (0, 900, 10000)[rank % 3]
                fx.flex_set_split(comm, fx.FLEX_REDUCESCATTER, fx.FLEX_SPLIT_STATIC, units)
                out = torch.full((rc + 4,), 3.0, dtype=dtype, device=DEV)
                fx.flex_reducescatter_local(comm, bufs, out, recv_count=rc)
                torch.cuda.synchronize()
                if rc:
                    assert_same_bits(out[:rc], oc.reducescatter(host, rank), "rank %d rc %d" % (rank, rc))
                assert torch.all(out[rc:] == 3.0)
                reduced.append(out[:rc].clone())
        if rc:
            # all-gather of the reduced slices = the AllReduce result
            with Comm(max_host_units=10000) as comm:
                full = torch.zeros(total, dtype=dtype, device=DEV)
                fx.flex_allgather_local(comm, reduced, full)
                torch.cuda.synchronize()
                assert_same_bits(full, want_full, "reduce-scatter + all-gather, rc %d" % rc)


# --------------------------------------------------------------- AllToAll

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_alltoall_receive_buffer(dtype):
    n = 8
    for cnt in (0, 1, 2049, 40001, (1 << 17) + 2048):
        bufs = [wl.random_bits(n * cnt, dtype, 60 + r, DEV) for r in range(n)]
        host = [wl.to_numpy_bits(b) for b in bufs]
        for rank, units, engine, paths in ((0, 0, 0, 1), (3, 1500, 0, 1), (7, 1500, 1, 1), (2, 1500, 2, 1), (5, 700, 0, 2),
                                           (6, 700, 1, 2), (4, 700, 2, 2)):
            with Comm(rank=rank, max_host_units=10000, host_engine=engine, num_aux_paths=paths,
                      min_step_bytes=16 << 10) as comm:
                fx.flex_set_split_paths(comm, fx.FLEX_ALLTOALL, fx.FLEX_SPLIT_STATIC, (units,) * paths)
                out = torch.full((n * cnt + 4,), 3.0, dtype=dtype, device=DEV)
                fx.flex_alltoall_local(comm, bufs, out, count=cnt)
                torch.cuda.synchronize()
                if cnt:
                    assert wl.to_numpy_bits(out[:n * cnt]).tobytes() == oc.alltoall(host, rank).tobytes(), (cnt, rank)
                assert torch.all(out[n * cnt:] == 3.0)


# ------------------------------------------ seeded random differential test

def test_random_calls_of_all_four_collectives_match_the_oracle():
    # 600 seeded cases: collective, element type, rank count, local rank, count,
    # per-buffer misalignment, host share, engine, hand-over and step size all
    # drawn at random; raw bit patterns as data; guard elements around the output
    import random
    rng = random.Random(20251015)
    dtypes = [torch.float32, torch.bfloat16, torch.float16]
    comms = {}

    def comm_for(nranks, rank, engine, sync, chunk, shift, paths):
        key = (nranks, rank, engine, sync, chunk, shift, paths)
        if key not in comms:
            if len(comms) >= 24:                         # bound the pinned memory held at once
                torch.cuda.synchronize()
                fx.flex_comm_destroy(comms.pop(next(iter(comms))))
            cfg = fx.flex_config_default()
            cfg.max_host_units, cfg.host_engine, cfg.slot_sync = 10000, engine, sync
            cfg.chunk_bytes, cfg.host_die_shift, cfg.num_aux_paths = chunk, shift, paths
            cfg.reduce_serial_loads = (engine + sync + shift) % 3
            cfg.min_step_bytes, cfg.min_split_bytes = 8 << 10, 4 << 10
            comms[key] = fx.flex_comm_create(nranks, rank, 16 << 20, cfg)
        return comms[key]

    try:
        for case in range(600):
            coll = rng.choice(["allreduce", "allgather", "reducescatter", "alltoall"])
            dtype = rng.choice(dtypes)
            es = 4 if dtype == torch.float32 else 2
            nranks = rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 8, 8])
            rank = rng.randrange(nranks)
            count = rng.choice([0, 1, rng.randrange(2, 64), rng.randrange(64, 5000), rng.randrange(5000, 300000),
                                1 << rng.randrange(4, 18), (1 << rng.randrange(4, 18)) + rng.choice([-1, 1, 3])])
            per_rank = count * nranks if coll in ("reducescatter", "alltoall") else count
            same_lead = rng.random() < 0.6               # all buffers congruent modulo 16 bytes, or not
            lead0 = rng.randrange(0, 16 // es)
            leads = [lead0 if same_lead else rng.randrange(0, 16 // es) for _ in range(nranks)]
            out_lead = lead0 if rng.random() < 0.7 else rng.randrange(0, 16 // es)
            engine, sync = rng.randrange(3), rng.randrange(2)
            chunk = rng.choice([16 << 10, 64 << 10, 1 << 20])
            shift, paths = rng.randrange(4), rng.choice([1, 1, 2])
            units = rng.choice([0, 1, 37, 500, 2500, 6000, 10000])
            units2 = rng.choice([0, 300, 2000]) if units + 2000 <= 10000 else 0
            say("random case", case, coll, dtype, "n", nranks, "rank", rank, "count", count, "leads", leads, out_lead,
                "engine", engine, "sync", sync, "chunk", chunk, "shift", shift, "paths", paths, "units", units, units2)
            raw = [wl.random_bits(per_rank + 8, dtype, 7000 + 10 * case + r, DEV) for r in range(nranks)]
            bufs = [raw[r][leads[r]:leads[r] + per_rank] for r in range(nranks)]
            host = [wl.to_numpy_bits(b) for b in bufs]
            out_count = {"allreduce": count, "allgather": nranks * count, "reducescatter": count,
                         "alltoall": nranks * count}[coll]
            guard = wl.random_bits(out_count + 24, dtype, 9000 + case, DEV, finite_only=True)
            before = wl.to_numpy_bits(guard).copy()
            out = guard[out_lead + 4:out_lead + 4 + out_count]
            comm = comm_for(nranks, rank, engine, sync, chunk, shift, paths)
            code = {"allreduce": fx.FLEX_ALLREDUCE, "allgather": fx.FLEX_ALLGATHER,
                    "reducescatter": fx.FLEX_REDUCESCATTER, "alltoall": fx.FLEX_ALLTOALL}[coll]
            # a one-rank communicator has no peers and therefore no host path
            fx.flex_set_split_paths(comm, code, fx.FLEX_SPLIT_STATIC, (units, units2)[:paths] if nranks > 1 else ())
            if coll == "allreduce":
                fx.flex_allreduce_local(comm, bufs, out, count=count)
                want = oc.allreduce(host) if count else None
            elif coll == "allgather":
                fx.flex_allgather_local(comm, bufs, out, slice_count=count)
                want = oc.allgather(host) if count else None
            elif coll == "reducescatter":
                fx.flex_reducescatter_local(comm, bufs, out, recv_count=count)
                want = oc.reducescatter(host, rank) if count else None
            else:
                fx.flex_alltoall_local(comm, bufs, out, count=count)
                want = oc.alltoall(host, rank) if count else None
            torch.cuda.synchronize()
            after = wl.to_numpy_bits(guard)
            lo, hi = out_lead + 4, out_lead + 4 + out_count
            assert after[:lo].tobytes() == before[:lo].tobytes(), "case %d wrote in front of out" % case
            assert after[hi:].tobytes() == before[hi:].tobytes(), "case %d wrote behind out" % case
            if count:
                if coll in ("allreduce", "reducescatter"):
                    assert_same_bits(out, want, "case %d" % case)
                else:
                    assert after[lo:hi].tobytes() == want.tobytes(), "case %d" % case
    finally:
        torch.cuda.synchronize()
        for h in comms.values():
            fx.flex_comm_destroy(h)


# ------------------------------------------------- split over both paths

ENGINES = [fx.FLEX_ENGINE_KERNEL, fx.FLEX_ENGINE_HYBRID, fx.FLEX_ENGINE_SDMA]


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_allreduce_bits_do_not_depend_on_split_chunk_or_rank(dtype, engine):
    count = (1 << 20) + 3
    w = wl.config(0) if dtype == torch.float32 else wl.config(2)
    bufs = wl.make_rank_buffers(w, DEV, count=count)
    want = oracle_allreduce(bufs)
    for chunk, slots, min_step in ((64 << 10, 2, 4 << 10), (4 << 20, 2, 4 << 20), (256 << 10, 3, 32 << 10),
                                   (4 << 20, 1, 32 << 10)):
        for rank in (0, 3, 7):
            with Comm(rank=rank, max_host_units=10000, chunk_bytes=chunk, num_slots=slots, host_engine=engine,
                      min_step_bytes=min_step) as comm:
                for units in (0, 1, 500, 1200, 2200, 10000):
                    say("allreduce split", dtype, chunk, rank, units)
                    fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
                    out = torch.zeros(count, dtype=dtype, device=DEV)
                    fx.flex_allreduce_local(comm, bufs, out)
                    torch.cuda.synchronize()
                    assert_same_bits(out, want, "chunk %d rank %d units %d" % (chunk, rank, units))
                    st = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, count, dtype)
                    assert st.last_split == op.partition(count, units, 10000, 2048, (64 << 10) // out.element_size())


@pytest.mark.parametrize("engine", ENGINES)
def test_allgather_bits_do_not_depend_on_split_chunk_or_rank(engine):
    dtype = torch.bfloat16
    count = (1 << 19) + 5
    slices = [wl.random_bits(count, dtype, 40 + r, DEV) for r in range(8)]
    want = oracle_allgather(slices).tobytes()
    for chunk in (64 << 10, 4 << 20):
        for rank in (0, 5):
            with Comm(rank=rank, max_host_units=10000, chunk_bytes=chunk, host_engine=engine) as comm:
                for units in (0, 1, 500, 2200, 10000):
                    say("allgather split", chunk, rank, units)
                    fx.flex_set_split(comm, fx.FLEX_ALLGATHER, fx.FLEX_SPLIT_STATIC, units)
                    out = torch.zeros(8 * count, dtype=dtype, device=DEV)
                    fx.flex_allgather_local(comm, slices, out)
                    torch.cuda.synchronize()
                    assert wl.to_numpy_bits(out).tobytes() == want, (chunk, rank, units)


@pytest.mark.parametrize("engine", [fx.FLEX_ENGINE_HYBRID, fx.FLEX_ENGINE_KERNEL])
@pytest.mark.parametrize("shift", [0, 1, 2, 3])
def test_host_kernels_confined_to_fewer_dies_give_the_same_bits(shift, engine):
    # the host-path grids are 2^shift times larger and only every 2^shift-th
    # workgroup works; ragged counts, every alignment fallback of the copy
    count = (1 << 20) + 2048 + 5
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    want_ar = oracle_allreduce(bufs)
    want_ag = oracle_allgather(bufs).tobytes()
    for blocks in (1, 16, 100):
        with Comm(max_host_units=10000, host_blocks=blocks, host_die_shift=shift, chunk_bytes=256 << 10,
                  min_step_bytes=32 << 10, host_engine=engine) as comm:
            for units in (1, 700, 10000):
                say("die shift", shift, blocks, units)
                fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
                fx.flex_set_split(comm, fx.FLEX_ALLGATHER, fx.FLEX_SPLIT_STATIC, units)
                out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
                fx.flex_allreduce_local(comm, bufs, out)
                big = torch.zeros(8 * count + 8, dtype=torch.bfloat16, device=DEV)
                for lead in (0, 1):               # 1: output 2 bytes off the inputs' alignment
                    fx.flex_allgather_local(comm, bufs, big[lead:lead + 8 * count])
                    torch.cuda.synchronize()
                    assert wl.to_numpy_bits(big[lead:lead + 8 * count]).tobytes() == want_ag, (blocks, units, lead)
                assert_same_bits(out, want_ar, "blocks %d units %d" % (blocks, units))
    with pytest.raises(fx.FlexError):
        Comm(host_die_shift=4).__enter__()


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("collective", ["allreduce", "allgather"])
def test_counter_handshake_gives_the_same_bits(engine, collective):
    # slots handed over by monotonically increasing counters and stream memory
    # operations instead of events; small chunks so that every slot is reused
    # many times within a call and across calls
    count = (1 << 20) + 4096 + 3
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    want = oracle_allreduce(bufs) if collective == "allreduce" else oracle_allgather(bufs)
    for slots in (1, 2, 3):
        with Comm(max_host_units=10000, chunk_bytes=64 << 10, num_slots=slots, host_engine=engine,
                  slot_sync=fx.FLEX_SYNC_COUNTERS, min_step_bytes=16 << 10) as comm:
            for call, units in enumerate((300, 2200, 1, 10000, 300)):
                say("counters", collective, engine, slots, units)
                if collective == "allreduce":
                    fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
                    out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
                    fx.flex_allreduce_local(comm, bufs, out)
                    torch.cuda.synchronize()
                    assert_same_bits(out, want, "slots %d units %d" % (slots, units))
                else:
                    fx.flex_set_split(comm, fx.FLEX_ALLGATHER, fx.FLEX_SPLIT_STATIC, units)
                    out = torch.zeros(8 * count, dtype=torch.bfloat16, device=DEV)
                    fx.flex_allgather_local(comm, bufs, out)
                    torch.cuda.synchronize()
                    assert wl.to_numpy_bits(out).tobytes() == want.tobytes(), (slots, units)
            # and queued back to back without host synchronisation
            if collective == "allreduce":
                fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, 700)
                outs = [torch.zeros(count, dtype=torch.bfloat16, device=DEV) for _ in range(12)]
                for o in outs:
                    fx.flex_allreduce_local(comm, bufs, o)
                torch.cuda.synchronize()
                for k, o in enumerate(outs):
                    assert_same_bits(o, want, "queued call %d" % k)


@pytest.mark.parametrize("engine", ENGINES)
def test_back_to_back_calls_on_one_stream_and_repeatability(engine):
    # many split calls queued without host synchronisation, staging slots and
    # scratch reused every call: every output must carry the same bits
    count = (1 << 20) + 2048 + 1
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    want = oracle_allreduce(bufs)
    stream = torch.cuda.Stream()
    with Comm(chunk_bytes=128 << 10, host_engine=engine, min_step_bytes=16 << 10) as comm:
        fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, 700)
        outs = [torch.zeros(count, dtype=torch.bfloat16, device=DEV) for _ in range(50)]
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            for o in outs:
                fx.flex_allreduce_local(comm, bufs, o, stream=stream)
        stream.synchronize()
        for k, o in enumerate(outs):
            assert_same_bits(o, want, "call %d" % k)
        fx.flex_evaluator_drain(comm)
        st = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16)
        assert st.calls == 50 and st.split_calls == 50 and st.samples == 50 and st.blocking_reads == 0
        assert st.last_time_s[0] > 0 and st.last_time_s[1] > 0


def test_unsampled_split_calls_use_ordering_only_events_and_give_the_same_bits():
    # sample_every = 4: three of four split calls record no timing events and take no
    # Evaluator record; results and Stage 2 are unaffected apart from the sampling rate
    count = (1 << 20) + 2048 + 9
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    want = oracle_allreduce(bufs)
    want_ag = oracle_allgather(bufs)
    cfg = fx.flex_config_default()
    with Comm(sample_every=4, chunk_bytes=128 << 10, min_step_bytes=16 << 10, num_aux_paths=2,
              max_host_units=5000) as comm:
        fx.flex_set_split_paths(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, (900, 300))
        fx.flex_set_split_paths(comm, fx.FLEX_ALLGATHER, fx.FLEX_SPLIT_STATIC, (700, 0))
        outs = [torch.zeros(count, dtype=torch.bfloat16, device=DEV) for _ in range(20)]
        outs_ag = [torch.zeros(8 * count, dtype=torch.bfloat16, device=DEV) for _ in range(4)]
        for k, o in enumerate(outs):
            fx.flex_allreduce_local(comm, bufs, o)
            if k % 5 == 0:
                fx.flex_allgather_local(comm, bufs, outs_ag[k // 5])
        torch.cuda.synchronize()
        for k, o in enumerate(outs):
            assert_same_bits(o, want, "call %d" % k)
        for o in outs_ag:
            assert np.array_equal(wl.to_numpy_bits(o), want_ag)
        fx.flex_evaluator_drain(comm)
        st = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16)
        sg = fx.flex_get_stats(comm, fx.FLEX_ALLGATHER, count, torch.bfloat16)
        assert st.split_calls == 20 and sg.split_calls == 4
        assert st.samples + sg.samples == 24 // 4          # every fourth split call of the communicator
        assert st.last_time_s[0] > 0 and st.last_time_s[1] > 0 and st.last_time_s[2] > 0
        # Stage 2 still runs, on every fourth call
        fx.flex_comm_set_shares(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, [9000, 1000, 0])
        fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_ADAPTIVE)
        out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
        for k in range(4 * cfg.balancer.window):
            fx.flex_allreduce_local(comm, bufs, out)
            torch.cuda.synchronize()
            fx.flex_evaluator_drain(comm)
        st = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16)
        assert st.balancer.adjustments == 1 and list(st.balancer.shares)[:2] == [9004, 996]
        assert_same_bits(out, want, "adaptive, sampled every fourth call")
    with pytest.raises(fx.FlexError):
        Comm(sample_every=0).__enter__()


# ------------------------------------------------------------ three paths

def test_device_path_calls_replay_from_a_graph_and_split_calls_refuse_capture():
    # launch-bound small messages: a captured sequence of device-path calls must
    # give the oracle's bits on every replay, with eager work between replays
    w = wl.config(0)
    bufs = wl.make_rank_buffers(w, DEV)
    want_ar = oracle_allreduce(bufs)
    slices = [b[:4099] for b in bufs]
    want_ag = oracle_allgather(slices).tobytes()
    outs = [torch.zeros(w.count, dtype=w.dtype, device=DEV) for _ in range(6)]
    gathered = torch.zeros(8 * 4099, dtype=w.dtype, device=DEV)
    with Comm(max_host_units=10000) as comm:
        # one split call still in flight in the Evaluator's ring while capturing
        fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, 5000)
        fx.flex_allreduce_local(comm, bufs, outs[0])
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            with pytest.raises(fx.FlexError):                      # host share 50 %: refused, nothing enqueued
                fx.flex_allreduce_local(comm, bufs, outs[0], stream=stream)
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, 0)
            for o in outs:
                fx.flex_allreduce_local(comm, bufs, o, stream=stream)
            fx.flex_allgather_local(comm, slices, gathered, stream=stream)
        torch.cuda.synchronize()
        for replay in range(4):
            say("graph replay", replay)
            for o in outs:
                o.zero_()
            gathered.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for k, o in enumerate(outs):
                assert_same_bits(o, want_ar, "replay %d call %d" % (replay, k))
            assert wl.to_numpy_bits(gathered).tobytes() == want_ag, replay
            # the communicator still works eagerly between replays, split included
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, 3000)
            eager = torch.zeros(w.count, dtype=w.dtype, device=DEV)
            fx.flex_allreduce_local(comm, bufs, eager)
            torch.cuda.synchronize()
            assert_same_bits(eager, want_ar, "eager after replay %d" % replay)
        fx.flex_evaluator_drain(comm)
        del graph


@pytest.mark.parametrize("first_engine", ENGINES)
@pytest.mark.parametrize("sync", [fx.FLEX_SYNC_EVENTS, fx.FLEX_SYNC_COUNTERS])
def test_three_paths_give_the_same_bits(first_engine, sync):
    # device path + two host-staged paths (copy kernels and DMA engines) at once
    count = (1 << 21) + 2048 * 3 + 5
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    host = [wl.to_numpy_bits(b) for b in bufs]
    want_ar, want_ag = oc.allreduce(host), oc.allgather(host)
    rs_bufs = [b[:8 * (count // 8)] for b in bufs]
    for rank in (0, 6):
        with Comm(rank=rank, max_host_units=10000, num_aux_paths=2, host_engine=first_engine, slot_sync=sync,
                  chunk_bytes=256 << 10, min_step_bytes=32 << 10) as comm:
            for shares in ((300, 500), (0, 700), (700, 0), (1, 1), (2500, 2500), (5000, 5000), (0, 10000)):
                say("three paths", first_engine, sync, rank, shares)
                for coll in (fx.FLEX_ALLREDUCE, fx.FLEX_ALLGATHER, fx.FLEX_REDUCESCATTER):
                    fx.flex_set_split_paths(comm, coll, fx.FLEX_SPLIT_STATIC, shares)
                out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
                fx.flex_allreduce_local(comm, bufs, out)
                out_ag = torch.zeros(8 * count, dtype=torch.bfloat16, device=DEV)
                fx.flex_allgather_local(comm, bufs, out_ag)
                out_rs = torch.zeros(count // 8, dtype=torch.bfloat16, device=DEV)
                fx.flex_reducescatter_local(comm, rs_bufs, out_rs)
                torch.cuda.synchronize()
                assert_same_bits(out, want_ar, "allreduce %s" % (shares,))
                assert wl.to_numpy_bits(out_ag).tobytes() == want_ag.tobytes(), shares
                assert_same_bits(out_rs, oc.reducescatter([wl.to_numpy_bits(b) for b in rs_bufs], rank),
                                 "reducescatter %s" % (shares,))
                st = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16)
                assert st.npaths == 3
                assert list(st.last_start)[:3] == op.partition_paths(count, [0, *shares], 10000, 2048, 32768)[:3]
            fx.flex_evaluator_drain(comm)
            st = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16)
            assert st.samples == st.split_calls == 7
            with pytest.raises(fx.FlexError):
                fx.flex_set_split_paths(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, (6000, 6000))
    with Comm() as comm:       # one host path only: a share for a second one is refused
        with pytest.raises(fx.FlexError):
            fx.flex_set_split_paths(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, (100, 100))


def test_three_path_balancer_on_hardware():
    # Algorithm 1 with three real paths, then Stage 2 from installed shares; every
    # decision is checked against the oracle fed with the same measured times
    count = 64 * wl.MIB        # 128 MiB per rank
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    want = oracle_allreduce(bufs)
    cfg = fx.flex_config_default()
    with Comm(max_bytes=count * 2, num_aux_paths=2) as comm:
        out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
        res = fx.flex_comm_tune(comm, fx.FLEX_ALLREDUCE, bufs, out)
        say("tune3", res.as_dict())
        torch.cuda.synchronize()
        assert_same_bits(out, want, "after tune")
        assert sum(res.shares) == 10000 and sum(res.initial_shares) == 10000 and res.iterations <= 100
        assert res.path_bw[0] > 0 and res.path_bw[1] > 0 and res.path_bw[2] > 0
        trace = check_stage1_against_oracle(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, res, cfg, npaths=3)
        say("stage 1 on three paths:", [(t["slow"], t["S"]) for t in trace])
        if res.reverted:
            assert list(res.shares)[:3] == [10000, 0, 0]
        # Stage 2 on three live paths
        fx.flex_comm_set_shares(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, [9880, 60, 60])
        fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_ADAPTIVE)
        twin = Stage2Twin(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, cfg, npaths=3)
        for k in range(60):
            fx.flex_allreduce_local(comm, bufs, out)
            st = twin.after_call()
            if k % 10 == 9:
                assert_same_bits(out, want, "adaptive call %d" % k)
        say("stage2 on three paths: moves", twin.moves, st.as_dict())
        assert st.samples == twin.samples and st.last_time_s[2] > 0 and len(twin.moves) <= 6
        for m in twin.moves:
            assert sorted(m) == [-4, 0, 4]          # one fixed step from one path to another


# --------------------------------------------------------- full-size configs

def test_config0_allreduce_f32_1MiB():
    w = wl.config(0)
    bufs = wl.make_rank_buffers(w, DEV)
    with Comm() as comm:
        out = torch.empty(w.count, dtype=w.dtype, device=DEV)
        fx.flex_allreduce_local(comm, bufs, out)
        torch.cuda.synchronize()
        assert_same_bits(out, oracle_allreduce(bufs), w.name)


def test_config1_allgather_bf16_256MiB():
    w = wl.config(1)
    slices = wl.make_rank_buffers(w, DEV)
    with Comm(max_bytes=w.bytes_per_rank) as comm:
        out = torch.empty(8 * w.count, dtype=w.dtype, device=DEV)
        fx.flex_allgather_local(comm, slices, out)
        torch.cuda.synchronize()
        assert wl.to_numpy_bits(out).tobytes() == oracle_allgather(slices).tobytes()


@pytest.mark.parametrize("engine", ENGINES)
def test_config2_allreduce_bf16_256MiB_split_sweep(engine):
    w = wl.config(2)
    say("generating", w.name)
    bufs = wl.make_rank_buffers(w, DEV)
    want = oracle_allreduce(bufs)
    with Comm(max_bytes=w.bytes_per_rank, host_engine=engine) as comm:
        for units in (0, 500, 1200, 2200):
            say("config2 units", units)
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
            out = torch.zeros(w.count, dtype=w.dtype, device=DEV)
            fx.flex_allreduce_local(comm, bufs, out)
            torch.cuda.synchronize()
            assert_same_bits(out, want, "%s units %d" % (w.name, units))


def sampled_windows(count, cuts=(), nwin=48, width=1 << 16, seed=5):
    """First, last, random windows and one across every cut, clipped to the message."""
    width = min(width, count)
    rng = np.random.default_rng(seed)
    starts = [0, count - width] + [int(x) for x in rng.integers(0, count - width + 1, nwin)]
    starts += [min(max(c - width // 2, 0), count - width) for c in cuts if 0 < c < count]
    return [(a, a + width) for a in starts]


class Config3Checker:
    """Compares an output of a configuration-3 case with the oracle: element by
    element up to 256 MiB per rank, above that on at least 50 windows (first,
    last, random, across every cut between two paths' pieces)."""

    def __init__(self, w, bufs):
        self.w, self.bufs = w, bufs
        self.is_ar = w.collective == "allreduce"
        self.full = w.bytes_per_rank <= 256 * wl.MIB
        if self.full:
            host = [wl.to_numpy_bits(b) for b in bufs]
            self.want = oc.allreduce(host) if self.is_ar else oc.allgather(host)

    def check(self, out, cuts, what):
        n = self.w.count
        if self.full:
            if self.is_ar:
                assert_same_bits(out, self.want, what)
            else:
                assert np.array_equal(wl.to_numpy_bits(out), self.want), what
            return
        for a, b in sampled_windows(n, cuts):
            host = [wl.to_numpy_bits(x[a:b]) for x in self.bufs]
            if self.is_ar:
                assert_same_bits(out[a:b], oc.allreduce(host), "%s window %d" % (what, a))
            else:
                got = torch.cat([out[r * n + a:r * n + b] for r in range(8)])
                assert np.array_equal(wl.to_numpy_bits(got), oc.allgather(host)), "%s window %d" % (what, a)


@pytest.mark.parametrize("mib", wl.SWEEP_MIB_PER_RANK)
@pytest.mark.parametrize("collective", ["allreduce", "allgather"])
def test_config3_sweep_point_under_its_own_protocol(collective, mib):
    # one point of the message-size sweep: Stage 1 on the hardware (rates, InitializeShares,
    # Algorithm 1, acceptance check), then 20 Stage-2 windows of adaptive calls; the output
    # is compared with the oracle after tuning and after the last window, every balancer
    # decision with the oracle balancer fed the same measured times.  If Stage 1 withdrew
    # the host path, a second leg installs the balanced shares so that three more windows
    # run with the host path live.
    w = [x for x in wl.sweep_workloads() if x.collective == collective and x.bytes_per_rank == mib * wl.MIB][0]
    say("generating", w.name)
    bufs = wl.make_rank_buffers(w, DEV)
    is_ar = collective == "allreduce"
    coll = fx.FLEX_ALLREDUCE if is_ar else fx.FLEX_ALLGATHER
    checker = Config3Checker(w, bufs)
    cfg = fx.flex_config_default()
    window = cfg.balancer.window

    def stats():
        return fx.flex_get_stats(comm, coll, w.count, w.dtype)

    with Comm(max_bytes=w.bytes_per_rank) as comm:
        out = torch.zeros(w.count if is_ar else 8 * w.count, dtype=w.dtype, device=DEV)

        def call():
            if is_ar:
                fx.flex_allreduce_local(comm, bufs, out)
            else:
                fx.flex_allgather_local(comm, bufs, out)

        res = fx.flex_comm_tune(comm, coll, bufs, out)
        say("tune", w.name, res.as_dict())
        torch.cuda.synchronize()
        checker.check(out, [stats().last_split], "after tune")
        check_stage1_against_oracle(comm, coll, w.count, w.dtype, res, cfg)

        fx.flex_set_split(comm, coll, fx.FLEX_SPLIT_ADAPTIVE)
        twin = Stage2Twin(comm, coll, w.count, w.dtype, cfg)
        trajectory = []
        for k in range(20 * window):
            if k == 20 * window - 1:
                out.zero_()
            share = twin.twin.S[1]
            call()
            st = twin.after_call()
            # the cut the call used is the oracle's cut for the share the oracle held
            assert st.last_split == op.partition(w.count, share, 10000, 2048, (64 << 10) // out.element_size())
            if k % window == window - 1:
                trajectory.append(twin.twin.S[1])
        say("host share after each of 20 windows:", trajectory)
        checker.check(out, [stats().last_split], "after 20 adaptive windows")

        if trajectory[-1] == 0:
            # host path withdrawn: run three windows with it live, from the shares Algorithm 1 balanced
            # at (or the probe share if it drained the path itself)
            units = res.balanced_shares[1] or res.initial_shares[1] or cfg.probe_units
            fx.flex_comm_set_shares(comm, coll, w.count, w.dtype, [10000 - units, units])
            twin = Stage2Twin(comm, coll, w.count, w.dtype, cfg)
            for k in range(3 * window):
                if k == 3 * window - 1:
                    out.zero_()
                share = twin.twin.S[1]
                call()
                st = twin.after_call()
                assert st.last_split == op.partition(w.count, share, 10000, 2048, (64 << 10) // out.element_size())
            say("host path live:", units, "->", twin.twin.S[1], "units; times", list(st.last_time_s)[:2])
            assert st.samples == twin.samples and st.split_calls >= 3 * window
            checker.check(out, [st.last_split], "host path live, after 3 windows")


@pytest.mark.parametrize("w", wl.evaluation_grid_workloads(), ids=lambda w: w.name)
def test_evaluation_grid_point(w):
    # One point of the paper's end-to-end grid (Evaluation, Table 2: AllReduce and AllGather
    # on 2, 4 and 8 ranks, 32..256 MiB) at full size, element by element: after Stage 1 on
    # the hardware (replayed through the oracle balancer), after a window of adaptive calls,
    # and with a static 5 % split so that the host path is live whatever Stage 1 decided.
    say("generating", w.name)
    n = w.nranks
    bufs = wl.make_rank_buffers(w, DEV)
    is_ar = w.collective == "allreduce"
    coll = fx.FLEX_ALLREDUCE if is_ar else fx.FLEX_ALLGATHER
    host = [wl.to_numpy_bits(b) for b in bufs]
    want = oc.allreduce(host) if is_ar else oc.allgather(host)
    del host
    cfg = fx.flex_config_default()

    def check(out, what):
        if is_ar:
            assert_same_bits(out, want, what)
        else:
            assert np.array_equal(wl.to_numpy_bits(out), want), what

    with Comm(nranks=n, rank=n - 1, max_bytes=w.bytes_per_rank) as comm:
        out = torch.zeros(w.count if is_ar else n * w.count, dtype=w.dtype, device=DEV)

        def call():
            if is_ar:
                fx.flex_allreduce_local(comm, bufs, out)
            else:
                fx.flex_allgather_local(comm, bufs, out)

        res = fx.flex_comm_tune(comm, coll, bufs, out)
        torch.cuda.synchronize()
        check(out, "after tune")
        check_stage1_against_oracle(comm, coll, w.count, w.dtype, res, cfg)
        say(w.name, "host share: initial", res.initial_shares[1], "balanced", res.balanced_shares[1],
            "kept" if not res.reverted else "reverted")

        fx.flex_set_split(comm, coll, fx.FLEX_SPLIT_ADAPTIVE)
        twin = Stage2Twin(comm, coll, w.count, w.dtype, cfg)
        for k in range(cfg.balancer.window):
            if k == cfg.balancer.window - 1:
                out.zero_()
            call()
            twin.after_call()
        check(out, "after a window of adaptive calls")

        out.zero_()
        fx.flex_set_split(comm, coll, fx.FLEX_SPLIT_STATIC, 500)
        call()
        torch.cuda.synchronize()
        st = fx.flex_get_stats(comm, coll, w.count, w.dtype)
        assert st.last_split == op.partition(w.count, 500, 10000, 2048, (64 << 10) // out.element_size()) < w.count
        check(out, "static 5 % split")


def test_messages_beyond_32_bit_element_counts_and_byte_offsets():
    # Two ranks of 2^31 + 2^26 + 37 bf16 elements (4 GiB + 128 MiB + 74 bytes each): element
    # indexes pass 2^31, byte offsets pass 2^32, and the AllGather's second slice starts
    # beyond 4 GiB.  Device path and a 1 % static split (the cut then lies beyond both
    # limits, so the host path's pieces start there), checked against the oracle on
    # windows at both ends, across 2^31 elements, across the cut and at random places.
    count = (1 << 31) + (1 << 26) + 37
    dtype = torch.bfloat16
    piece = 1 << 28
    bufs = []
    for r in range(2):
        t = torch.empty(count, dtype=dtype, device=DEV)
        for k, a in enumerate(range(0, count, piece)):
            wl.fill_rank(t[a:a + piece], "normal", 1.0, wl.rank_seed(9, r) + 100 * k)
        bufs.append(t)
    say("generated 2 x", count, "elements")
    landmarks = [1 << 31, (1 << 31) + 1024, count - 37]

    def windows(cut):
        return sampled_windows(count, [c for c in landmarks + [cut] if c], nwin=16, width=1 << 15)

    with Comm(nranks=2, rank=1, max_bytes=2 * count) as comm:
        out = torch.zeros(count, dtype=dtype, device=DEV)
        for units in (0, 100):
            out.zero_()
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
            fx.flex_allreduce_local(comm, bufs, out)
            torch.cuda.synchronize()
            cut = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, count, dtype).last_split
            assert cut == op.partition(count, units, 10000, 2048, (64 << 10) // 2)
            assert units == 0 or (1 << 31) < cut < count
            for a, b in windows(cut):
                assert_same_bits(out[a:b], oracle_allreduce([x[a:b] for x in bufs]), "AR %d units, window %d" % (units, a))
            say("allreduce", units, "units ok, cut", cut)
        del out
        out = torch.zeros(2 * count, dtype=dtype, device=DEV)
        for units in (0, 100):
            out.zero_()
            fx.flex_set_split(comm, fx.FLEX_ALLGATHER, fx.FLEX_SPLIT_STATIC, units)
            fx.flex_allgather_local(comm, bufs, out)
            torch.cuda.synchronize()
            cut = fx.flex_get_stats(comm, fx.FLEX_ALLGATHER, count, dtype).last_split
            assert cut == op.partition(count, units, 10000, 2048, (64 << 10) // 2)
            for a, b in windows(cut):
                got = torch.cat([out[r * count + a:r * count + b] for r in range(2)])
                want = oracle_allgather([x[a:b] for x in bufs])
                assert np.array_equal(wl.to_numpy_bits(got), want), "AG %d units, window %d" % (units, a)
            say("allgather", units, "units ok, cut", cut)


def test_config4_prefill_allreduce_adaptive_50_calls():
    w = wl.config(4)
    say("generating", w.name)
    bufs = wl.make_rank_buffers(w, DEV)
    want = oracle_allreduce(bufs)
    with Comm(max_bytes=w.bytes_per_rank) as comm:
        out = torch.zeros(w.count, dtype=w.dtype, device=DEV)
        res = fx.flex_comm_tune(comm, fx.FLEX_ALLREDUCE, bufs, out)
        say("tune:", res.as_dict())
        torch.cuda.synchronize()
        assert_same_bits(out, want, "after tune")
        assert sum(res.shares) == 10000 and res.path_bw[0] > 0
        check_stage1_against_oracle(comm, fx.FLEX_ALLREDUCE, w.count, w.dtype, res, fx.flex_config_default())
        fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_ADAPTIVE)
        outs = [torch.zeros(w.count, dtype=w.dtype, device=DEV) for _ in range(2)]
        for k in range(50):
            fx.flex_allreduce_local(comm, bufs, outs[k % 2])
        torch.cuda.synchronize()
        assert_same_bits(outs[0], want, "call 48")
        assert_same_bits(outs[1], want, "call 49")
        fx.flex_evaluator_drain(comm)
        st = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, w.count, w.dtype)
        say("stats:", st.as_dict())
        assert st.balancer.npaths == 2 and sum(st.balancer.shares) == 10000
        assert st.balancer.stage == fx.FLEX_STAGE_RUNTIME


# ------------------------------------------------------ balancer on hardware

def test_tune_then_adaptive_stays_exact_and_balanced():
    count = 16 * wl.MIB        # 32 MiB per rank, bf16
    bufs = wl.make_rank_buffers(wl.config(1), DEV, count=count)
    want_ag = oracle_allgather(bufs).tobytes()
    want_ar = oracle_allreduce(bufs)
    with Comm() as comm:
        out_ag = torch.zeros(8 * count, dtype=torch.bfloat16, device=DEV)
        out_ar = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
        for coll, out in ((fx.FLEX_ALLGATHER, out_ag), (fx.FLEX_ALLREDUCE, out_ar)):
            res = fx.flex_comm_tune(comm, coll, bufs, out)
            say("tune", coll, res.as_dict())
            assert sum(res.shares) == 10000 and res.iterations <= 100
            check_stage1_against_oracle(comm, coll, count, torch.bfloat16, res, fx.flex_config_default())
            if res.active_mask & 2:
                t = res.path_time_s
                # Algorithm 1 stopped either balanced or at the iteration cap
                assert res.iterations == 100 or abs(t[1] - t[0]) / min(t[0], t[1]) < 0.05 + 1e-9
            else:
                assert res.shares[1] == 0
            fx.flex_set_split(comm, coll, fx.FLEX_SPLIT_ADAPTIVE)
        for k in range(35):
            fx.flex_allgather_local(comm, bufs, out_ag)
            fx.flex_allreduce_local(comm, bufs, out_ar)
        torch.cuda.synchronize()
        assert wl.to_numpy_bits(out_ag).tobytes() == want_ag
        assert_same_bits(out_ar, want_ar, "adaptive allreduce")
        fx.flex_evaluator_drain(comm)
        for coll in (fx.FLEX_ALLGATHER, fx.FLEX_ALLREDUCE):
            st = fx.flex_get_stats(comm, coll, count, torch.bfloat16)
            say("stats", coll, st.as_dict())
            assert sum(st.balancer.shares) == 10000
            assert st.balancer.adjustments <= 3           # at most one move per 10-call window
        # a size class that was never tuned borrows the nearest tuned one
        half = [b[:count // 2] for b in bufs]
        fx.flex_allreduce_local(comm, half, out_ar[:count // 2], count=count // 2)
        torch.cuda.synchronize()
        assert_same_bits(out_ar[:count // 2], oracle_allreduce(half), "borrowed class")


@pytest.mark.parametrize("engine", ENGINES)
def test_stage2_runs_on_hardware(engine):
    # explicit shares keep the host path active, so the Evaluator feeds real
    # per-path times into Stage 2 while calls keep coming; the oracle's Stage 2,
    # fed the same times, must hold the same shares after every call
    count = 32 * wl.MIB        # 64 MiB per rank
    bufs = wl.make_rank_buffers(wl.config(1), DEV, count=count)
    want = oracle_allreduce(bufs)
    cfg = fx.flex_config_default()
    with Comm(max_bytes=count * 2, host_engine=engine) as comm:
        out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
        with pytest.raises(fx.FlexError):
            fx.flex_comm_set_shares(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, [9000, 999])
        fx.flex_comm_set_shares(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, [9900, 100])
        fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_ADAPTIVE)
        twin = Stage2Twin(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, cfg)
        trajectory = [100]
        for k in range(80):
            fx.flex_allreduce_local(comm, bufs, out)
            st = twin.after_call()
            if k % 10 == 9:
                assert_same_bits(out, want, "adaptive call %d" % k)
                trajectory.append(int(st.balancer.shares[1]))
                assert sum(st.balancer.shares) == 10000 and st.balancer.stage == fx.FLEX_STAGE_RUNTIME
        say("stats", st.as_dict(), trajectory, twin.moves)
        assert st.samples == 80 and st.split_calls == 80
        assert 1 <= st.balancer.adjustments <= 8                # the paths are far from balance at 1 %
        # every window moves at most one fixed step of 4 units, from the slower path to the device path
        assert all(m in ([4, -4], [-4, 4]) for m in twin.moves)
        # queued without draining in between, samples taken before a share change are dropped:
        # a move needs a full window of 10 samples at the current shares
        fx.flex_comm_set_shares(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, [9900, 100])
        for k in range(40):
            fx.flex_allreduce_local(comm, bufs, out)
        torch.cuda.synchronize()
        fx.flex_evaluator_drain(comm)
        st = fx.flex_get_stats(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16)
        assert st.balancer.adjustments <= 40 // 10 and sum(st.balancer.shares) == 10000
        assert (10000 - st.balancer.shares[0]) % 4 == 0
        assert_same_bits(out, want, "queued adaptive calls")


@pytest.mark.parametrize("coll", [fx.FLEX_REDUCESCATTER, fx.FLEX_ALLTOALL])
def test_tune_and_adaptive_calls_for_reducescatter_and_alltoall(coll):
    # the two other collectives through Stage 1 and Stage 2, against both oracles
    n, rank = 8, 5
    cnt = 4 * wl.MIB + 2048 + 3          # elements per slice / piece: 8 MiB of bf16 and a ragged end
    dtype = torch.bfloat16
    bufs = [wl.random_bits(n * cnt, dtype, 300 + r, DEV, finite_only=True) for r in range(n)]
    bufs = [torch.ldexp(torch.frexp(b.float())[0], torch.tensor(r % 3, device=DEV)).to(dtype) for r, b in enumerate(bufs)]
    host = [wl.to_numpy_bits(b) for b in bufs]
    is_rs = coll == fx.FLEX_REDUCESCATTER
    want = oc.reducescatter(host, rank) if is_rs else oc.alltoall(host, rank)
    cfg = fx.flex_config_default()
    with Comm(rank=rank, max_bytes=n * cnt * 2) as comm:
        out = torch.zeros(cnt if is_rs else n * cnt, dtype=dtype, device=DEV)

        def call():
            if is_rs:
                fx.flex_reducescatter_local(comm, bufs, out, recv_count=cnt)
            else:
                fx.flex_alltoall_local(comm, bufs, out, count=cnt)

        def check(what):
            if is_rs:
                assert_same_bits(out, want, what)
            else:
                assert np.array_equal(wl.to_numpy_bits(out), want), what

        res = fx.flex_comm_tune(comm, coll, bufs, out, count=cnt)
        say("tune", coll, res.as_dict())
        torch.cuda.synchronize()
        check("after tune")
        check_stage1_against_oracle(comm, coll, cnt, dtype, res, cfg)
        fx.flex_set_split(comm, coll, fx.FLEX_SPLIT_ADAPTIVE)
        twin = Stage2Twin(comm, coll, cnt, dtype, cfg)
        for k in range(20):
            out.zero_()
            call()
            twin.after_call()
        check("adaptive, tuned shares")
        # and with the host path kept live
        fx.flex_comm_set_shares(comm, coll, cnt, dtype, [9850, 150])
        twin = Stage2Twin(comm, coll, cnt, dtype, cfg)
        for k in range(30):
            out.zero_()
            share = twin.twin.S[1]
            call()
            st = twin.after_call()
            assert st.last_split == op.partition(cnt, share, 10000, 2048, 32768)
        check("adaptive, host path live")
        assert st.samples >= 30 and st.last_time_s[1] > 0


def test_tune_acceptance_check_needs_a_gain_beyond_the_noise():
    count = 64 * wl.MIB        # 128 MiB per rank
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    cfg = fx.flex_config_default()
    with Comm(max_bytes=count * 2) as comm:
        out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
        res = fx.flex_comm_tune(comm, fx.FLEX_ALLREDUCE, bufs, out)
        say("tune", res.as_dict())
        check_stage1_against_oracle(comm, fx.FLEX_ALLREDUCE, count, torch.bfloat16, res, cfg)
        if res.balanced_shares[1] > 0:
            # Algorithm 1 left the host path active: the check ran, interleaved
            assert res.accept_samples == cfg.accept_pairs * cfg.tune_reps
            assert res.combined_s > 0 and res.device_alone_s > 0
            gain = res.device_alone_s - res.combined_s
            noise = 3 * max(res.combined_mad_s, res.device_alone_mad_s)
            if res.reverted:
                assert not gain > noise
                assert list(res.shares)[:2] == [10000, 0] and res.active_mask == 1
            else:
                assert gain > noise and res.active_mask == 3 and res.shares[1] == res.balanced_shares[1]
        else:
            assert res.accept_samples == 0 and not res.reverted
        torch.cuda.synchronize()
        assert_same_bits(out, oracle_allreduce(bufs), "after tune")
    # switched off, the balanced split is kept whatever it costs
    with Comm(max_bytes=count * 2, tune_accept_check=0) as comm:
        res = fx.flex_comm_tune(comm, fx.FLEX_ALLREDUCE, bufs, out)
        assert not res.reverted and res.accept_samples == 0 and list(res.shares) == list(res.balanced_shares)
        torch.cuda.synchronize()
        assert_same_bits(out, oracle_allreduce(bufs), "after tune without the check")


# ------------------------------------------------------------ error handling

def test_invalid_arguments_are_rejected_without_enqueueing():
    bufs = wl.make_rank_buffers(wl.config(0), DEV, count=4096)
    out = torch.zeros(4096, dtype=torch.float32, device=DEV)
    L = fx.lib()
    with pytest.raises(fx.FlexError) as e:
        fx.flex_comm_create(9, 0, 1 << 20)
    assert e.value.status == fx.FLEX_ERR_INVALID_ARG
    with pytest.raises(fx.FlexError):
        fx.flex_comm_create(8, 8, 1 << 20)
    with Comm(max_bytes=4096 * 4) as comm:
        ptrs = fx._pointer_array(bufs)
        s = fx._stream_handle(None)
        assert L.flex_allreduce_local(comm, ptrs, out.data_ptr(), 4097, fx.FLEX_F32, fx.FLEX_SUM, s) == fx.FLEX_ERR_INVALID_ARG
        assert "max_bytes" in fx.flex_last_error()
        assert L.flex_allreduce_local(comm, ptrs, out.data_ptr(), 4096, 7, fx.FLEX_SUM, s) == fx.FLEX_ERR_UNSUPPORTED
        assert L.flex_allreduce_local(comm, ptrs, out.data_ptr(), 4096, fx.FLEX_F32, 3, s) == fx.FLEX_ERR_UNSUPPORTED
        assert L.flex_allreduce_local(comm, ptrs, None, 4096, fx.FLEX_F32, fx.FLEX_SUM, s) == fx.FLEX_ERR_INVALID_ARG
        assert L.flex_allreduce_local(comm, None, out.data_ptr(), 4096, fx.FLEX_F32, fx.FLEX_SUM, s) == fx.FLEX_ERR_INVALID_ARG
        assert L.flex_allreduce_local(None, ptrs, out.data_ptr(), 4096, fx.FLEX_F32, fx.FLEX_SUM, s) == fx.FLEX_ERR_INVALID_ARG
        bad = fx._pointer_array(bufs)
        bad[5] = None
        assert L.flex_allgather_local(comm, bad, out.data_ptr(), 512, fx.FLEX_F32, s) == fx.FLEX_ERR_INVALID_ARG
        odd = fx._pointer_array(bufs)
        odd[1] = bufs[1].data_ptr() + 2
        assert L.flex_allreduce_local(comm, odd, out.data_ptr(), 16, fx.FLEX_F32, fx.FLEX_SUM, s) == fx.FLEX_ERR_INVALID_ARG
        with pytest.raises(fx.FlexError):
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, 2501)
        with pytest.raises(fx.FlexError):
            fx.flex_set_split(comm, 4, fx.FLEX_SPLIT_STATIC, 0)
        torch.cuda.synchronize()
        assert out.abs().sum() == 0          # nothing ran
        # count 0 is fine and does nothing
        assert L.flex_allreduce_local(comm, ptrs, None, 0, fx.FLEX_F32, fx.FLEX_SUM, s) == fx.FLEX_OK
        # and the communicator still works after all the rejected calls
        fx.flex_allreduce_local(comm, bufs, out)
        torch.cuda.synchronize()
        assert_same_bits(out, oracle_allreduce(bufs), "after errors")


# ------------------------------------------------- the C ABI from plain C

def test_plain_c_program_through_the_c_abi():
    # no Python between the caller and the library: a C99 program linked against
    # libflexlink.so, the HIP runtime and the C oracle (built beforehand by
    # tests/c_abi/build.py), run as one child process
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "c_abi_check")
    if not os.path.exists(exe):
        pytest.skip("tests/c_abi/c_abi_check is not built (python -m tests.c_abi.build, or the build entry point)")
    torch.cuda.synchronize()
    run = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    say(run.stdout, run.stderr)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.count("ok  ") == 10 and "C ABI check passed" in run.stdout

