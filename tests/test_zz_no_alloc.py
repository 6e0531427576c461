"""flex_allreduce_staged_noalloc (the entry point for callers that cannot
allocate) against flex_allreduce_local and the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import collectives as oc
from paper_2510_15882_amd import binding as fx
from paper_2510_15882_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits(t):
    return wl.to_numpy_bits(t).view(np.uint32 if t.dtype == torch.float32 else np.uint16)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_noalloc_allreduce_matches_the_existing_entry_point_twice_in_a_row(dtype):
    assert torch.cuda.is_available(), "needs the MI355X"
    torch.cuda.set_device(0)
    es = 2 if dtype == torch.bfloat16 else 4
    n, rank = 8, 3
    big = (24 << 20) // es + 2048 + 5          # 24 MiB per rank and a ragged end
    small = (3 << 20) // es + 77               # second call: a smaller input
    w = wl.config(2) if dtype == torch.bfloat16 else wl.config(0)
    bufs = wl.make_rank_buffers(w, DEV, count=big)
    cfg = fx.flex_config_default()
    cfg.host_engine = fx.FLEX_ENGINE_SDMA      # the existing entry point whose kernels read a library-owned scratch
    comm = fx.flex_comm_create(n, rank, big * es, cfg)
    stream = torch.cuda.Stream()
    try:
        for count, units in ((big, 1200), (small, 2200), (big, 0), (small, 1)):
            ins = [b[:count] for b in bufs]
            want = torch.zeros(count, dtype=dtype, device=DEV)
            fx.flex_set_split(comm, fx.FLEX_ALLREDUCE, fx.FLEX_SPLIT_STATIC, units)
            fx.flex_allreduce_local(comm, ins, want)
            got = torch.full((count + 16,), 5.0, dtype=dtype, device=DEV)
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                fx.flex_allreduce_staged_noalloc(ins, rank, got[:count], count=count, staged_units=units, stream=stream)
            torch.cuda.synchronize()
            assert np.array_equal(bits(got[:count]), bits(want)), (count, units)
            assert np.array_equal(bits(want), oc.allreduce([wl.to_numpy_bits(b) for b in ins]).view(bits(want).dtype))
            assert torch.all(got[count:] == 5.0), "wrote past the end"
        # a staged part beyond the built-in transit buffer is refused and nothing runs
        got = torch.zeros(big, dtype=dtype, device=DEV)
        with pytest.raises(fx.FlexError) as e:
            fx.flex_allreduce_staged_noalloc(bufs, rank, got, staged_units=5000)
        assert e.value.status == fx.FLEX_ERR_INVALID_ARG and "transit buffer" in str(e.value)
        torch.cuda.synchronize()
        assert got.abs().sum() == 0
    finally:
        torch.cuda.synchronize()
        fx.flex_comm_destroy(comm)


def test_noalloc_allreduce_in_a_captured_graph():
    # nothing is allocated and everything sits on the caller's stream, so a call
    # with a staged part can be captured; replays with eager work in between
    assert torch.cuda.is_available(), "needs the MI355X"
    torch.cuda.set_device(0)
    count = (1 << 20) + 2048 + 3
    bufs = wl.make_rank_buffers(wl.config(2), DEV, count=count)
    want = oc.allreduce([wl.to_numpy_bits(b) for b in bufs])
    out = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
    fx.flex_allreduce_staged_noalloc(bufs, 0, out, staged_units=2500)      # first call outside the capture
    torch.cuda.synchronize()
    assert np.array_equal(wl.to_numpy_bits(out), want)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        fx.flex_allreduce_staged_noalloc(bufs, 0, out, staged_units=2500, stream=stream)
    torch.cuda.synchronize()
    for replay in range(3):
        out.fill_(1.0)                                                     # a fill kernel, no memset node
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(wl.to_numpy_bits(out), want), replay
        other = torch.zeros(count, dtype=torch.bfloat16, device=DEV)
        fx.flex_allreduce_staged_noalloc(bufs, 5, other, staged_units=700)  # eager call between replays
        torch.cuda.synchronize()
        assert np.array_equal(wl.to_numpy_bits(other), want)
    del graph
