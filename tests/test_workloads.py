"""The seeded input generators: reproducible, rank-distinct, of the stated shape."""
import numpy as np
import torch

from paper_2510_15882_amd import workloads as wl


def test_configs_have_the_stated_shapes():
    assert wl.config(0).count == 262144 and wl.config(0).dtype == torch.float32 and wl.config(0).bytes_per_rank == 1 << 20
    assert wl.config(1).bytes_per_rank == 32 << 20 and wl.config(1).collective == "allgather"
    assert wl.config(2).bytes_per_rank == 256 << 20 and wl.config(2).scale == 0.02
    assert wl.config(4).count == 65536 * 5120 and wl.config(4).bytes_per_rank == 640 << 20
    sweep = wl.sweep_workloads()
    assert len(sweep) == 12 and {w.bytes_per_rank >> 20 for w in sweep} == {1, 4, 16, 64, 256, 1024}
    for name, dt in (("f32", torch.float32), ("f16", torch.float16)):
        other = wl.sweep_workloads(name)
        assert [w.bytes_per_rank for w in other] == [w.bytes_per_rank for w in sweep]
        assert all(w.dtype == dt and name in w.name for w in other)


def test_evaluation_grid_has_the_sizes_of_the_paper_s_table():
    grid = wl.evaluation_grid_workloads()
    assert len(grid) == 24 and {w.nranks for w in grid} == {2, 4, 8}
    for w in grid:
        message = w.bytes_per_rank * (w.nranks if w.collective == "allgather" else 1)
        assert message >> 20 in (32, 64, 128, 256) and message % (1 << 20) == 0
        assert len(wl.make_rank_buffers(w, count=16)) == w.nranks


def test_generation_is_reproducible_and_rank_distinct():
    a = wl.make_rank_buffers(wl.config(2), count=4096)
    b = wl.make_rank_buffers(wl.config(2), count=4096)
    assert len(a) == 8
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))
    assert not torch.equal(a[0], a[1])
    u = wl.make_rank_buffers(wl.config(0), count=100000)[3]
    assert u.min() >= -1 and u.max() < 1 and abs(u.mean()) < 0.02
    n = wl.make_rank_buffers(wl.config(2), count=100000)[5].float()
    assert abs(n.std() - 0.02) < 0.001


def test_random_bits_cover_specials_and_finite_only_removes_them():
    for dt in (torch.float32, torch.bfloat16, torch.float16):
        x = wl.random_bits(200000, dt, 9)
        assert torch.isnan(x.float()).any()
        y = wl.random_bits(200000, dt, 9, finite_only=True)
        assert torch.isfinite(y.float()).all()
        bits = wl.to_numpy_bits(y)
        assert bits.nbytes == y.numel() * y.element_size()
