"""Seeded synthetic inputs for the local-share collectives.

This module holds input generation only: none of the method's arithmetic lives
here, so both the HIP path and the CPU oracle may be fed from it.

The paper measured nccl-tests-style buffers (Evaluation, "Baselines and
Metrics") with message sizes of 32-256 MB on N = 2, 4, 8 GPUs (Table 2) and
motivates the work with the tensor-parallel AllReduce of a 32B-class model's
64K-token prefill (Introduction).  The configurations below carry those shapes
over; the value distributions are this build's choice and stand in for the
paper's unspecified buffer contents.

Rank r of configuration k draws from a generator seeded
BASE_SEED + 1000 * k + r, so every rank's contribution differs and any
configuration can be regenerated rank by rank.
"""
from dataclasses import dataclass

import torch

BASE_SEED = 20251015
MIB = 1 << 20


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    collective: str      # "allreduce" | "allgather"
    dtype: torch.dtype
    count: int           # elements contributed by each rank
    dist: str            # "uniform_pm1" | "normal"
    scale: float
    nranks: int = 8

    @property
    def bytes_per_rank(self) -> int:
        return self.count * torch.empty((), dtype=self.dtype).element_size()


CONFIGS = (
    Workload(0, "allreduce_f32_1MiB", "allreduce", torch.float32, 262144, "uniform_pm1", 1.0),
    Workload(1, "allgather_bf16_32MiB", "allgather", torch.bfloat16, 16 * MIB, "normal", 1.0),
    Workload(2, "allreduce_bf16_256MiB", "allreduce", torch.bfloat16, 128 * MIB, "normal", 0.02),
    # 3: message-size sweep, see sweep_workloads()
    Workload(4, "allreduce_bf16_prefill_65536x5120", "allreduce", torch.bfloat16,
             65536 * 5120, "normal", 1.0),
)

SWEEP_MIB_PER_RANK = (1, 4, 16, 64, 256, 1024)


DTYPE_NAMES = {"bf16": torch.bfloat16, "f32": torch.float32, "f16": torch.float16}


def sweep_workloads(dtype_name="bf16"):
    """Configuration 3: AllReduce and AllGather, N(0,1), 1..1024 MiB per rank;
    bf16 as configured, or the same byte sizes in f32 / f16."""
    dtype = DTYPE_NAMES[dtype_name]
    esize = torch.empty((), dtype=dtype).element_size()
    out = []
    for coll in ("allreduce", "allgather"):
        for mib in SWEEP_MIB_PER_RANK:
            out.append(Workload(3, "%s_%s_%dMiB" % (coll, dtype_name, mib), coll, dtype,
                                mib * MIB // esize, "normal", 1.0))
    return out


GRID_RANKS = (2, 4, 8)
GRID_MIB = (32, 64, 128, 256)


def evaluation_grid_workloads():
    """The grid of the paper's end-to-end table (Evaluation, Table 2): AllReduce
    and AllGather on 2, 4 and 8 ranks with messages of 32..256 MiB, bf16 N(0,1).
    The message size is the collective's buffer size as nccl-tests counts it:
    every rank's whole buffer for AllReduce, the gathered output for AllGather
    (each rank contributes 1/N of it), as in configuration 1."""
    out = []
    for coll in ("allreduce", "allgather"):
        for nranks in GRID_RANKS:
            for mib in GRID_MIB:
                count = mib * MIB // 2 // (nranks if coll == "allgather" else 1)
                out.append(Workload(5, "%s_bf16_%dranks_%dMiB" % (coll, nranks, mib), coll, torch.bfloat16,
                                    count, "normal", 1.0, nranks))
    return out


def config(index: int) -> Workload:
    for w in CONFIGS:
        if w.index == index:
            return w
    raise KeyError(index)


def rank_seed(config_index: int, rank: int) -> int:
    return BASE_SEED + 1000 * config_index + rank


def fill_rank(out: torch.Tensor, dist: str, scale: float, seed: int) -> torch.Tensor:
    """Fill `out` in place from a generator on out's device seeded with `seed`."""
    g = torch.Generator(device=out.device)
    g.manual_seed(seed)
    if dist == "uniform_pm1":
        out.uniform_(-1.0, 1.0, generator=g)
    elif dist == "normal":
        out.normal_(0.0, 1.0, generator=g)
    else:
        raise ValueError(dist)
    if scale != 1.0:
        out.mul_(scale)
    return out


def make_rank_buffers(w: Workload, device="cpu", count=None, nranks=None):
    """One tensor per simulated rank, shape (count,), w.dtype, on `device`.

    `count` overrides the element count (tests use shortened messages of the
    same distribution); `nranks` overrides the number of simulated ranks.
    """
    count = w.count if count is None else count
    nranks = w.nranks if nranks is None else nranks
    bufs = []
    for r in range(nranks):
        t = torch.empty(count, dtype=w.dtype, device=device)
        fill_rank(t, w.dist, w.scale, rank_seed(w.index, r))
        bufs.append(t)
    return bufs


def random_bits(count: int, dtype: torch.dtype, seed: int, device="cpu", finite_only=False):
    """A tensor whose elements are uniformly random bit patterns (denormals,
    infinities and, unless finite_only, NaNs included)."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    if dtype == torch.float32:
        bits = torch.randint(-(1 << 31), 1 << 31, (count,), dtype=torch.int64,
                             generator=g, device=device).to(torch.int32)
        if finite_only:
            exp_all_ones = (bits & 0x7F800000) == 0x7F800000
            bits = torch.where(exp_all_ones, bits & ~0x40000000, bits)
        return bits.view(torch.float32)
    if dtype == torch.bfloat16:
        bits = torch.randint(-(1 << 15), 1 << 15, (count,), dtype=torch.int64,
                             generator=g, device=device).to(torch.int16)
        if finite_only:
            exp_all_ones = (bits & 0x7F80) == 0x7F80
            bits = torch.where(exp_all_ones, bits & ~0x4000, bits)
        return bits.view(torch.bfloat16)
    if dtype == torch.float16:
        bits = torch.randint(-(1 << 15), 1 << 15, (count,), dtype=torch.int64,
                             generator=g, device=device).to(torch.int16)
        if finite_only:
            exp_all_ones = (bits & 0x7C00) == 0x7C00
            bits = torch.where(exp_all_ones, bits & ~0x4000, bits)
        return bits.view(torch.float16)
    raise ValueError(dtype)


def to_numpy_bits(t: torch.Tensor):
    """Host numpy view for the oracle: float32 stays float32, bfloat16 becomes
    its raw 16-bit patterns (uint16)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    if t.dtype == torch.float16:
        return t.numpy()
    raise ValueError(t.dtype)
