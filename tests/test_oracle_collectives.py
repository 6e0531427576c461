"""Pins for the CPU oracle of the collectives: each test checks the oracle
against something other than itself (a library routine on a special case, exact
rational arithmetic, a hand-derived value, an invariant)."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import collectives as oc
from paper_2510_15882_amd import workloads as wl


def bf16_bits(values):
    """bfloat16 bit patterns of values that are exactly representable."""
    t = torch.tensor(values, dtype=torch.float32)
    b = t.to(torch.bfloat16)
    assert torch.equal(b.float(), t), "test value not representable in bf16"
    return wl.to_numpy_bits(b)


# ---------------------------------------------------------------- AllGather

@pytest.mark.parametrize("n", [1, 2, 3, 8])
@pytest.mark.parametrize("count", [0, 1, 7, 4099])
@pytest.mark.parametrize("dtype", [np.uint16, np.float32])
def test_allgather_is_concatenation(n, count, dtype):
    rng = np.random.default_rng(100 * n + count)
    if dtype == np.float32:
        slices = [rng.integers(0, 1 << 32, count, dtype=np.uint64).astype(np.uint32).view(np.float32)
                  for _ in range(n)]
    else:
        slices = [rng.integers(0, 1 << 16, count, dtype=np.uint32).astype(np.uint16) for _ in range(n)]
    got = oc.allgather(slices)
    want = np.concatenate(slices)
    # compare raw bits: NaN payloads, -0.0 and denormals must survive
    assert got.tobytes() == want.tobytes()


# ------------------------------------------------- AllReduce, special cases

def test_allreduce_one_rank_is_identity():
    x32 = wl.random_bits(10007, torch.float32, 1, finite_only=True).numpy()
    assert oc.allreduce([x32]).tobytes() == x32.tobytes()
    x16 = wl.to_numpy_bits(wl.random_bits(10007, torch.bfloat16, 2, finite_only=True))
    assert oc.allreduce([x16]).tobytes() == x16.tobytes()


def test_allreduce_two_ranks_f32_is_ieee_add():
    a = wl.random_bits(50021, torch.float32, 3, finite_only=True).numpy()
    b = wl.random_bits(50021, torch.float32, 4, finite_only=True).numpy()
    # bring exponents close enough that sums are not dominated by one operand
    b = (b * np.float32(0) + a * np.float32(0.37)).astype(np.float32)
    b = np.where(np.isfinite(b), b, np.float32(1.5)).astype(np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        want = a + b
    got = oc.allreduce([a, b])
    ok = np.isfinite(want) | np.isinf(want)
    assert np.array_equal(got.view(np.uint32)[ok], want.view(np.uint32)[ok])
    assert np.all(np.isnan(got[~ok]))


def test_allreduce_f32_denormals_are_kept():
    tiny = np.float32(1e-40)           # subnormal in binary32
    a = np.full(5, tiny, dtype=np.float32)
    got = oc.allreduce([a, a, a])
    want = (a + a) + a
    assert want[0] != 0 and got.tobytes() == want.tobytes()
    # subnormal bf16 in, subnormal bf16 out
    h = np.full(4, 0x0001, dtype=np.uint16)     # smallest positive bf16 subnormal
    assert oc.allreduce([h, h]).tolist() == [0x0002] * 4


@pytest.mark.parametrize("n", [2, 5, 8])
def test_allreduce_small_integers_sum_exactly(n):
    rng = np.random.default_rng(7 + n)
    ints = rng.integers(-16, 17, size=(n, 3001))
    want = ints.sum(axis=0)                     # |sum| <= 128: exact in bf16
    bufs16 = [bf16_bits(ints[r].astype(np.float32).tolist()) for r in range(n)]
    got16 = torch.from_numpy(oc.allreduce(bufs16).view(np.int16)).view(torch.bfloat16).float().numpy()
    assert np.array_equal(got16, want.astype(np.float32))
    big = rng.integers(-(1 << 20), 1 << 20, size=(n, 3001))
    bufs32 = [big[r].astype(np.float32) for r in range(n)]
    assert np.array_equal(oc.allreduce(bufs32).astype(np.int64), big.sum(axis=0))


def test_allreduce_order_is_rank_0_first_left_to_right():
    # ((2^24 + 1) + -2^24) + 0... : 2^24 + 1 rounds back to 2^24, so the
    # left-to-right sum is 0; adding the 1 last, or pairing the two large
    # terms first, would give 1.
    vals = [2.0 ** 24, 1.0, -(2.0 ** 24), 0.0, 0.0, 0.0, 0.0, 0.0]
    bufs = [np.full(3, v, dtype=np.float32) for v in vals]
    assert oc.allreduce(bufs).tolist() == [0.0, 0.0, 0.0]
    # and the other way round: (1 + 2^24) + -2^24 is also 0, but
    # (2^24 + -2^24) + 1 is 1 - rank order decides.
    vals2 = [2.0 ** 24, -(2.0 ** 24), 1.0]
    assert oc.allreduce([np.full(2, v, dtype=np.float32) for v in vals2]).tolist() == [1.0, 1.0]


def test_allreduce_bf16_accumulates_in_f32_and_rounds_once():
    # 1 + 3 * 2^-9 = 1.005859375.  The bf16 neighbours of that are 1 and
    # 1 + 2^-7 (= 1.0078125); it lies above the midpoint 1 + 2^-8, so a single
    # final rounding gives 0x3F81.  Rounding to bf16 after every add would
    # drop each 2^-9 in turn and give 1.0 (0x3F80).
    vals = [1.0, 2.0 ** -9, 2.0 ** -9, 2.0 ** -9, 0.0, 0.0, 0.0, 0.0]
    bufs = [bf16_bits([v] * 4) for v in vals]
    assert oc.allreduce(bufs).tolist() == [0x3F81] * 4


def test_allreduce_starts_from_rank0_not_from_zero():
    # (-0) + (-0) = -0, whereas (+0) + (-0) = +0 under round-to-nearest.
    neg0_32 = np.full(3, -0.0, dtype=np.float32)
    out = oc.allreduce([neg0_32] * 8)
    assert out.view(np.uint32).tolist() == [0x80000000] * 3
    neg0_16 = np.full(3, 0x8000, dtype=np.uint16)
    assert oc.allreduce([neg0_16] * 8).tolist() == [0x8000] * 3


# ------------------------------------------------------ bf16 conversions

def test_bf16_widening_is_exact_for_all_patterns():
    allbits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    want = torch.from_numpy(allbits.view(np.int16)).view(torch.bfloat16).float().numpy()
    got = np.array([oc.bf16_to_f32(int(h)) for h in allbits[::17]], dtype=np.float32)
    w = want[::17]
    fin = ~np.isnan(w)
    assert np.array_equal(got[fin].view(np.uint32), w[fin].view(np.uint32))
    assert np.all(np.isnan(got[~fin]))


def test_bf16_rounding_matches_library_rne_on_all_high_halves():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000], dtype=np.uint32)
    bits = (hi[:, None] | lows[None, :]).reshape(-1).astype(np.uint32)
    got = oc.f32_bits_to_bf16(bits)
    f = torch.from_numpy(bits.view(np.int32)).view(torch.float32)
    want = wl.to_numpy_bits(f.to(torch.bfloat16))
    nan = np.isnan(f.numpy())
    assert np.array_equal(got[~nan], want[~nan])
    # NaN in, NaN out (sign kept); payload is not pinned
    g = got[nan]
    assert np.all((g & 0x7F80) == 0x7F80) and np.all((g & 0x007F) != 0)
    assert np.array_equal(g >> 15, (bits[nan] >> 31).astype(np.uint16))


def test_bf16_rounding_hand_values():
    # ties to even: 1 + 2^-8 is halfway between 1 (even mantissa) and 1 + 2^-7
    assert oc.f32_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    # 1 + 3 * 2^-8 is halfway between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    assert oc.f32_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # largest binary32 rounds up to +inf in bf16
    assert oc.f32_to_bf16(float(np.finfo(np.float32).max)) == 0x7F80
    assert oc.f32_to_bf16(-1.0) == 0xBF80


# ---------------------------------------- independent second formulations

def torch_formulation(bufs):
    acc = bufs[0].float()
    for b in bufs[1:]:
        acc = acc + b.float()
    return acc.to(bufs[0].dtype)


@pytest.mark.parametrize("cfg", [0, 1, 2, 4])
def test_allreduce_equals_torch_cpu_left_fold(cfg):
    w = wl.config(cfg)
    bufs = wl.make_rank_buffers(w, count=70001)
    want = wl.to_numpy_bits(torch_formulation(bufs))
    got = oc.allreduce([wl.to_numpy_bits(b) for b in bufs])
    assert got.tobytes() == want.tobytes()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_allreduce_equals_torch_cpu_on_random_bit_patterns(dtype):
    bufs = [wl.random_bits(40009, dtype, 50 + r, finite_only=True) for r in range(8)]
    want_t = torch_formulation(bufs)
    want = wl.to_numpy_bits(want_t)
    got = oc.allreduce([wl.to_numpy_bits(b) for b in bufs])
    nan = torch.isnan(want_t.float()).numpy()
    assert np.array_equal(got[~nan], want[~nan])
    if dtype == torch.float32:
        assert np.all(np.isnan(got[nan]))
    else:
        assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x7F) != 0)


def round_to_nearest_even(x: Fraction, mant_bits: int, emin: int, emax: int):
    """Round an exact rational to a binary float with `mant_bits` stored
    mantissa bits, minimum normal exponent emin, maximum exponent emax.
    Returns a Fraction, or +-inf as float.  Brute-force definition."""
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, emin)
    quantum = Fraction(2) ** (e - mant_bits)
    q = a / quantum
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    r = n * quantum
    if r >= Fraction(2) ** (emax + 1):
        return sign * float("inf")
    return sign * r


def exact_reference(columns, to_bf16):
    out = []
    for col in columns:
        acc = Fraction(float(col[0]))
        for v in col[1:]:
            if isinstance(acc, float):      # already +-inf
                break
            acc = round_to_nearest_even(acc + Fraction(float(v)), 23, -126, 127)
        if to_bf16 and not isinstance(acc, float):
            acc = round_to_nearest_even(acc, 7, -126, 127)
        out.append(float(acc))
    return out


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_allreduce_equals_exact_rational_brute_force(dtype):
    n, count = 8, 300
    cols = []
    bufs = [wl.random_bits(count, dtype, 900 + r, finite_only=True) for r in range(n)]
    # squeeze exponents into a band so that roundings actually interact, and
    # keep some extreme columns (denormals, near-overflow) as they are
    for r in range(n):
        f = bufs[r].float()
        mid = torch.ldexp(torch.frexp(f)[0], torch.randint(-3, 4, (count,), generator=torch.Generator().manual_seed(r)))
        f[: count - 60] = mid[: count - 60]
        bufs[r] = f.to(dtype)
    finite = torch.stack([torch.isfinite(b.float()) for b in bufs]).all(0)
    for i in range(count):
        cols.append([bufs[r][i].float().item() for r in range(n)])
    want = exact_reference(cols, dtype == torch.bfloat16)
    got_bits = oc.allreduce([wl.to_numpy_bits(b) for b in bufs])
    if dtype == torch.float32:
        got = got_bits.astype(np.float64)
    else:
        got = torch.from_numpy(got_bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    checked = 0
    for i in range(count):
        if not finite[i] or np.isnan(want[i]) or np.isnan(got[i]):
            continue
        # inf - inf style cases excluded above; everything else must match exactly
        assert got[i] == want[i], (i, cols[i], got[i], want[i])
        assert np.signbit(got[i]) == np.signbit(want[i]) or want[i] != 0
        checked += 1
    assert checked > count * 0.9


def test_allreduce_error_bound_against_float64_sum():
    w = wl.config(0)
    bufs = wl.make_rank_buffers(w, count=100003)
    got = oc.allreduce([wl.to_numpy_bits(b) for b in bufs]).astype(np.float64)
    stack = np.stack([b.double().numpy() for b in bufs])
    exact = stack.sum(axis=0)
    # (N-1) roundings, each at most half an ulp of a partial sum bounded by sum|b|
    bound = (len(bufs) - 1) * 2.0 ** -24 * np.abs(stack).sum(axis=0)
    assert np.all(np.abs(got - exact) <= bound)
    assert np.any(got != exact.astype(np.float32))   # the bound is not vacuous: roundings happen


def test_allreduce_depends_on_rank_order():
    w = wl.config(0)
    bufs = [wl.to_numpy_bits(b) for b in wl.make_rank_buffers(w, count=100003)]
    fwd = oc.allreduce(bufs)
    rev = oc.allreduce(bufs[::-1])
    assert np.any(fwd != rev)           # rounding makes fp32 addition order-sensitive
    assert np.allclose(fwd, rev, atol=1e-5)


def test_every_rank_contributes_once():
    # one-hot contributions: rank r holds 2^r at every index; the sum's bits
    # name exactly which ranks were added, and how many times
    n = 8
    bufs = [np.full(11, float(1 << r), dtype=np.float32) for r in range(n)]
    assert oc.allreduce(bufs).tolist() == [255.0] * 11
    bufs16 = [bf16_bits([float(1 << r)] * 11) for r in range(n)]
    assert oc.allreduce(bufs16).tolist() == bf16_bits([255.0] * 11).tolist()
    # per-index data: element i of rank r is r * 1000 + i (exact in fp32)
    bufs = [np.arange(500, dtype=np.float32) + 1000 * r for r in range(n)]
    want = np.arange(500, dtype=np.int64) * n + 1000 * sum(range(n))
    assert np.array_equal(oc.allreduce(bufs).astype(np.int64), want)


# ------------------------------------------------------------- binary16

def test_f16_widening_is_exact_for_all_patterns():
    allbits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    want = allbits.view(np.float16).astype(np.float32)
    got = np.array([oc.f16_to_f32(int(h)) for h in allbits[::7]], dtype=np.float32)
    w = want[::7]
    fin = ~np.isnan(w)
    assert np.array_equal(got[fin].view(np.uint32), w[fin].view(np.uint32))
    assert np.all(np.isnan(got[~fin]))


def test_f16_rounding_matches_library_rne():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x0FFF, 0x1000, 0x1001, 0x1FFF, 0x2000, 0x3000, 0x7FFF, 0x8000, 0xFFFF],
                    dtype=np.uint32)
    bits = (hi[:, None] | lows[None, :]).reshape(-1).astype(np.uint32)
    # dense sweeps where the format changes character: subnormal range, the
    # smallest normal, and the overflow threshold 65520
    dense = [np.arange(np.float32(a).view(np.uint32), np.float32(b).view(np.uint32), step, dtype=np.uint64)
             for a, b, step in ((2.0 ** -27, 2.0 ** -13, 97), (65400.0, 65600.0, 1), (2.0 ** -15, 2.0 ** -14 * 1.01, 3))]
    bits = np.concatenate([bits] + [d.astype(np.uint32) for d in dense] +
                          [d.astype(np.uint32) | np.uint32(0x80000000) for d in dense])
    got = oc.f32_bits_to_f16(bits)
    f = bits.view(np.float32)
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    nan = np.isnan(f)
    assert np.array_equal(got[~nan], want[~nan])
    g = got[nan]
    assert np.all((g & 0x7C00) == 0x7C00) and np.all((g & 0x03FF) != 0)


def test_f16_rounding_hand_values():
    r = lambda x: int(oc.f32_bits_to_f16(np.array([x], dtype=np.float32).view(np.uint32))[0])
    assert r(1.0) == 0x3C00 and r(-2.0) == 0xC000
    assert r(65504.0) == 0x7BFF                   # largest finite
    assert r(65519.99) == 0x7BFF and r(65520.0) == 0x7C00      # halfway to 2^16 ties to "even" = infinity
    assert r(2.0 ** -24) == 0x0001                # smallest subnormal
    assert r(2.0 ** -25) == 0x0000                # tie with zero -> even
    assert r(2.0 ** -25 * 1.0000001) == 0x0001
    assert r(2.0 ** -14) == 0x0400                # smallest normal
    assert r(1.0 + 2.0 ** -11) == 0x3C00 and r(1.0 + 3 * 2.0 ** -11) == 0x3C02   # ties to even


def test_allreduce_f16_equals_torch_cpu_and_exact_rational():
    n, count = 8, 40009
    bufs = [wl.random_bits(count, torch.float16, 300 + r, finite_only=True) for r in range(n)]
    for r in range(n):   # bring most exponents within reach of each other
        f = bufs[r].float()
        mid = torch.ldexp(torch.frexp(f)[0], torch.randint(-2, 3, (count,), generator=torch.Generator().manual_seed(r)))
        f[: count - 2000] = mid[: count - 2000]
        bufs[r] = f.to(torch.float16)
    want_t = torch_formulation(bufs)
    got = oc.allreduce([wl.to_numpy_bits(b) for b in bufs])
    nan = torch.isnan(want_t).numpy()
    assert np.array_equal(got.view(np.uint16)[~nan], want_t.numpy().view(np.uint16)[~nan])
    assert np.all(np.isnan(got[nan]))
    # brute force on a sample, last 2000 columns (raw exponents) included
    idx = list(range(0, 200)) + list(range(count - 100, count))
    cols = [[bufs[r][i].float().item() for r in range(n)] for i in idx]
    ref = []
    for col in cols:
        acc = Fraction(float(col[0]))
        for v in col[1:]:
            if isinstance(acc, float):
                break
            acc = round_to_nearest_even(acc + Fraction(float(v)), 23, -126, 127)
        if not isinstance(acc, float):
            acc = round_to_nearest_even(acc, 10, -14, 15)
        ref.append(float(acc))
    for k, i in enumerate(idx):
        g = float(got[i])
        if np.isnan(g) or np.isnan(ref[k]):
            continue
        assert g == ref[k], (i, cols[k], g, ref[k])


def test_reducescatter_is_the_rank_slice_of_allreduce():
    n, rc = 8, 5003
    bufs = [wl.to_numpy_bits(b) for b in wl.make_rank_buffers(wl.config(2), count=n * rc)]
    full = oc.allreduce(bufs)
    for rank in (0, 3, 7):
        assert oc.reducescatter(bufs, rank).tobytes() == full[rank * rc:(rank + 1) * rc].tobytes()
    ints = [np.arange(n * 4, dtype=np.float32) + 100 * r for r in range(n)]
    assert oc.reducescatter(ints, 2).tolist() == [float(8 * (8 + j) + 100 * 28) for j in range(4)]


def test_alltoall_is_a_transpose_of_pieces():
    n, cnt = 8, 1237
    rng = np.random.default_rng(3)
    bufs = [rng.integers(0, 1 << 16, n * cnt, dtype=np.uint32).astype(np.uint16) for _ in range(n)]
    cube = np.stack(bufs).reshape(n, n, cnt)                 # [sender, destination, element]
    for rank in (0, 5, 7):
        want = cube[:, rank, :].reshape(-1)                  # library slicing: what everybody sends to `rank`
        assert oc.alltoall(bufs, rank).tobytes() == want.tobytes()
    # doing it for every rank and stacking is the transpose of the first two axes
    allrecv = np.stack([oc.alltoall(bufs, r) for r in range(n)]).reshape(n, n, cnt)
    assert np.array_equal(allrecv, cube.transpose(1, 0, 2))
