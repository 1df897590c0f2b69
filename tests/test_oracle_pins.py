"""Pins for the CPU oracle: each check rests on something other than the oracle's own
formula (closed forms, exact integer arithmetic, a library routine, permutation identities,
brute force in Python integers/fractions, hand-worked bit patterns)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2504_09014_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")

COUNTS = [0, 1, 2, 3, 7, 8, 9, 15, 16, 17, 63, 64, 65, 1023, 1024, 1025]
RANKS = [1, 2, 3, 4, 8]


def _read_table(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


# ---------------------------------------------------------------- bf16 conversion

def test_bf16_golden_cases(orc):
    for f32_hex, bf_hex in _read_table("bf16_rne_cases.txt"):
        x = np.array([int(f32_hex, 16)], np.uint32).view(np.float32)
        got = int(orc.f32_to_bf16(x)[0])
        assert got == int(bf_hex, 16), (f32_hex, hex(got), bf_hex)


def test_bf16_roundtrip_exhaustive(orc):
    bits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    f = orc.bf16_to_f32(bits)
    assert np.array_equal(f.view(np.uint32), bits.astype(np.uint32) << 16)   # widening is a shift
    back = orc.f32_to_bf16(f)
    nan = np.isnan(f)
    assert np.array_equal(back[~nan], bits[~nan])
    assert np.all(np.isnan(orc.bf16_to_f32(back[nan])))


def test_bf16_matches_torch_library_rounding(orc):
    g = torch.Generator().manual_seed(5)
    x = torch.randn(1_000_000, generator=g) * torch.exp(torch.randn(1_000_000, generator=g) * 8)
    raw = torch.randint(0, 2 ** 31 - 1, (200_000,), generator=g, dtype=torch.int32).view(torch.float32)
    x = torch.cat([x, raw[torch.isfinite(raw)], -raw[torch.isfinite(raw)]])
    want = x.bfloat16().view(torch.uint16).numpy()
    got = orc.f32_to_bf16(x.numpy())
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- AllReduce fp32

@pytest.mark.parametrize("n", RANKS)
def test_allreduce_f32_closed_forms(orc, n):
    count = 1000
    i = np.arange(count)
    tri = n * (n + 1) // 2
    x = np.stack([np.full(count, r + 1, np.float32) for r in range(n)])
    assert np.array_equal(orc.allreduce_f32(x), np.full(count, tri, np.float32))
    x = np.stack([((i % 251) * (r + 1)).astype(np.float32) for r in range(n)])
    assert np.array_equal(orc.allreduce_f32(x), (tri * (i % 251)).astype(np.float32))
    x = np.stack([(i == r).astype(np.float32) for r in range(n)])
    assert np.array_equal(orc.allreduce_f32(x), (i < n).astype(np.float32))


@pytest.mark.parametrize("n", RANKS)
@pytest.mark.parametrize("count", COUNTS)
def test_allreduce_f32_bruteforce_integers(orc, n, count):
    x = synth.int_valued_f32(n, count, seed=count + 100 * n).numpy()
    want = [sum(int(x[r, i]) for r in range(n)) for i in range(count)]      # Python ints
    got = orc.allreduce_f32(x)
    assert got.shape == (count,)
    assert [int(v) for v in got] == want
    assert list(orc.allreduce_f32_as_i64(x)) == want


def test_allreduce_f32_is_column_sum_library(orc):
    x = synth.int_valued_f32(8, 262144, seed=0).numpy()                      # config-1 shape
    want = np.sum(x.astype(np.float64), axis=0)                              # library routine, exact here
    got = orc.allreduce_f32(x)
    assert np.array_equal(got.astype(np.float64), want)
    assert np.array_equal(orc.allreduce_f32_as_i64(x), want.astype(np.int64))
    assert np.abs(want).max() <= 8000


def test_allreduce_f32_linearity_and_rank_permutation(orc):
    a = synth.int_valued_f32(8, 4097, seed=1).numpy()
    b = synth.int_valued_f32(8, 4097, seed=2).numpy()
    assert np.array_equal(orc.allreduce_f32(a + b), orc.allreduce_f32(a) + orc.allreduce_f32(b))
    perm = np.array([3, 7, 0, 5, 1, 6, 2, 4])
    assert np.array_equal(orc.allreduce_f32(a[perm]), orc.allreduce_f32(a))


def test_allreduce_f32_rank_order_and_accumulator_width(orc):
    # 2^24 + 1 is not representable in fp32 (ties to even -> 2^24), so the canonical order
    # ((x0 + x1) + x2) loses the 1, any order that cancels first keeps it, and a wider
    # accumulator keeps it too.  Worked by hand from the binary32 format.
    big = float(2 ** 24)
    x = np.array([[big], [1.0], [-big]], np.float32)
    assert orc.allreduce_f32(x)[0] == 0.0
    assert orc.allreduce_f32(x[[0, 2, 1]])[0] == 1.0
    assert orc.allreduce_f32(x[[1, 0, 2]])[0] == 0.0        # (1 + 2^24) also rounds to 2^24


def test_allreduce_f32_rejects_non_integers_in_exact_check(orc):
    with pytest.raises(ValueError):
        orc.allreduce_f32_as_i64(np.array([[0.5], [1.0]], np.float32))


def test_allreduce_f32_ieee_specials(orc):
    nz = np.float32(-0.0)
    out = orc.allreduce_f32(np.array([[nz, np.inf, np.inf, np.nan, 0.0]] * 1 +
                                     [[nz, 1.0, -np.inf, 1.0, nz]], np.float32))
    assert np.signbit(out[0]) and out[0] == 0.0             # -0 + -0 = -0
    assert out[1] == np.inf and np.isnan(out[2]) and np.isnan(out[3])
    assert out[4] == 0.0 and not np.signbit(out[4])         # +0 + -0 = +0


# ---------------------------------------------------------------- AllReduce bf16

def _ulp_bf16(v):
    """spacing of bf16 numbers around |v| (8 significand bits), for finite v != 0."""
    v = np.abs(np.asarray(v, np.float64))
    e = np.floor(np.log2(np.maximum(v, 2.0 ** -126)))
    return 2.0 ** (e - 7)


@pytest.mark.parametrize("n", RANKS)
def test_allreduce_bf16_within_one_ulp_of_fp64(orc, n):
    x = synth.normal(n, 50_001, seed=3)
    bits = synth.bf16_bits(x)
    out, ref = orc.allreduce_bf16(bits, want_ref64=True)
    want64 = np.sum(x.double().numpy(), axis=0)             # library column sum in fp64
    assert np.allclose(ref, want64, rtol=0, atol=1e-12)
    got = orc.bf16_to_f32(out).astype(np.float64)
    absmax = np.abs(x.double().numpy()).max(axis=0)
    # one bf16 ulp at the result, plus fp32 accumulation error (n ulps of fp32 at the
    # largest partial sum), which matters only when the sum nearly cancels
    tol = _ulp_bf16(want64) + n * absmax * n * 2.0 ** -24
    assert np.all(np.abs(got - want64) <= tol)


def test_allreduce_bf16_small_integers_exact_any_order(orc):
    g = torch.Generator().manual_seed(11)
    xi = torch.randint(-16, 17, (8, 9999), generator=g)      # |sum| <= 128: exact in bf16
    bits = synth.bf16_bits(xi.to(torch.bfloat16))
    want = synth.bf16_bits(xi.sum(0).to(torch.bfloat16))
    assert np.array_equal(orc.allreduce_bf16(bits), want)
    perm = np.array([5, 2, 7, 0, 3, 6, 1, 4])
    assert np.array_equal(orc.allreduce_bf16(bits[perm]), want)


def test_allreduce_bf16_one_and_two_ranks_vs_torch(orc):
    x = synth.normal(2, 100_003, seed=4)
    bits = synth.bf16_bits(x)
    assert np.array_equal(orc.allreduce_bf16(bits[:1]), bits[0])                     # N = 1: identity
    want = synth.bf16_bits((x[0].float() + x[1].float()).bfloat16())                  # library ops
    assert np.array_equal(orc.allreduce_bf16(bits), want)


def test_allreduce_bf16_order_accumulator_and_single_rounding(orc):
    f = lambda *v: synth.bf16_bits(torch.tensor(v, dtype=torch.float32).bfloat16().view(-1, 1))
    one = 0x3F80
    # fp32 accumulator, canonical order: (2^24 + 1) -> 2^24, then - 2^24 -> 0
    assert orc.allreduce_bf16(f(2.0 ** 24, 1.0, -2.0 ** 24))[0] == 0x0000
    assert orc.allreduce_bf16(f(2.0 ** 24, -2.0 ** 24, 1.0))[0] == one
    # single rounding at the end: 1 + 2^-8 + 2^-8 = 1 + 2^-7 exactly (one bf16 ulp above 1);
    # rounding to bf16 after every add would give 1 (each 2^-8 is a tie that goes to even)
    assert orc.allreduce_bf16(f(1.0, 2.0 ** -8, 2.0 ** -8))[0] == one + 1
    # accumulating in bf16-width would be wrong here, a wider-than-fp32 accumulator not needed


@pytest.mark.parametrize("n", [2, 3, 8])
@pytest.mark.parametrize("count", [1, 5, 64, 257])
def test_allreduce_bf16_bruteforce_fractions(orc, n, count):
    # fp32 accumulation replayed with exact rationals rounded to 24 bits at each step
    x = synth.normal(n, count, seed=20 + n)
    bits = synth.bf16_bits(x)
    out = orc.allreduce_bf16(bits)

    def rnd(fr, p):
        """round a Fraction to p significand bits, ties to even (no overflow/underflow here)"""
        if fr == 0:
            return fr
        s = -1 if fr < 0 else 1
        a = abs(fr)
        e = math.floor(math.log2(float(a)))
        while Fraction(2) ** e > a:
            e -= 1
        while Fraction(2) ** (e + 1) <= a:
            e += 1
        q = Fraction(2) ** (e - p + 1)
        k = a / q
        lo = k.numerator // k.denominator
        rem = k - lo
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
            lo += 1
        return s * lo * q

    for i in range(count):
        acc = Fraction(float(x[0, i]))
        for r in range(1, n):
            acc = rnd(acc + Fraction(float(x[r, i])), 24)
        want = float(rnd(acc, 8))
        got = float(orc.bf16_to_f32(out[i:i + 1])[0])
        assert got == want, (i, got, want)


# ---------------------------------------------------------------- fp16 and max / min

def test_f16_conversions_against_numpy(orc):
    codes = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    lib = codes.view(np.float16).astype(np.float32)                     # library decode, exact
    got = np.array([orc.f16_to_f32(c) for c in codes], np.float32)
    ok = ~np.isnan(lib)
    assert np.array_equal(got[ok].view(np.uint32), lib[ok].view(np.uint32)) and np.all(np.isnan(got[~ok]))
    for c in codes[ok][::7]:                                             # round trip
        assert orc.f32_to_f16(orc.f16_to_f32(c)) == c
    g = np.random.default_rng(4)
    x = (g.standard_normal(200_000) * np.exp(g.standard_normal(200_000) * 6)).astype(np.float32)
    x = np.concatenate([x, np.float32([65504, 65519.9, 65520, 65536, 1e9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
                                       2.0 ** -25 * 1.0001, 3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 * 0.9999, 0.0, -0.0,
                                       np.inf, -np.inf])])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)                     # library encode (round to nearest even)
    got = np.array([orc.f32_to_f16(v) for v in x], np.uint16)
    assert np.array_equal(got, want)
    assert orc.f32_to_f16(float("nan")) & 0x7C00 == 0x7C00 and orc.f32_to_f16(float("nan")) & 0x3FF


@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("n", [1, 2, 8])
def test_allreduce_any_against_numpy(orc, dtype, n):
    count = 5000
    g = torch.Generator().manual_seed(dtype * 10 + n)
    xf = torch.randn(n, count, generator=g) * 4
    if dtype == 0:
        x = xf.numpy()
        as_f32 = x
    elif dtype == 1:
        x = synth.bf16_bits(xf.bfloat16())
        as_f32 = xf.bfloat16().float().numpy()
    else:
        x = xf.numpy().astype(np.float16).view(np.uint16)
        as_f32 = xf.numpy().astype(np.float16).astype(np.float32)

    def back(bits):
        if dtype == 0:
            return bits
        return orc.bf16_to_f32(bits) if dtype == 1 else bits.view(np.float16).astype(np.float32)

    assert np.array_equal(back(orc.allreduce_any(x, dtype, 1)), as_f32.max(axis=0))       # exact: no rounding involved
    assert np.array_equal(back(orc.allreduce_any(x, dtype, 2)), as_f32.min(axis=0))
    acc = as_f32[0].copy()
    for r in range(1, n):
        acc = acc + as_f32[r]
    want = acc if dtype == 0 else (synth.bf16_bits(torch.from_numpy(acc).bfloat16()) if dtype == 1
                                   else acc.astype(np.float16).view(np.uint16))
    assert np.array_equal(orc.allreduce_any(x, dtype, 0), want)
    if dtype == 1:
        assert np.array_equal(orc.allreduce_any(x, 1, 0), orc.allreduce_bf16(x))
    # NaN rule: a later NaN never replaces a number, a NaN in rank 0 stays
    if n > 1 and dtype == 0:
        y = x.copy()
        y[1, 0] = np.nan
        y[0, 1] = np.nan
        out = orc.allreduce_any(y, 0, 1)
        assert out[0] == np.delete(y[:, 0], 1).max() and np.isnan(out[1])


@pytest.mark.parametrize("n", [1, 2, 3, 8])
def test_allreduce_any_int32_against_python_integers(orc, n):
    rng = np.random.default_rng(n)
    count = 3000
    x = rng.integers(-2**31, 2**31, (n, count), dtype=np.int64).astype(np.int32)
    x[0, :4] = [2**31 - 1, -2**31, 2**31 - 1, -1]                      # wrap-around on purpose
    if n > 1:
        x[1, :4] = [1, -1, 2**31 - 1, -2**31]
    exact = x.astype(np.int64).sum(axis=0)                            # no overflow in int64
    want = ((exact + 2**31) % 2**32 - 2**31).astype(np.int32)         # modulo 2^32, as a signed value
    assert np.array_equal(orc.allreduce_any(x, 3, 0), want)
    assert np.array_equal(orc.allreduce_any(x, 3, 1), x.max(axis=0))
    assert np.array_equal(orc.allreduce_any(x, 3, 2), x.min(axis=0))
    if n > 1:
        assert orc.allreduce_any(x, 3, 0)[0] == (2**31 - 1 + 1 + int(x[2:, 0].astype(np.int64).sum()) + 2**31) % 2**32 - 2**31
    small = rng.integers(-1000, 1001, (n, count)).astype(np.int32)    # the same numbers as floats: both paths agree
    assert np.array_equal(orc.allreduce_any(small, 3, 0), orc.allreduce_f32(small.astype(np.float32)).astype(np.int32))


# ---------------------------------------------------------------- ring order

@pytest.mark.parametrize("n", [1, 2, 3, 8])
def test_ring_order_allreduce(orc, n):
    c = 37
    count = n * c
    # integers: any order is exact
    xi = synth.int_valued_f32(n, count, seed=n).numpy()
    assert np.array_equal(orc.allreduce_ring(xi), orc.allreduce_f32(xi))
    # fp32: chunk k in ring order = rank-order sum of the ranks rotated so that rank k comes first
    g = torch.Generator().manual_seed(n)
    xf = (torch.randn(n, count, generator=g) * torch.exp(torch.randn(n, count, generator=g) * 4)).numpy()
    ring = orc.allreduce_ring(xf)
    for k in range(n):
        rolled = np.ascontiguousarray(np.roll(xf, -k, axis=0))
        assert np.array_equal(ring[k * c:(k + 1) * c], orc.allreduce_f32(rolled)[k * c:(k + 1) * c]), k
    # bf16: the partial is rounded at every hop; replay with torch's own conversions
    xb = synth.normal(n, count, seed=40 + n)
    ring = orc.allreduce_ring(synth.bf16_bits(xb))
    for k in range(n):
        part = xb[k, k * c:(k + 1) * c]
        for h in range(1, n):
            part = (part.float() + xb[(k + h) % n, k * c:(k + 1) * c].float()).bfloat16()
        assert np.array_equal(ring[k * c:(k + 1) * c], synth.bf16_bits(part)), k
    # and stays within the any-order tolerance of the fp64 sum
    ref = np.sum(xb.double().numpy(), axis=0)
    got = orc.bf16_to_f32(ring).astype(np.float64)
    absmax = np.abs(xb.double().numpy()).max(axis=0)
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref) + n * _ulp_bf16(n * absmax))


# ---------------------------------------------------------------- residual fusion

def test_residual_zero_and_zero_input(orc):
    x, res = synth.decode_activations(8, 2, hidden=512, seed=6)
    xb, rb = synth.bf16_bits(x), synth.bf16_bits(res)
    zero = np.zeros_like(rb)
    assert np.array_equal(orc.allreduce_residual_bf16(xb, zero), orc.allreduce_bf16(xb))
    assert np.array_equal(orc.allreduce_residual_bf16(np.zeros_like(xb), rb), rb)
    # single rounding: equals torch's fp32 chain rounded once
    acc = x[0].float()
    for r in range(1, 8):
        acc = acc + x[r].float()
    want = synth.bf16_bits((acc + res.float()).bfloat16())
    assert np.array_equal(orc.allreduce_residual_bf16(xb, rb), want)
    xf = x.float().numpy()
    assert np.array_equal(orc.allreduce_residual_f32(xf, res.float().numpy()),
                          (acc + res.float()).numpy())


# ---------------------------------------------------------------- ReduceScatter / AllGather / AllToAll

@pytest.mark.parametrize("n", RANKS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_allgather_of_reducescatter_is_allreduce(orc, n, dtype):
    count = n * 333
    if dtype == "f32":
        x = synth.int_valued_f32(n, count, seed=8).numpy()
        ar = orc.allreduce_f32(x)
    else:
        x = synth.bf16_bits(synth.normal(n, count, seed=8))
        ar = orc.allreduce_bf16(x)
    rs = orc.reducescatter(x)
    assert rs.shape == (n, count // n)
    ag = orc.allgather(rs)
    for r in range(n):
        assert np.array_equal(ag[r], ar)


@pytest.mark.parametrize("n", RANKS)
def test_reducescatter_bruteforce(orc, n):
    c = 5
    x = synth.int_valued_f32(n, n * c, seed=9).numpy()
    rs = orc.reducescatter(x)
    for r in range(n):
        for k in range(c):
            assert int(rs[r, k]) == sum(int(x[j, r * c + k]) for j in range(n))
    with pytest.raises(ValueError):
        orc.reducescatter(np.zeros((3, 4), np.float32))


@pytest.mark.parametrize("n", RANKS)
def test_allgather_alltoall_are_attributable_permutations(orc, n):
    c = 37
    # every element names its rank and position, so a misplaced one is attributable
    x = (np.arange(n)[:, None].astype(np.uint32) << 24) | np.arange(c, dtype=np.uint32)[None, :]
    ag = orc.allgather(x)
    for r in range(n):
        for j in range(n):
            assert np.array_equal(ag[r, j * c:(j + 1) * c], x[j])
    y = (np.arange(n)[:, None].astype(np.uint32) << 24) | np.arange(n * c, dtype=np.uint32)[None, :]
    a2a = orc.alltoall(y)
    for d in range(n):
        for s in range(n):
            assert np.array_equal(a2a[d, s * c:(s + 1) * c], y[s, d * c:(d + 1) * c])
    assert np.array_equal(orc.alltoall(a2a), y)             # involution
    y16 = y.astype(np.uint16)
    assert np.array_equal(orc.alltoall(orc.alltoall(y16)), y16)
    # numpy library form of the same block transpose
    want = y.reshape(n, n, c).transpose(1, 0, 2).reshape(n, n * c)
    assert np.array_equal(a2a, want)


# ---------------------------------------------------------------- LL units

def test_ll_unit_byte_layout_golden(orc):
    for data_hex, flag_hex, *mem in _read_table("ll_unit_layout.txt"):
        unit = orc.ll_encode(int(data_hex, 16), int(flag_hex, 16))
        got = list(np.array([unit], np.uint64).view(np.uint8))
        assert got == [int(b, 16) for b in mem]


def test_ll_roundtrip_and_flag_mismatch(orc):
    g = np.random.default_rng(3)
    words = [0, 1, 0xFFFFFFFF, 0x80000000, 0x7FFFFFFF] + [int(v) for v in g.integers(0, 2 ** 32, 200)]
    flags = [1, 2, 0x7FFFFFFF, 0xFFFFFFFF]
    for w in words:
        for fl in flags:
            u = orc.ll_encode(w, fl)
            assert orc.ll_decode(u, fl) == (True, w)
            assert orc.ll_decode(u, (fl + 1) & 0xFFFFFFFF) == (False, None)
            assert orc.ll_decode(u, fl ^ 0x80000000) == (False, None)
    # zero-initialised scratch never validates for a non-zero flag, whatever the data
    for fl in flags:
        assert orc.ll_decode(0, fl) == (False, None)


@pytest.mark.parametrize("nbytes", [0, 1, 3, 4, 5, 8, 9, 15, 16, 17, 1024, 1027])
def test_ll_buffer_encode_decode(orc, nbytes):
    g = np.random.default_rng(nbytes)
    payload = g.integers(0, 256, nbytes, dtype=np.uint8)
    flag = 0x1234
    units = orc.ll_encode_buf(payload, flag)
    assert units.size == 2 * ((nbytes + 7) // 8)
    ok, back = orc.ll_decode_buf(units, nbytes, flag)
    assert ok and np.array_equal(back, payload)
    raw = units.view(np.uint8).reshape(-1, 8)
    assert np.all(raw[:, 4:].view(np.uint32) == flag)        # every unit carries the flag
    padded = np.zeros(units.size * 4, np.uint8)
    padded[:nbytes] = payload
    assert np.array_equal(raw[:, :4].reshape(-1), padded)    # data words in order, zero padded
    if units.size:
        # a packet is ready only when BOTH of its units carry the flag
        for victim in (0, units.size - 1):
            broken = units.copy()
            broken[victim] = orc.ll_encode(int(broken[victim]) & 0xFFFFFFFF, flag - 1)
            assert orc.ll_decode_buf(broken, nbytes, flag) == (False, None)


# ---------------------------------------------------------------- token dispatch

def _dest_sets(topk, n, n_experts):
    per = n_experts // n
    return [[sorted({int(e) // per for e in tok}) for tok in rank] for rank in topk]


def test_moe_dispatch_properties(orc):
    n, T, H, K, E = 8, 96, 24, 8, 256
    tokens = synth.bf16_bits(synth.moe_tokens(n, T, H, seed=1))
    topk = synth.moe_routing(n, T, K, E, seed=1).numpy()
    recv, src, counts, rc = orc.moe_dispatch(tokens, topk, E)
    assert rc == 0
    dests = _dest_sets(topk, n, E)
    # conservation per source
    for s in range(n):
        assert counts[:, s].sum() == sum(len(d) for d in dests[s])
    # brute-force expected order, built independently in Python
    for d in range(n):
        want = [(s, t) for s in range(n) for t in range(T) if d in dests[s][t]]
        got = src[d, :len(want)]
        assert [int(v) for v in got] == [s * T + t for s, t in want]
        assert np.all(src[d, len(want):] == -1)
        for slot, (s, t) in enumerate(want):
            assert np.array_equal(recv[d, slot], tokens[s, t])
        for s in range(n):
            assert counts[d, s] == sum(1 for (ss, _) in want if ss == s)


def test_moe_dispatch_special_cases(orc):
    n, T, H, E = 8, 40, 8, 256
    tokens = synth.bf16_bits(synth.moe_tokens(n, T, H, seed=2))
    # K = 1: every token appears exactly once overall
    topk1 = synth.moe_routing(n, T, 1, E, seed=2).numpy()
    _, src, counts, rc = orc.moe_dispatch(tokens, topk1, E)
    assert rc == 0 and counts.sum() == n * T
    seen = sorted(int(v) for v in src[src >= 0])
    assert seen == list(range(n * T))
    # all experts of every token on rank 3: a plain gather to rank 3
    topk3 = np.tile(np.arange(96, 104, dtype=np.int32), (n, T, 1))
    recv, src, counts, rc = orc.moe_dispatch(tokens, topk3, E)
    assert rc == 0 and counts[3].tolist() == [T] * n and counts.sum() == n * T
    assert np.array_equal(recv[3, :n * T].reshape(n, T, H), tokens)
    # one expert on every rank: full replication == AllGather of the token blocks
    topk_all = np.tile(np.arange(0, 256, 32, dtype=np.int32), (n, T, 1))
    recv, src, counts, rc = orc.moe_dispatch(tokens, topk_all, E)
    ag = orc.allgather(tokens.reshape(n, T * H))
    assert rc == 0 and np.all(counts == T)
    assert np.array_equal(recv.reshape(n, n * T * H), ag)
    # duplicates of one expert or one rank do not duplicate the row
    topk_dup = np.zeros((n, T, 8), np.int32)
    _, _, counts, _ = orc.moe_dispatch(tokens, topk_dup, E)
    assert counts[0].tolist() == [T] * n and counts[1:].sum() == 0
    # capacity overflow and bad expert ids are reported
    assert orc.moe_dispatch(tokens, topk_all, E, cap=T)[3] == -1
    bad = topk_all.copy()
    bad[0, 0, 0] = 256
    assert orc.moe_dispatch(tokens, bad, E)[3] == -2


def test_moe_combine_properties(orc):
    n, T, H, K, E = 8, 64, 16, 8, 256
    tokens = synth.moe_tokens(n, T, H, seed=3)
    tb = synth.bf16_bits(tokens)
    topk = synth.moe_routing(n, T, K, E, seed=3).numpy()
    recv, src, counts, rc = orc.moe_dispatch(tb, topk, E)
    assert rc == 0
    dests = _dest_sets(topk, n, E)
    fan = np.array([[len(d) for d in rank] for rank in dests])
    # 1. combine of the dispatched rows themselves = fan-out x token, built independently with torch:
    #    repeated fp32 addition of the same value, one rounding
    out, rc = orc.moe_combine_bf16(recv, topk, E)
    assert rc == 0
    want = torch.zeros(n, T, H)
    tf = tokens.float()
    for k in range(1, 9):
        acc = tf.clone()
        for _ in range(k - 1):
            acc = acc + tf
        m = torch.from_numpy(fan == k)
        want[m] = acc[m]
    assert np.array_equal(out, synth.bf16_bits(want.bfloat16()))
    # 2. rows that carry their destination rank as value: result = sum of the destination ids,
    #    which pins WHICH rows are summed for each token
    y = np.zeros_like(recv)
    for d in range(n):
        y[d] = synth.bf16_bits(torch.full((1,), float(d + 1)).bfloat16())[0]
    out, _ = orc.moe_combine_bf16(y, topk, E)
    want_ids = np.array([[sum(d + 1 for d in ds) for ds in rank] for rank in dests], np.float32)
    got = orc.bf16_to_f32(out)
    assert np.array_equal(got, np.repeat(want_ids[:, :, None], H, axis=2))
    # 3. rows that carry their source position: every summed row must be the token's own
    y = np.zeros_like(recv)
    for d in range(n):
        for slot in range(int(counts[d].sum())):
            y[d, slot] = synth.bf16_bits(torch.full((1,), float(src[d, slot] % 31)).bfloat16())[0]
    out, _ = orc.moe_combine_bf16(y, topk, E)
    idx = (np.arange(n)[:, None] * T + np.arange(T)[None, :]) % 31
    assert np.array_equal(orc.bf16_to_f32(out)[:, :, 0], (idx * fan).astype(np.float32))   # <= 240: exact in bf16
    # 4. order and single rounding: ranks 0,1,2 deliver 2^24*2^-16.. use the probe 256, 1, -256 scaled to bf16
    topk3 = np.tile(np.array([0, 32, 64, 1, 2, 3, 4, 5], np.int32), (n, T, 1))             # ranks 0,1,2
    recv3, _, counts3, _ = orc.moe_dispatch(tb, topk3, E)
    y = np.zeros_like(recv3)
    vals = {0: 2.0 ** 24, 1: 1.0, 2: -(2.0 ** 24)}
    for d, v in vals.items():
        y[d, :int(counts3[d].sum())] = synth.bf16_bits(torch.full((1,), v).bfloat16())[0]
    out, _ = orc.moe_combine_bf16(y, topk3, E)
    assert np.all(out == 0)                                   # (2^24 + 1) - 2^24 = 0 in fp32, rank order
    # 5. capacity and id errors are reported
    assert orc.moe_combine_bf16(recv[:, :10], topk, E)[1] == -1
    bad = topk.copy()
    bad[1, 2, 3] = -1
    assert orc.moe_combine_bf16(recv, bad, E)[1] == -2


def test_moe_expected_fanout_of_the_seeded_routing():
    n, T, K, E = 8, 4096, 8, 256
    topk = synth.moe_routing(n, T, K, E, seed=0).numpy()
    assert np.all(np.sort(topk, axis=2)[:, :, 1:] != np.sort(topk, axis=2)[:, :, :-1])   # distinct
    fan = np.mean([len(set((tok // 32).tolist())) for rank in topk for tok in rank])
    p_miss = math.comb(224, 8) / math.comb(256, 8)
    expect = 8 * (1 - p_miss)
    assert abs(expect - 5.295) < 1e-3
    assert abs(fan - expect) < 0.03


# ---------------------------------------------------------------- FP8 E4M3

def test_e4m3_decode_all_codes_closed_form_and_torch(orc):
    codes = np.arange(256, dtype=np.uint8)
    got = np.array([orc.e4m3_to_f32(c) for c in codes], np.float32)
    for c in codes:
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            assert np.isnan(got[c])
            continue
        want = (2.0 ** -6) * (m / 8.0) if e == 0 else (2.0 ** (int(e) - 7)) * (1 + m / 8.0)
        assert got[c] == np.float32(-want if s else want), c
    assert got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).float().numpy()      # library decode
    ok = ~np.isnan(lib)
    assert np.array_equal(got[ok], lib[ok]) and np.all(np.isnan(got[~ok]))


def test_e4m3_encode_roundtrip_ties_saturation_and_torch(orc):
    for c in range(256):
        v = orc.e4m3_to_f32(c)
        if v != v:
            assert orc.f32_to_e4m3(v) == 0x7F
        else:
            assert orc.f32_to_e4m3(v) == c, c                      # includes -0 -> 0x80
    # hand-worked: spacing is 0.125 in [1,2): 1.0625 is the tie between 1.0 (0x38, even) and 1.125 (0x39)
    assert orc.f32_to_e4m3(1.0625) == 0x38 and orc.f32_to_e4m3(1.1875) == 0x3A   # tie between 0x39 and 0x3A -> even
    assert orc.f32_to_e4m3(1.07) == 0x39 and orc.f32_to_e4m3(1.05) == 0x38
    assert orc.f32_to_e4m3(2.0 ** -10) == 0x00 and orc.f32_to_e4m3(2.0 ** -10 * 1.01) == 0x01   # subnormal tie / just above
    assert orc.f32_to_e4m3(3 * 2.0 ** -10) == 0x02                                       # tie 1.5 ulp -> even (2)
    assert orc.f32_to_e4m3(448.0) == 0x7E and orc.f32_to_e4m3(464.0) == 0x7E and orc.f32_to_e4m3(1e30) == 0x7E
    assert orc.f32_to_e4m3(-1e30) == 0xFE and orc.f32_to_e4m3(float("inf")) == 0x7E
    assert orc.f32_to_e4m3(440.0) == 0x7E                          # above the tie (432) between 416 and 448
    assert orc.f32_to_e4m3(432.0) == 0x7E                          # the tie itself: 0x7D is odd -> up
    assert orc.f32_to_e4m3(float("nan")) == 0x7F
    g = torch.Generator().manual_seed(2)
    x = torch.randn(20000, generator=g) * torch.exp(torch.randn(20000, generator=g) * 3)
    x = x[x.abs() <= 448.0]
    lib = x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()                              # library encode (RNE)
    got = np.array([orc.f32_to_e4m3(v) for v in x.numpy()], np.uint8)
    assert np.array_equal(got, lib)


def test_fp8_row_quantisation(orc):
    x = synth.normal(6, 7168, seed=12)
    x[2] *= 1000.0
    x[3] = 0
    x[4, :128] = 0.5                                                                      # a constant group
    q, scales = orc.fp8_quantize_rows(synth.bf16_bits(x))
    xf = x.float().view(6, 56, 128)
    # IEEE fp32 division and multiplication with numpy (torch's scalar / tensor goes through a
    # reciprocal and is not correctly rounded), torch's float8 type as the library encoder
    xn = xf.numpy()
    amax = np.maximum(np.abs(xn).max(axis=2), np.float32(1e-4)).astype(np.float32)
    assert np.array_equal(scales, amax / np.float32(448.0))
    scaled = xn * (np.float32(448.0) / amax)[:, :, None]
    assert scaled.dtype == np.float32
    lib = torch.from_numpy(scaled).to(torch.float8_e4m3fn).view(torch.uint8).view(6, 7168).numpy()
    assert np.array_equal(q, lib)
    assert np.all(q[3] == 0) and np.all(scales[3] == np.float32(1e-4) / np.float32(448.0))
    assert np.all(q[4, :128] == 0x7E) and scales[4, 0] == np.float32(0.5) / np.float32(448.0)
    # every group uses the top code at least once (the element that set amax), dequantisation is close
    deq = np.array([[orc.e4m3_to_f32(c) for c in row] for row in q[:2]]).reshape(2, 56, 128) * scales[:2, :, None]
    assert np.all((q[:2].reshape(2, 56, 128) & 0x7F).max(axis=2) == 0x7E)
    err = np.abs(deq - xn[:2])
    assert np.all(err <= 0.0625 * np.abs(xn[:2]) + scales[:2, :, None] * 2.0 ** -9 + 1e-7)


# ---------------------------------------------------------------- semaphore counter

def test_sem_reached_is_wrap_safe(orc):
    assert orc.sem_reached(5, 5) and orc.sem_reached(6, 5) and not orc.sem_reached(4, 5)
    assert orc.sem_reached(1, 0xFFFFFFFE)                    # counter wrapped past the target
    assert not orc.sem_reached(0xFFFFFFFE, 1)                # target is ahead across the wrap
    assert orc.sem_reached(0, 0) and not orc.sem_reached(0, 1)
