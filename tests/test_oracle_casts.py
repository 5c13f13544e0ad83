"""Pins of the oracle's element conversions (paper Section III-B: data type conversion in the same
pass, e.g. BFloat16 <-> half).  Round to nearest, ties to even, defined on bit patterns.

Independent references: numpy's float16 and torch's CPU bfloat16 for every non-NaN input; IEEE-754
closed-form constants typed here; NaN results by properties only (the two libraries disagree with
each other on NaN payloads, so library parity is unpinned there)."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc

ALL16 = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)


def _is_nan16(bits, exp_mask, man_mask):
    return ((bits & exp_mask) == exp_mask) & ((bits & man_mask) != 0)


def _f32_samples():
    rng = np.random.default_rng(0)
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    ties = [hi | lo for lo in (0x0000, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x0001)]      # bf16 ties
    hi13 = (np.arange(1 << 19, dtype=np.uint32) << 13)
    ties16 = [hi13 | lo for lo in (0x0000, 0x0FFF, 0x1000, 0x1001, 0x1FFF)]           # fp16 ties
    sub = np.uint32(0x33000000) + np.arange(0, 0x05800000, 0x3FF, dtype=np.uint32)   # fp16 subnormal zone
    rnd = rng.integers(0, 1 << 32, 4_000_000, dtype=np.uint64).astype(np.uint32)
    x = np.concatenate(ties + ties16 + [sub, sub | np.uint32(0x80000000), rnd])
    return x


def test_f16_to_f32_exhaustive_vs_numpy():
    got = orc.cast_array(ALL16, "F16", "F32")
    ref = ALL16.view(np.float16).astype(np.float32).view(np.uint32)
    nan = _is_nan16(ALL16, 0x7C00, 0x03FF)
    assert np.array_equal(got[~nan], ref[~nan])


def test_bf16_to_f32_exhaustive_vs_torch():
    got = orc.cast_array(ALL16, "BF16", "F32")
    ref = torch.from_numpy(ALL16.view(np.int16)).view(torch.bfloat16).to(torch.float32).view(torch.int32).numpy().view(np.uint32)
    nan = _is_nan16(ALL16, 0x7F80, 0x007F)
    assert np.array_equal(got[~nan], ref[~nan])
    # a bfloat16 is the upper half of the binary32 with the same value
    assert np.array_equal(got[~nan], ALL16[~nan].astype(np.uint32) << 16)


def test_f16_to_bf16_exhaustive_vs_torch():
    got = orc.cast_array(ALL16, "F16", "BF16")
    ref = torch.from_numpy(ALL16.view(np.int16)).view(torch.float16).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = _is_nan16(ALL16, 0x7C00, 0x03FF)
    assert np.array_equal(got[~nan], ref[~nan])


def test_bf16_to_f16_exhaustive_vs_numpy_and_torch():
    got = orc.cast_array(ALL16, "BF16", "F16")
    nan = _is_nan16(ALL16, 0x7F80, 0x007F)
    f32 = (ALL16.astype(np.uint32) << 16).view(np.float32)
    with np.errstate(over="ignore"):
        ref_np = f32.astype(np.float16).view(np.uint16)
    ref_t = torch.from_numpy(ALL16.view(np.int16)).view(torch.bfloat16).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got[~nan], ref_np[~nan])
    assert np.array_equal(got[~nan], ref_t[~nan])


def test_f32_to_bf16_vs_torch():
    x = _f32_samples()
    got = orc.cast_array(x, "F32", "BF16")
    ref = torch.from_numpy(x.view(np.int32)).view(torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = (x & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(got[~nan], ref[~nan])


def test_f32_to_f16_vs_numpy():
    x = _f32_samples()
    got = orc.cast_array(x, "F32", "F16")
    with np.errstate(over="ignore"):
        ref = x.view(np.float32).astype(np.float16).view(np.uint16)
    nan = (x & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(got[~nan], ref[~nan])


def test_widen_then_narrow_is_identity():
    for dt, em, mm in (("F16", 0x7C00, 0x03FF), ("BF16", 0x7F80, 0x007F)):
        wide = orc.cast_array(ALL16, dt, "F32")
        back = orc.cast_array(wide, "F32", dt)
        nan = _is_nan16(ALL16, em, mm)
        assert np.array_equal(back[~nan], ALL16[~nan])
    # fp16 -> bf16 -> ... is lossy, but bf16 values that fp16 holds exactly survive bf16 -> f16 -> bf16
    h = orc.cast_array(ALL16, "BF16", "F16")
    b = orc.cast_array(h, "F16", "BF16")
    f = (ALL16.astype(np.uint32) << 16).view(np.float32)
    exact = np.isfinite(f) & (np.abs(f) <= 65504) & ((np.abs(f) >= 2.0 ** -14) | (f == 0))
    assert np.array_equal(b[exact], ALL16[exact])


def test_ieee_constants():
    """Values fixed by IEEE-754 binary16/binary32 and the bfloat16 layout, typed by hand."""
    c = lambda v, s, d: int(orc.cast_array(np.array([v], np.uint32 if s == "F32" else np.uint16), s, d)[0])
    assert c(0x3C00, "F16", "F32") == 0x3F800000            # 1.0
    assert c(0x0001, "F16", "F32") == 0x33800000            # 2^-24, smallest subnormal
    assert c(0x03FF, "F16", "F32") == 0x387FC000            # largest subnormal = 1023 * 2^-24
    assert c(0x7BFF, "F16", "F32") == 0x477FE000            # 65504
    assert c(0xFC00, "F16", "F32") == 0xFF800000            # -inf
    assert c(0x8000, "F16", "F32") == 0x80000000            # -0
    assert c(0x477FE000, "F32", "F16") == 0x7BFF
    assert c(0x477FEFFF, "F32", "F16") == 0x7BFF            # just below the midpoint to 65536
    assert c(0x477FF000, "F32", "F16") == 0x7C00            # 65520: tie, even is 65536 -> inf
    assert c(0x33000000, "F32", "F16") == 0x0000            # 2^-25: tie between 0 and 2^-24 -> 0
    assert c(0x33000001, "F32", "F16") == 0x0001
    assert c(0x33C00000, "F32", "F16") == 0x0002            # 1.5 * 2^-24: tie -> even (2)
    assert c(0x387FE000, "F32", "F16") == 0x0400            # 1023.5 * 2^-24: tie -> 1024 = min normal
    assert c(0x38800000, "F32", "F16") == 0x0400            # 2^-14
    assert c(0xB3000001, "F32", "F16") == 0x8001
    assert c(0x3F808000, "F32", "BF16") == 0x3F80           # tie -> even (down)
    assert c(0x3F818000, "F32", "BF16") == 0x3F82           # tie -> even (up)
    assert c(0x3F808001, "F32", "BF16") == 0x3F81
    assert c(0x7F7FFFFF, "F32", "BF16") == 0x7F80           # max finite rounds to inf
    assert c(0x7F7F7FFF, "F32", "BF16") == 0x7F7F
    assert c(0x00000001, "F32", "BF16") == 0x0000           # tiny subnormal -> +0
    assert c(0x80008000, "F32", "BF16") == 0x8000           # tie at the bottom -> even (-0)
    assert c(0x00018000, "F32", "BF16") == 0x0002
    assert c(0x3C00, "F16", "BF16") == 0x3F80
    assert c(0x0001, "F16", "BF16") == 0x3380               # 2^-24 is a normal bfloat16
    assert c(0x3C08, "F16", "BF16") == 0x3F81               # 1 + 2^-7 exactly representable
    assert c(0x3C04, "F16", "BF16") == 0x3F80               # 1 + 2^-8: tie -> even
    assert c(0x3C0C, "F16", "BF16") == 0x3F82               # 1 + 3*2^-8: tie -> even (up)
    assert c(0x4780, "BF16", "F16") == 0x7C00               # 65536 overflows
    assert c(0x3380, "BF16", "F16") == 0x0001
    assert c(0x3300, "BF16", "F16") == 0x0000               # 2^-25: tie -> 0


def test_nan_properties():
    """NaN in -> NaN out, sign kept, quiet bit set, leading payload bits kept."""
    h = ALL16[_is_nan16(ALL16, 0x7C00, 0x03FF)]
    b = ALL16[_is_nan16(ALL16, 0x7F80, 0x007F)]
    w = orc.cast_array(h, "F16", "F32")
    assert np.all((w & 0x7FC00000) == 0x7FC00000) and np.array_equal(w >> 31, h >> 15)
    assert np.array_equal((w >> 13) & 0x1FF, h & 0x1FF)
    w = orc.cast_array(b, "BF16", "F32")
    assert np.all((w & 0x7FC00000) == 0x7FC00000) and np.array_equal(w >> 31, b >> 15)
    assert np.array_equal((w >> 16) & 0x3F, b & 0x3F) and np.all((w & 0xFFFF) == 0)
    n = orc.cast_array(h, "F16", "BF16")
    assert np.all((n & 0x7FC0) == 0x7FC0) and np.array_equal(n >> 15, h >> 15)
    assert np.array_equal(n & 0x3F, (h >> 3) & 0x3F)
    n = orc.cast_array(b, "BF16", "F16")
    assert np.all((n & 0x7E00) == 0x7E00) and np.array_equal(n >> 15, b >> 15)
    rng = np.random.default_rng(1)
    x = (rng.integers(0, 1 << 32, 200000, dtype=np.uint64).astype(np.uint32) | np.uint32(0x7F800000))
    x = x[(x & 0x7FFFFF) != 0]
    n = orc.cast_array(x, "F32", "BF16")
    assert np.all((n & 0x7FC0) == 0x7FC0) and np.array_equal(n >> 15, (x >> 31).astype(np.uint16))
    assert np.array_equal(n & 0x3F, ((x >> 16) & 0x3F).astype(np.uint16))
    n = orc.cast_array(x, "F32", "F16")
    assert np.all((n & 0x7E00) == 0x7E00) and np.array_equal(n >> 15, (x >> 31).astype(np.uint16))
    assert np.array_equal(n & 0x1FF, ((x >> 13) & 0x1FF).astype(np.uint16))


def _f64_samples():
    """binary64 inputs around everything binary32 rounding can meet: every 1021st binary32 value
    widened exactly, its exact midpoint to the next binary32 value (a tie) and the neighbours of that
    midpoint and of the value itself; random patterns; the binary32 subnormal zone with its ties (odd
    multiples of 2^-150); the overflow zone."""
    rng = np.random.default_rng(3)
    b = np.arange(0, 1 << 32, 1021, dtype=np.uint64).astype(np.uint32)
    b = b[(b & 0x7FFFFFFF) < 0x7F800000]
    w = b.view(np.float32).astype(np.float64).view(np.uint64)          # exact widening by numpy
    parts = [w, w + np.uint64(1 << 28), w + np.uint64((1 << 28) - 1), w + np.uint64((1 << 28) + 1),
             w + np.uint64(1), w - np.uint64(1)]
    parts.append(rng.integers(0, 1 << 64, 2_000_000, dtype=np.uint64))
    e = rng.integers(860, 900, 1_000_000, dtype=np.uint64)
    m = rng.integers(0, 1 << 52, 1_000_000, dtype=np.uint64)
    z = (e << np.uint64(52)) | m
    parts += [z, z | np.uint64(1 << 63)]
    parts.append((np.arange(1, 1 << 19, dtype=np.uint64).astype(np.float64) * 2.0 ** -150).view(np.uint64))
    e = rng.integers(1023 + 120, 1023 + 130, 300_000, dtype=np.uint64)
    m = rng.integers(0, 1 << 52, 300_000, dtype=np.uint64)
    parts.append((e << np.uint64(52)) | m)
    return np.concatenate(parts)


def test_f64_to_f32_vs_numpy():
    d = _f64_samples()
    got = orc.cast_array(d, "F64", "F32")
    with np.errstate(over="ignore", invalid="ignore"):
        ref = d.view(np.float64).astype(np.float32).view(np.uint32)
    ok = (d & np.uint64(0x7FFFFFFFFFFFFFFF)) <= np.uint64(0x7FF0000000000000)
    assert np.array_equal(got[ok], ref[ok])
    # and against torch, a second library
    ref2 = torch.from_numpy(d.view(np.float64)).to(torch.float32).view(torch.int32).numpy().view(np.uint32)
    assert np.array_equal(got[ok], ref2[ok])


def test_f32_to_f64_vs_numpy_and_back():
    x = np.concatenate([_f32_samples(), np.arange(0, 0x01000000, 7, dtype=np.uint32)])       # plus many subnormals
    got = orc.cast_array(x, "F32", "F64")
    with np.errstate(invalid="ignore"):
        ref = x.view(np.float32).astype(np.float64).view(np.uint64)
    ok = (x & 0x7FFFFFFF) <= 0x7F800000
    assert np.array_equal(got[ok], ref[ok])
    assert np.array_equal(orc.cast_array(got[ok], "F64", "F32"), x[ok])     # widening is exact


def test_f64_constants_and_nan():
    """binary64 <-> binary32 values fixed by IEEE-754, typed by hand."""
    n = lambda v: int(orc.cast_array(np.array([v], np.uint64), "F64", "F32")[0])
    w = lambda v: int(orc.cast_array(np.array([v], np.uint32), "F32", "F64")[0])
    assert w(0x3F800000) == 0x3FF0000000000000                     # 1.0
    assert w(0x00000001) == 0x36A0000000000000                     # 2^-149
    assert w(0x007FFFFF) == 0x380FFFFFC0000000                     # largest subnormal
    assert w(0x7F7FFFFF) == 0x47EFFFFFE0000000                     # largest finite
    assert w(0xFF800000) == 0xFFF0000000000000 and w(0x80000000) == 0x8000000000000000
    assert n(0x3FF0000000000000) == 0x3F800000
    assert n(0x3FF0000010000000) == 0x3F800000                     # 1 + 2^-24: tie -> even (down)
    assert n(0x3FF0000030000000) == 0x3F800002                     # 1 + 3*2^-24: tie -> even (up)
    assert n(0x3FF0000010000001) == 0x3F800001
    assert n(0x47EFFFFFEFFFFFFF) == 0x7F7FFFFF                     # just below the midpoint to 2^128
    assert n(0x47EFFFFFF0000000) == 0x7F800000                     # the midpoint: tie -> even = infinity
    assert n(0x47F0000000000000) == 0x7F800000                     # 2^128
    assert n(0x36A0000000000000) == 0x00000001                     # 2^-149
    assert n(0x3690000000000000) == 0x00000000                     # 2^-150: tie between 0 and 2^-149 -> 0
    assert n(0x3690000000000001) == 0x00000001
    assert n(0x36A8000000000000) == 0x00000002                     # 1.5 * 2^-149: tie -> even (2)
    assert n(0x380FFFFFE0000000) == 0x00800000                     # (2^24 - 1) * 2^-150: tie -> smallest normal
    assert n(0xB690000000000001) == 0x80000001 and n(0x0000000000000001) == 0 and n(0x8000000000000001) == 0x80000000
    rng = np.random.default_rng(4)
    d = rng.integers(0, 1 << 64, 100000, dtype=np.uint64) | np.uint64(0x7FF0000000000000)
    d = d[(d & np.uint64(0xFFFFFFFFFFFFF)) != 0]
    f = orc.cast_array(d, "F64", "F32")
    assert np.all((f & 0x7FC00000) == 0x7FC00000) and np.array_equal(f >> 31, (d >> np.uint64(63)).astype(np.uint32))
    assert np.array_equal(f & 0x3FFFFF, ((d >> np.uint64(29)) & np.uint64(0x3FFFFF)).astype(np.uint32))
    x = rng.integers(0, 1 << 32, 100000, dtype=np.uint64).astype(np.uint32) | np.uint32(0x7F800000)
    x = x[(x & 0x7FFFFF) != 0]
    g = orc.cast_array(x, "F32", "F64")
    assert np.all((g & np.uint64(0x7FF8000000000000)) == np.uint64(0x7FF8000000000000))
    assert np.array_equal((g >> np.uint64(63)).astype(np.uint32), x >> 31)
    assert np.array_equal(((g >> np.uint64(29)) & np.uint64(0x3FFFFF)).astype(np.uint32), x & 0x3FFFFF)
    assert np.all((g & np.uint64(0x1FFFFFFF)) == 0)


def test_identity_and_unsupported():
    x = np.arange(256, dtype=np.uint8)
    for dt in ("BOOL", "U8", "I8", "F8_E5M2", "F8_E4M3"):
        assert np.array_equal(orc.cast_array(x, dt, dt), x)
    assert np.array_equal(orc.cast_array(ALL16, "F16", "F16"), ALL16)     # NaN payloads untouched
    for s, d in (("I16", "F16"), ("U16", "BF16"), ("F64", "I64"), ("U8", "BOOL"), ("F8_E5M2", "F64"), ("F8_E4M3", "F8_E5M2"),
                 ("F16", "F8_E4M3"), ("F32", "F8_E5M2"), ("I64", "F64")):
        with pytest.raises(orc.OracleError) as e:
            orc.cast_array(np.zeros(8, np.uint8), s, d)
        assert e.value.kind == "CAST"


# ---------------------------------------------------------------- binary64 <-> 16-bit types
# One rounding from the 53-bit significand.  Independent references: numpy's direct float64 -> float16
# conversion; round-half-even on exact rationals (Python's fractions); inputs built a hair beside every
# tie of the target format, whose result is known by construction and which rounding twice (through
# binary32) gets wrong; torch for the exact widenings.

_FMT = {"F16": (10, 15), "BF16": (7, 127)}          # stored mantissa bits, exponent bias


def _widen16(bits, fmt):
    """Exact binary64 value of 16-bit patterns, by a library (numpy float16 / torch bfloat16)."""
    bits = np.ascontiguousarray(bits, np.uint16)
    if fmt == "F16":
        return bits.view(np.float16).astype(np.float64)
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


def _near_tie_inputs(fmt):
    """For every pair of neighbouring finite values a < b of the format (same sign): the midpoint
    (exact in binary64) and the binary64 numbers just below and just above it, with the expected
    16-bit result: lower neighbour, the even one, upper neighbour."""
    mb, _ = _FMT[fmt]
    top = 0x7C00 if fmt == "F16" else 0x7F80
    lo = np.arange(0, top - 1, dtype=np.uint16)                 # 0 .. largest finite - 1
    hi = lo + np.uint16(1)
    a, b = _widen16(lo, fmt), _widen16(hi, fmt)
    mid = (a + b) / 2                                           # exact: one more significant bit
    below, above = np.nextafter(mid, -np.inf), np.nextafter(mid, np.inf)
    even = np.where(lo & 1, hi, lo)
    x = np.concatenate([below, mid, above])
    want = np.concatenate([lo, even, hi]).astype(np.uint16)
    # and the negative half
    return np.concatenate([x, -x]), np.concatenate([want, want | np.uint16(0x8000)])


@pytest.mark.parametrize("fmt", ["F16", "BF16"])
def test_f64_to_16bit_near_every_tie(fmt):
    x, want = _near_tie_inputs(fmt)
    got = orc.cast_array(x.view(np.uint64), "F64", fmt)
    assert np.array_equal(got, want)
    # the same inputs rounded twice (binary64 -> binary32 -> 16 bit) differ: the pin can tell the two apart
    twice = orc.cast_array(orc.cast_array(x.view(np.uint64), "F64", "F32"), "F32", fmt)
    assert np.count_nonzero(twice != want) > 1000


def _f64_samples_16(fmt):
    """binary64 inputs over the 16-bit format's whole range: random patterns with the exponent drawn from
    the format's span (a few binades beyond both ends), binary32 values widened (rounding twice is exact
    there), plus the near-tie set."""
    mb, bias = _FMT[fmt]
    rng = np.random.default_rng(11)
    e = rng.integers(1023 - bias - mb - 4, 1023 + bias + 4, 1_500_000, dtype=np.uint64)
    m = rng.integers(0, 1 << 52, 1_500_000, dtype=np.uint64)
    s = rng.integers(0, 2, 1_500_000, dtype=np.uint64) << np.uint64(63)
    # low mantissa bits zeroed in a third of the samples: exact ties of the 16-bit format and values on its grid
    keep = rng.integers(52 - mb - 2, 53, 1_500_000, dtype=np.uint64)
    m2 = np.where(rng.random(1_500_000) < 0.33, (m >> keep) << keep, m)
    return np.concatenate([s | (e << np.uint64(52)) | m2, rng.integers(0, 1 << 64, 500_000, dtype=np.uint64)])


def test_f64_to_f16_vs_numpy():
    d = np.concatenate([_f64_samples_16("F16"), _f64_samples()[::7]])
    got = orc.cast_array(d, "F64", "F16")
    with np.errstate(over="ignore", invalid="ignore", under="ignore"):
        ref = d.view(np.float64).astype(np.float16).view(np.uint16)
    ok = (d & np.uint64(0x7FFFFFFFFFFFFFFF)) <= np.uint64(0x7FF0000000000000)
    assert np.array_equal(got[ok], ref[ok])


@pytest.mark.parametrize("fmt", ["F16", "BF16"])
def test_f64_to_16bit_vs_exact_rationals(fmt):
    """Definition of round-to-nearest-even, carried out on exact rationals: the result is the multiple of
    the local unit closest to x, ties to the even multiple (Python's round() on a Fraction does that)."""
    from fractions import Fraction
    mb, bias = _FMT[fmt]
    emin = 1 - bias                                            # exponent of the smallest normal
    d = _f64_samples_16(fmt)[::97]
    d = d[(d & np.uint64(0x7FFFFFFFFFFFFFFF)) < np.uint64(0x7FF0000000000000)]
    got = orc.cast_array(d, "F64", fmt)
    max_finite = Fraction(2 - Fraction(1, 1 << mb)) * Fraction(2) ** bias
    for bits, g in zip(d.tolist(), got.tolist()):
        x = float(np.array([bits], np.uint64).view(np.float64)[0])
        sign = 0x8000 if bits >> 63 else 0
        ax = abs(Fraction(x))
        if ax == 0:
            assert g == sign
            continue
        e = max(ax.numerator.bit_length() - ax.denominator.bit_length(), emin - 1)
        while Fraction(2) ** e > ax and e > emin:              # floor(log2 |x|), not below emin
            e -= 1
        while Fraction(2) ** (e + 1) <= ax:
            e += 1
        e = max(e, emin)
        unit = Fraction(2) ** (e - mb)
        q = round(ax / unit)                                   # half to even
        val = q * unit
        if val > max_finite:                                   # rounds past the largest finite value
            want = sign | (0x7C00 if fmt == "F16" else 0x7F80)
        else:
            # encode val = q * 2^(e-mb): q < 2^mb is subnormal (e == emin), q == 2^(mb+1) carries into the next binade
            if q == 1 << (mb + 1):
                q, e = 1 << mb, e + 1
            want = sign | (q if q < (1 << mb) else ((e + bias) << mb) | (q - (1 << mb)))
        assert g == want, (hex(bits), hex(g), hex(want))


@pytest.mark.parametrize("fmt", ["F16", "BF16"])
def test_16bit_to_f64_exhaustive_and_back(fmt):
    got = orc.cast_array(ALL16, fmt, "F64")
    ref = _widen16(ALL16, fmt).view(np.uint64)
    nan = _is_nan16(ALL16, *((0x7C00, 0x03FF) if fmt == "F16" else (0x7F80, 0x007F)))
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(orc.cast_array(got[~nan], "F64", fmt), ALL16[~nan])      # widening is exact
    # widening in two exact steps or one gives the same bits, NaN included
    assert np.array_equal(got, orc.cast_array(orc.cast_array(ALL16, fmt, "F32"), "F32", "F64"))


def test_f64_16bit_constants_and_nan():
    h = lambda v: int(orc.cast_array(np.array([v], np.uint64), "F64", "F16")[0])
    b = lambda v: int(orc.cast_array(np.array([v], np.uint64), "F64", "BF16")[0])
    assert h(0x3FF0000000000000) == 0x3C00 and b(0x3FF0000000000000) == 0x3F80        # 1.0
    assert h(0xC004000000000000) == 0xC100 and b(0xC004000000000000) == 0xC020        # -2.5
    assert h(0x3FF0020000000000) == 0x3C00            # 1 + 2^-11: tie -> even (down)
    assert h(0x3FF0020000000001) == 0x3C01            # one binary64 ulp above the tie: up (via binary32: 0x3C00)
    assert h(0x3FF0060000000000) == 0x3C02            # 1 + 3*2^-11: tie -> even (up)
    assert b(0x3FF0100000000000) == 0x3F80            # 1 + 2^-8: tie -> even (down)
    assert b(0x3FF0100000000001) == 0x3F81            # just above (via binary32: 0x3F80)
    assert b(0x3FF0300000000000) == 0x3F82
    assert h(0x40EFFC0000000000) == 0x7BFF            # 65504, largest finite
    assert h(0x40EFFDFFFFFFFFFF) == 0x7BFF            # just below 65520
    assert h(0x40EFFE0000000000) == 0x7C00            # 65520: tie -> even = infinity
    assert h(0x3E70000000000000) == 0x0001            # 2^-24, smallest subnormal
    assert h(0x3E60000000000000) == 0x0000            # 2^-25: tie between 0 and 2^-24 -> 0
    assert h(0x3E60000000000001) == 0x0001
    assert h(0x3E78000000000000) == 0x0002            # 1.5 * 2^-24: tie -> even
    assert h(0x3F0FFE0000000000) == 0x0400            # (2^11 - 1) * 2^-25: tie -> smallest normal
    assert b(0x47EFE00000000000) == 0x7F7F            # largest finite bfloat16
    assert b(0x47EFF00000000000) == 0x7F80            # midpoint to 2^128: tie -> even = infinity
    assert b(0x47EFEFFFFFFFFFFF) == 0x7F7F
    assert b(0x37A0000000000000) == 0x0001            # 2^-133, smallest subnormal
    assert b(0x3790000000000000) == 0x0000 and b(0x3790000000000001) == 0x0001
    assert b(0x0000000000000001) == 0 and h(0x8000000000000001) == 0x8000
    assert h(0x7FF0000000000000) == 0x7C00 and b(0xFFF0000000000000) == 0xFF80
    rng = np.random.default_rng(12)
    d = rng.integers(0, 1 << 64, 100000, dtype=np.uint64) | np.uint64(0x7FF0000000000000)
    d = d[(d & np.uint64(0xFFFFFFFFFFFFF)) != 0]
    n = orc.cast_array(d, "F64", "F16")
    assert np.all((n & 0x7E00) == 0x7E00) and np.array_equal(n >> 15, (d >> np.uint64(63)).astype(np.uint16))
    assert np.array_equal(n & 0x1FF, ((d >> np.uint64(42)) & np.uint64(0x1FF)).astype(np.uint16))
    n = orc.cast_array(d, "F64", "BF16")
    assert np.all((n & 0x7FC0) == 0x7FC0) and np.array_equal(n >> 15, (d >> np.uint64(63)).astype(np.uint16))
    assert np.array_equal(n & 0x3F, ((d >> np.uint64(45)) & np.uint64(0x3F)).astype(np.uint16))


# ---------------------------------------------------------------- 8-bit floats -> F16, BF16, F32
# The two 8-bit formats (paper Section VI; layouts from the FP8 formats reference cited there): E5M2 =
# 1-5-2, bias 15, IEEE infinities and NaNs; E4M3 = 1-4-3, bias 7, no infinity, S.1111.111 is the NaN.
# All 256 inputs of each.  Independent references: torch's CPU float8 types; the value formula of the
# format evaluated on exact rationals; constants of the formats typed here; E5M2 = the upper byte of a
# binary16.

ALL8 = np.arange(256, dtype=np.uint8)
_F8 = {"F8_E5M2": (2, 15, torch.float8_e5m2), "F8_E4M3": (3, 7, torch.float8_e4m3fn)}


def _f8_is_nan(fmt):
    if fmt == "F8_E5M2":
        return ((ALL8 & 0x7C) == 0x7C) & ((ALL8 & 0x03) != 0)
    return (ALL8 & 0x7F) == 0x7F


@pytest.mark.parametrize("fmt", ["F8_E5M2", "F8_E4M3"])
def test_f8_widenings_exhaustive_vs_torch(fmt):
    nan = _f8_is_nan(fmt)
    t8 = torch.from_numpy(ALL8.copy()).view(_F8[fmt][2])
    for dst, tdt, view, npdt in (("F32", torch.float32, torch.int32, np.uint32), ("F16", torch.float16, torch.int16, np.uint16),
                                 ("BF16", torch.bfloat16, torch.int16, np.uint16)):
        got = orc.cast_array(ALL8, fmt, dst)
        ref = t8.to(tdt).view(view).numpy().view(npdt)
        assert np.array_equal(got[~nan], ref[~nan]), (fmt, dst)
        # the NaNs: NaN in the target, sign kept, quiet
        f = torch.from_numpy(got[nan].view(np.int32 if npdt is np.uint32 else np.int16)).view(tdt)
        assert bool(torch.isnan(f).all())
        top = got.dtype.itemsize * 8 - 1
        assert np.array_equal(got[nan] >> top, (ALL8[nan] >> 7).astype(got.dtype))


@pytest.mark.parametrize("fmt", ["F8_E5M2", "F8_E4M3"])
def test_f8_to_f32_vs_the_value_formula_on_rationals(fmt):
    from fractions import Fraction
    mb, bias, _ = _F8[fmt]
    nan = _f8_is_nan(fmt)
    got = orc.cast_array(ALL8, fmt, "F32").view(np.float32)
    emax = (1 << (7 - mb)) - 1
    for b in range(256):
        if nan[b]:
            continue
        s, e, m = b >> 7, (b >> mb) & emax, b & ((1 << mb) - 1)
        if fmt == "F8_E5M2" and e == emax:
            assert np.isinf(got[b]) and (got[b] < 0) == bool(s)
            continue
        if e == 0:
            v = Fraction(m, 1 << mb) * Fraction(2) ** (1 - bias)
        else:
            v = (1 + Fraction(m, 1 << mb)) * Fraction(2) ** (e - bias)
        assert Fraction(float(got[b])) == (-v if s else v), (fmt, b)
        assert np.signbit(got[b]) == bool(s)                     # -0 keeps its sign


def test_f8_constants():
    f32 = lambda fmt, b: float(orc.cast_array(np.array([b], np.uint8), fmt, "F32").view(np.float32)[0])
    bits = lambda fmt, b, dst: int(orc.cast_array(np.array([b], np.uint8), fmt, dst)[0])
    # E4M3: largest 448 = S.1111.110, smallest normal 2^-6, smallest subnormal 2^-9, no infinity
    assert f32("F8_E4M3", 0x7E) == 448.0 and f32("F8_E4M3", 0xFE) == -448.0
    assert f32("F8_E4M3", 0x78) == 256.0                        # exponent field all ones is an ordinary binade
    assert f32("F8_E4M3", 0x08) == 2.0 ** -6 and f32("F8_E4M3", 0x01) == 2.0 ** -9 and f32("F8_E4M3", 0x07) == 7 * 2.0 ** -9
    assert f32("F8_E4M3", 0x38) == 1.0 and f32("F8_E4M3", 0xC2) == -2.5 and f32("F8_E4M3", 0x39) == 1.125
    # E5M2: largest 57344 = S.11110.11, smallest normal 2^-14, smallest subnormal 2^-16, infinity S.11111.00
    assert f32("F8_E5M2", 0x7B) == 57344.0 and f32("F8_E5M2", 0x04) == 2.0 ** -14 and f32("F8_E5M2", 0x01) == 2.0 ** -16
    assert f32("F8_E5M2", 0x3C) == 1.0 and f32("F8_E5M2", 0xC1) == -2.5 and f32("F8_E5M2", 0x3D) == 1.25
    assert bits("F8_E5M2", 0x7C, "F32") == 0x7F800000 and bits("F8_E5M2", 0xFC, "F16") == 0xFC00
    assert bits("F8_E5M2", 0xFC, "BF16") == 0xFF80
    # bit patterns typed by hand
    assert bits("F8_E4M3", 0x38, "F16") == 0x3C00 and bits("F8_E4M3", 0x38, "BF16") == 0x3F80
    assert bits("F8_E4M3", 0x01, "F16") == 0x1800 and bits("F8_E4M3", 0x01, "BF16") == 0x3B00       # 2^-9
    assert bits("F8_E4M3", 0x7E, "F16") == 0x5F00 and bits("F8_E4M3", 0x7E, "BF16") == 0x43E0       # 448
    assert bits("F8_E5M2", 0x01, "F16") == 0x0100 and bits("F8_E5M2", 0x01, "BF16") == 0x3780       # 2^-16: subnormal in F16
    assert bits("F8_E5M2", 0x80, "F32") == 0x80000000 and bits("F8_E4M3", 0x80, "F16") == 0x8000    # -0
    # NaN rule: sign kept, mantissa field in the leading mantissa bits, quiet bit set
    assert bits("F8_E5M2", 0x7D, "F32") == 0x7FE00000 and bits("F8_E5M2", 0xFE, "F32") == 0xFFC00000
    assert bits("F8_E5M2", 0x7F, "F16") == 0x7F00 and bits("F8_E5M2", 0x7D, "BF16") == 0x7FE0
    assert bits("F8_E4M3", 0x7F, "F32") == 0x7FF00000 and bits("F8_E4M3", 0xFF, "F16") == 0xFF80
    assert bits("F8_E4M3", 0x7F, "BF16") == 0x7FF0


def test_f8_e5m2_is_the_upper_byte_of_binary16():
    got = orc.cast_array(ALL8, "F8_E5M2", "F16")
    nan = _f8_is_nan("F8_E5M2")
    assert np.array_equal(got[~nan], ALL8[~nan].astype(np.uint16) << 8)
    assert np.array_equal(orc.cast_array(ALL8, "F8_E5M2", "F32"),
                          orc.cast_array((ALL8.astype(np.uint16) << 8), "F16", "F32"))


@pytest.mark.parametrize("fmt", ["F8_E5M2", "F8_E4M3"])
def test_f8_widenings_agree_with_each_other_and_keep_order(fmt):
    f32 = orc.cast_array(ALL8, fmt, "F32")
    assert np.array_equal(orc.cast_array(orc.cast_array(ALL8, fmt, "F16"), "F16", "F32"), f32)
    assert np.array_equal(orc.cast_array(orc.cast_array(ALL8, fmt, "BF16"), "BF16", "F32"), f32)
    top = 0x7C if fmt == "F8_E5M2" else 0x7E                     # largest finite pattern
    v = f32[:top + 1].view(np.float32)
    assert np.all(np.diff(v) > 0)                               # positive patterns ascend strictly
    assert np.array_equal(f32[128:], f32[:128] | np.uint32(0x80000000))
