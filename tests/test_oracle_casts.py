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
    for s, d in (("I16", "F16"), ("F16", "F64"), ("F64", "BF16"), ("U8", "BOOL"), ("F8_E5M2", "F16"), ("I64", "F64")):
        with pytest.raises(orc.OracleError) as e:
            orc.cast_array(np.zeros(8, np.uint8), s, d)
        assert e.value.kind == "CAST"
