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


def test_identity_and_unsupported():
    x = np.arange(256, dtype=np.uint8)
    for dt in ("BOOL", "U8", "I8", "F8_E5M2", "F8_E4M3"):
        assert np.array_equal(orc.cast_array(x, dt, dt), x)
    assert np.array_equal(orc.cast_array(ALL16, "F16", "F16"), ALL16)     # NaN payloads untouched
    for s, d in (("I16", "F16"), ("F32", "F64"), ("F64", "F32"), ("U8", "BOOL"), ("F8_E5M2", "F16")):
        with pytest.raises(orc.OracleError) as e:
            orc.cast_array(np.zeros(8, np.uint8), s, d)
        assert e.value.kind == "CAST"
