"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit
(paper Section III-B: alignment fix, type conversion and partition on the GPU)."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2505_23072_amd import binding as B
from paper_2505_23072_amd import device
from synth import writer
from util_cases import FLOATS, cast_targets, make_file, random_bits, random_request
from util_gpu import (first_diff, headers_of, materialize_packed, materialize_resident, materialize_slots,
                      oracle_outputs, upload_resident)

pytestmark = pytest.mark.gpu


def _check(got, want, names, reqs, tag=""):
    for i, (g, w) in enumerate(zip(got, want)):
        assert g == w, f"{tag} output {i} {names[i]} {reqs[i]}: {first_diff(g, w)}"


@pytest.mark.parametrize("seed", range(10))
def test_random_files(seed):
    rng = np.random.default_rng(1000 + seed)
    world = int(rng.choice([1, 2, 4, 8]))
    rank = int(rng.integers(world))
    blobs, names, reqs = [], [], []
    for f in range(int(rng.integers(1, 4))):
        blob, ts = make_file(rng, n_tensors=8, big=True, prefix=f"f{f}.")
        blobs.append(blob)
        names += [n for n, _, _ in ts]
        reqs += [random_request(rng, d, s, world) for _, d, s in ts]
    print(f"seed {seed} world {world} rank {rank} files {[len(b) for b in blobs]}", flush=True)
    want = oracle_outputs(blobs, names, reqs, rank, world)
    got, plan = materialize_resident(blobs, names, reqs, rank, world)
    _check(got, want, names, reqs, "all-groups")
    got, _ = materialize_resident(blobs, names, reqs, rank, world, max_group_bytes=8192, per_group=True)
    _check(got, want, names, reqs, "per-group")
    got, _ = materialize_slots(blobs, names, reqs, rank, world, 16384)
    _check(got, want, names, reqs, "slots")
    # only the byte ranges the requests read are present (0xDD elsewhere / packed extents in the slot)
    got, _ = materialize_resident(blobs, names, reqs, rank, world, max_group_bytes=0, min_gap_bytes=0)
    _check(got, want, names, reqs, "sparse resident")
    got, _ = materialize_slots(blobs, names, reqs, rank, world, 32768, min_gap_bytes=300)
    _check(got, want, names, reqs, "sparse slots")
    # strided shares staged as their row segments back to back (every segment of at least 2 / 64 bytes)
    got, _ = materialize_slots(blobs, names, reqs, rank, world, 16384, min_gap_bytes=300, min_segment_bytes=2)
    _check(got, want, names, reqs, "compacted slots")
    got, plan = materialize_packed(blobs, names, reqs, rank, world, 1 << 16, min_gap_bytes=0, min_segment_bytes=64)
    _check(got, want, names, reqs, "compacted, packed")
    assert plan.packed_bytes() == sum(plan.group(g)["slot_bytes"] for g in range(plan.group_count()))
    got, _ = materialize_packed(blobs, names, reqs, rank, world)
    _check(got, want, names, reqs, "packed, one group per file")
    # the files shifted in device memory: tensor data on a 256-byte boundary, and an arbitrary phase per file
    for phases in ("aligned", [int(x) for x in rng.integers(0, 256, len(blobs))]):
        got, _ = materialize_resident(blobs, names, reqs, rank, world, phases=phases)
        _check(got, want, names, reqs, f"all-groups, phases {phases}")
        got, _ = materialize_resident(blobs, names, reqs, rank, world, max_group_bytes=0, min_gap_bytes=0, phases=phases)
        _check(got, want, names, reqs, f"sparse resident, phases {phases}")
        got, _ = materialize_slots(blobs, names, reqs, rank, world, 16384, min_gap_bytes=300, min_segment_bytes=2, phases=phases)
        _check(got, want, names, reqs, f"compacted slots, phases {phases}")
        got, _ = materialize_packed(blobs, names, reqs, rank, world, 1 << 16, min_gap_bytes=0, min_segment_bytes=64, phases=phases)
        _check(got, want, names, reqs, f"compacted, packed, phases {phases}")


# several tiles (a tile is 16 KiB of output) and a ragged tail
SHAPE = (523, 264)


@pytest.mark.parametrize("residue", range(16))
def test_every_source_alignment(residue):
    """Body start at every residue mod 16, with an odd-sized tensor in front to shift the rest by one."""
    rng = np.random.default_rng(residue)
    ts = [("pad", "U8", (residue % 3,), random_bits(rng, "U8", (residue % 3,)).tobytes())]
    for dt in ("BF16", "F16", "F32", "F64", "I8", "I64", "F8_E4M3", "F8_E5M2"):
        ts.append((f"w.{dt}", dt, SHAPE, random_bits(rng, dt, SHAPE).tobytes()))
        ts.append((f"v.{dt}", dt, (1031,), random_bits(rng, dt, (1031,)).tobytes()))
    blob = writer.write_file(None, ts, None, residue)
    names, reqs = [], []
    for n, dt, shape, _ in ts[1:]:
        for dst in [None] + cast_targets(dt):
            for dim, blocks in ((-1, 1), (0, 1), (1, 1)) if len(shape) == 2 else ((-1, 1),):
                names.append(n)
                reqs.append((dst, dim, blocks))
    print(f"residue {residue}: {len(names)} requests", flush=True)
    # world 1 for every request (vectors included); the matrices get a real split below
    want = oracle_outputs([blob], names, reqs, 0, 1)
    got, _ = materialize_resident([blob], names, reqs, 0, 1)
    _check(got, want, names, reqs, "world 1")
    mats = [(n, r) for n, r in zip(names, reqs) if n.startswith("w.")]
    mn, mr = [n for n, _ in mats], [r for _, r in mats]
    # 523 rows do not split; use the 264 columns (dim 1) for world 8/3 and a blocked dim 0 elsewhere
    mr1 = [(dst, 1, 1) for dst, _, _ in mr]
    for world, rank in ((8, 5), (3, 1)):
        want = oracle_outputs([blob], mn, mr1, rank, world)
        got, _ = materialize_resident([blob], mn, mr1, rank, world)
        _check(got, want, mn, mr1, f"world {world}")


def test_blocked_and_ragged_rows():
    """Fused-QKV style blocked split, rows whose byte length is not a multiple of 16, 3-D and 4-D."""
    rng = np.random.default_rng(77)
    ts = [("odd", "I8", (5,), random_bits(rng, "I8", (5,)).tobytes()),
          ("qkv", "BF16", (3 * 8 * 40, 72), random_bits(rng, "BF16", (960, 72)).tobytes()),
          ("qkv_b", "F16", (960,), random_bits(rng, "F16", (960,)).tobytes()),
          ("ragged", "BF16", (64, 37), random_bits(rng, "BF16", (64, 37)).tobytes()),
          ("ragged8", "I8", (40, 63), random_bits(rng, "I8", (40, 63)).tobytes()),
          ("t3", "F32", (6, 16, 24), random_bits(rng, "F32", (6, 16, 24)).tobytes()),
          ("t4", "F16", (2, 3, 8, 40), random_bits(rng, "F16", (2, 3, 8, 40)).tobytes())]
    blob = writer.write_file(None, ts, None, 7)
    for world in (1, 2, 4, 8):
        names = ["qkv", "qkv", "qkv_b", "qkv_b", "t3", "t3", "t3", "t4", "t4", "t4", "odd"]
        reqs = [(None, 0, 3), ("F16", 0, 3), (None, 0, 3), ("F32", 0, 3), ("BF16", 1, 1), (None, 2, 1),
                ("F16", 0, 1) if 6 % world == 0 else ("F16", -1, 1),
                (None, 2, 1), ("BF16", 3, 1), ("F32", 2, 1), (None, -1, 1)]
        if world == 1:
            names += ["ragged", "ragged8"]
            reqs += [("F32", 1, 1), (None, 1, 1)]
        for rank in sorted({0, world - 1}):
            print(f"world {world} rank {rank}", flush=True)
            want = oracle_outputs([blob], names, reqs, rank, world)
            got, _ = materialize_resident([blob], names, reqs, rank, world)
            _check(got, want, names, reqs, f"world {world} rank {rank}")
    # rows of 37 two-byte / 63 one-byte elements split by a world that divides them: row pieces of
    # 2, 9 and 7 bytes, none a multiple of 16
    for world, rank, name, req in ((37, 11, "ragged", (None, 1, 1)), (37, 36, "ragged", ("F32", 1, 1)),
                                   (7, 3, "ragged8", (None, 1, 1)), (9, 8, "ragged8", (None, 1, 1)),
                                   (8, 3, "ragged8", (None, 0, 1))):
        want = oracle_outputs([blob], [name], [req], rank, world)
        got, _ = materialize_resident([blob], [name], [req], rank, world)
        _check(got, want, [name], [req], f"ragged world {world}")


def test_hand_derived_partitions_and_conversions():
    """The kernels against results worked out by hand (tests/golden/handmade_partition.txt): one plan
    per request, and all requests of a (rank, world) pair in one plan."""
    from util_golden import load_fixture
    g = load_fixture("handmade_partition.txt")
    blob = g["file"]
    for nm, dst, dim, blocks, rank, world, shape, want in g["parts"]:
        got, plan = materialize_resident([blob], [nm], [(dst, dim, blocks)], rank, world)
        assert plan.output(0)["shape"] == shape and got == [want], (nm, dst, dim, blocks, rank, world)
    names = [p[0] for p in g["parts"]]
    reqs = [(p[1], p[2], p[3], p[4]) for p in g["parts"]]
    worlds = sorted({p[5] for p in g["parts"]})
    for world in worlds:
        sel = [i for i, p in enumerate(g["parts"]) if p[5] == world]
        got, _ = materialize_resident([blob], [names[i] for i in sel], [reqs[i] for i in sel], 0, world)
        assert got == [g["parts"][i][7] for i in sel], f"world {world}"


@pytest.mark.parametrize("residue", [0, 1, 2, 7, 12])
def test_ragged_rows_of_at_least_one_chunk(residue):
    """Shares whose row segments are not a multiple of 16 bytes (274, 44, 25, 18, 420, 550 and 740 bytes):
    chunks of the output stream that straddle a row end are spliced from two rows.  Several tiles, tails
    of one element, every conversion, first and last rank."""
    rng = np.random.default_rng(300 + residue)
    spec = [("a", "BF16", (300, 1096), 8), ("b", "F32", (200, 44), 4), ("c", "I8", (300, 100), 4),
            ("d", "F16", (129, 72), 8), ("e", "BF16", (6, 50, 21), 5), ("f", "BF16", (4099, 1100), 4),
            ("g", "F32", (1031, 72), 8), ("h", "F64", (300, 44), 4), ("i", "F64", (129, 40), 8),
            ("m", "F8_E4M3", (300, 100), 4), ("n", "F8_E5M2", (129, 72), 8)]
    ts = [("lead", "U8", (residue % 3,), bytes(residue % 3))]
    ts += [(n, dt, shape, random_bits(rng, dt, shape).tobytes()) for n, dt, shape, _ in spec]
    ts.append(("qkv", "BF16", (120, 37), random_bits(rng, "BF16", (120, 37)).tobytes()))
    blob = writer.write_file(None, ts, None, residue)
    for world in (4, 5, 8):
        names, reqs = [], []
        for n, dt, shape, w in spec:
            if w != world:
                continue
            for dst in [None] + cast_targets(dt):
                names.append(n)
                reqs.append((dst, 1, 1))
        if world == 4:
            names += ["qkv", "qkv"]
            reqs += [(None, 0, 3), ("F32", 0, 3)]
        for rank in (0, world - 1):
            print(f"residue {residue} world {world} rank {rank}: {len(names)} requests", flush=True)
            want = oracle_outputs([blob], names, reqs, rank, world)
            got, _ = materialize_resident([blob], names, reqs, rank, world)
            _check(got, want, names, reqs, f"world {world} rank {rank}")
            got, _ = materialize_slots([blob], names, reqs, rank, world, 1 << 20)
            _check(got, want, names, reqs, f"slots world {world} rank {rank}")
            # groups cut between ragged rows: pieces that start off a 16-byte boundary of their output
            got, plan = materialize_resident([blob], names, reqs, rank, world, max_group_bytes=40000, per_group=True)
            _check(got, want, names, reqs, f"groups of 40000 bytes, world {world} rank {rank}")
            got, _ = materialize_packed([blob], names, reqs, rank, world, 40000, min_gap_bytes=1 << 20, min_segment_bytes=16)
            _check(got, want, names, reqs, f"compacted groups of 40000 bytes, world {world} rank {rank}")


@pytest.mark.parametrize("src,dst", [("F16", "BF16"), ("BF16", "F16"), ("F16", "F32"), ("BF16", "F32")])
def test_exhaustive_16bit_conversions_on_device(src, dst):
    """All 65536 source patterns, NaN payloads and subnormals included, at an odd source offset too."""
    allbits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    for lead in (0, 1, 2):
        ts = [("lead", "U8", (lead,), bytes(lead)), ("x", src, (1 << 16,), allbits.tobytes())]
        blob = writer.write_file(None, ts, None, 0)
        got, _ = materialize_resident([blob], ["x"], [(dst, -1, 1)])
        want = orc.cast_array(allbits, src, dst).tobytes()
        assert got[0] == want, f"{src}->{dst} lead {lead}: {first_diff(got[0], want)}"


@pytest.mark.parametrize("src", ["F8_E5M2", "F8_E4M3"])
def test_8bit_float_widenings_on_device(src):
    """All 256 patterns of an 8-bit float to F16, BF16 and F32: in order (chunks that hold NaNs or infinities
    take the integer formulation), every finite pattern eight times in a row (chunks without any take the
    other one), random bytes over several tiles; sources at every offset modulo 4."""
    rng = np.random.default_rng(8)
    allbits = np.arange(256, dtype=np.uint8)
    special = ((allbits & 0x7C) == 0x7C) if src == "F8_E5M2" else ((allbits & 0x7F) == 0x7F)
    x = np.concatenate([allbits, np.repeat(allbits[~special], 8), rng.integers(0, 256, 70_001, dtype=np.uint8)])
    for lead in (0, 1, 2, 3):
        ts = [("lead", "U8", (lead,), bytes(lead)), ("x", src, (len(x),), x.tobytes())]
        blob = writer.write_file(None, ts, None, 0)
        dsts = ["F16", "BF16", "F32"]
        got, _ = materialize_resident([blob], ["x"] * 3, [(d, -1, 1) for d in dsts])
        for d, g in zip(dsts, got):
            want = orc.cast_array(x, src, d).tobytes()
            assert g == want, f"{src}->{d} lead {lead}: {first_diff(g, want)}"


@pytest.mark.parametrize("dst", ["BF16", "F16"])
def test_f32_conversions_on_device(dst):
    rng = np.random.default_rng(5)
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    parts = [hi | lo for lo in (0x0000, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x0001)]
    hi13 = np.arange(1 << 19, dtype=np.uint32) << 13
    parts += [hi13 | lo for lo in (0x0000, 0x0FFF, 0x1000, 0x1001, 0x1FFF)]
    sub = np.uint32(0x33000000) + np.arange(0, 0x05800000, 0x3FF, dtype=np.uint32)
    parts += [sub, sub | np.uint32(0x80000000), rng.integers(0, 1 << 32, 2_000_000, dtype=np.uint64).astype(np.uint32)]
    x = np.concatenate(parts)
    for lead in (0, 3):
        blob = writer.write_file(None, [("lead", "U8", (lead,), bytes(lead)), ("x", "F32", (len(x),), x.tobytes())], None, 0)
        got, _ = materialize_resident([blob], ["x"], [(dst, -1, 1)])
        want = orc.cast_array(x, "F32", dst).tobytes()
        assert got[0] == want, f"F32->{dst} lead {lead}: {first_diff(got[0], want)}"


@pytest.mark.parametrize("residue", [0, 1, 2, 4, 13])
def test_rows_shorter_than_a_chunk(residue):
    """Partitions whose row segments are shorter than one chunk (1 to 15 bytes when copying, 1 to 7 elements when
    converting): every chunk of the output is gathered from several rows.  Segment lengths and strides with
    every power-of-two alignment (the kernel loads 4, 2 or 1 bytes at a time accordingly), several tiles,
    every conversion, groups cut between rows."""
    rng = np.random.default_rng(500 + residue)
    # (name, dtype, shape, world): the share along the last dimension is shape[-1] / world elements
    spec = [("a", "U8", (5000, 24), 8), ("b", "U8", (3001, 26), 2), ("c", "I16", (4100, 12), 4), ("d", "BF16", (2900, 8), 8),
            ("e", "F32", (1500, 6), 2), ("f", "F16", (2050, 14), 2), ("g", "F64", (900, 6), 2), ("h", "I64", (700, 2), 2),
            ("i", "BF16", (33, 7, 10), 5), ("j", "F32", (1100, 9), 3), ("k", "U8", (2000, 30), 2), ("l", "F64", (1200, 3), 3),
            ("m", "F8_E4M3", (3000, 12), 4), ("n", "F8_E5M2", (1000, 14), 2)]
    ts = [("lead", "U8", (residue % 3,), bytes(residue % 3))]
    ts += [(n, dt, shape, random_bits(rng, dt, shape).tobytes()) for n, dt, shape, _ in spec]
    blob = writer.write_file(None, ts, None, residue)
    for world in (2, 3, 4, 5, 8):
        names, reqs = [], []
        for n, dt, shape, w in spec:
            if w != world:
                continue
            for dst in [None] + cast_targets(dt):
                names.append(n)
                reqs.append((dst, len(shape) - 1, 1))
        for rank in sorted({0, world - 1}):
            print(f"residue {residue} world {world} rank {rank}: {len(names)} requests", flush=True)
            want = oracle_outputs([blob], names, reqs, rank, world)
            got, _ = materialize_resident([blob], names, reqs, rank, world)
            _check(got, want, names, reqs, f"world {world} rank {rank}")
            got, _ = materialize_resident([blob], names, reqs, rank, world, max_group_bytes=30000, per_group=True)
            _check(got, want, names, reqs, f"groups of 30000 bytes, world {world} rank {rank}")
            got, _ = materialize_slots([blob], names, reqs, rank, world, 1 << 20, min_gap_bytes=0)
            _check(got, want, names, reqs, f"slots world {world} rank {rank}")


def _f64_inputs_for_16bit(fmt):
    """binary64 inputs around every rounding decision of a 16-bit format: for every pair of neighbouring
    finite values their midpoint and the binary64 numbers next to it, exponents over and beyond the format's
    range with the low mantissa bits cleared in a third of them, random patterns (NaNs included)."""
    mb, bias = (10, 15) if fmt == "F16" else (7, 127)
    rng = np.random.default_rng(17)
    top = 0x7C00 if fmt == "F16" else 0x7F80
    lo = np.arange(0, top - 1, dtype=np.uint16)
    a = orc.cast_array(lo, fmt, "F64").view(np.float64)
    b = orc.cast_array(lo + np.uint16(1), fmt, "F64").view(np.float64)
    mid = (a + b) / 2
    ties = np.concatenate([np.nextafter(mid, -np.inf), mid, np.nextafter(mid, np.inf)])
    n = 1_000_000
    e = rng.integers(1023 - bias - mb - 4, 1023 + bias + 4, n, dtype=np.uint64)
    m = rng.integers(0, 1 << 52, n, dtype=np.uint64)
    keep = rng.integers(52 - mb - 2, 53, n, dtype=np.uint64)
    m = np.where(rng.random(n) < 0.33, (m >> keep) << keep, m)
    sign = rng.integers(0, 2, n, dtype=np.uint64) << np.uint64(63)
    return np.concatenate([ties.view(np.uint64), (-ties).view(np.uint64), sign | (e << np.uint64(52)) | m,
                           rng.integers(0, 1 << 64, 500_000, dtype=np.uint64)])


@pytest.mark.parametrize("fmt", ["F16", "BF16"])
def test_binary64_and_16bit_conversions_on_device(fmt):
    """binary64 -> binary16 / bfloat16 (one rounding from 53 bits) around every tie of the target format, and
    the exact widenings of all 65536 patterns; sources at an aligned and at an odd offset."""
    d = _f64_inputs_for_16bit(fmt)
    allbits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    print(f"{len(d)} binary64 inputs", flush=True)
    want_d = orc.cast_array(d, "F64", fmt).tobytes()
    want_w = orc.cast_array(allbits, fmt, "F64").tobytes()
    for lead in (0, 3):
        ts = [("lead", "U8", (lead,), bytes(lead)), ("d", "F64", (len(d),), d.tobytes()),
              ("w", fmt, (1 << 16,), allbits.tobytes())]
        blob = writer.write_file(None, ts, None, 0)
        got, _ = materialize_resident([blob], ["d", "w"], [(fmt, -1, 1), ("F64", -1, 1)])
        assert got[0] == want_d, f"F64->{fmt} lead {lead}: {first_diff(got[0], want_d)}"
        assert got[1] == want_w, f"{fmt}->F64 lead {lead}: {first_diff(got[1], want_w)}"


def test_binary64_conversions_on_device():
    """binary64 -> binary32 on inputs around everything the rounding can meet (every 509th binary32 value
    widened, its midpoints to the neighbours and the values next to those, the subnormal zone with its
    ties, the overflow zone, random patterns with NaNs), and binary32 -> binary64 on a stride of all
    binary32 patterns plus all subnormals; sources at an aligned and at an odd offset."""
    rng = np.random.default_rng(6)
    b = np.arange(0, 1 << 32, 509, dtype=np.uint64).astype(np.uint32)
    w = orc.cast_array(b[(b & 0x7FFFFFFF) < 0x7F800000], "F32", "F64")
    parts = [w, w + np.uint64(1 << 28), w + np.uint64((1 << 28) - 1), w + np.uint64((1 << 28) + 1), w + np.uint64(1),
             w - np.uint64(1), rng.integers(0, 1 << 64, 3_000_000, dtype=np.uint64)]
    e = rng.integers(860, 900, 1_000_000, dtype=np.uint64)
    z = (e << np.uint64(52)) | rng.integers(0, 1 << 52, 1_000_000, dtype=np.uint64)
    parts += [z, z | np.uint64(1 << 63), (np.arange(1, 1 << 20, dtype=np.uint64) << np.uint64(28)) + np.uint64(0x3690000000000000)]
    e = rng.integers(1023 + 120, 1023 + 130, 300_000, dtype=np.uint64)
    parts.append((e << np.uint64(52)) | rng.integers(0, 1 << 52, 300_000, dtype=np.uint64))
    d = np.concatenate(parts)
    x = np.concatenate([np.arange(0, 1 << 32, 61, dtype=np.uint64).astype(np.uint32), np.arange(0, 0x00800000, dtype=np.uint32),
                        np.arange(0x7F000000, 0x80000000, 5, dtype=np.uint32)])
    print(f"{len(d)} binary64 inputs, {len(x)} binary32 inputs", flush=True)
    for lead in (0, 3):
        ts = [("lead", "U8", (lead,), bytes(lead)), ("d", "F64", (len(d),), d.tobytes()), ("x", "F32", (len(x),), x.tobytes())]
        blob = writer.write_file(None, ts, None, 0)
        got, _ = materialize_resident([blob], ["d", "x"], [("F32", -1, 1), ("F64", -1, 1)])
        want_d = orc.cast_array(d, "F64", "F32").tobytes()
        want_x = orc.cast_array(x, "F32", "F64").tobytes()
        assert got[0] == want_d, f"F64->F32 lead {lead}: {first_diff(got[0], want_d)}"
        assert got[1] == want_x, f"F32->F64 lead {lead}: {first_diff(got[1], want_x)}"


@pytest.mark.parametrize("dst", ["BF16", "F16"])
def test_every_binary32_pattern_on_device(dst):
    """All 2^32 binary32 inputs, in slabs of 2^27, the source one byte off dword alignment in every
    other slab.  The oracle side runs on a thread pool (its conversion is a plain C loop) and is itself
    compared with torch's CPU conversion on every input that is not a NaN (numpy's binary16 conversion,
    a second library, pins it on a sample in the CPU tests; over 2^32 inputs it would take minutes)."""
    from concurrent.futures import ThreadPoolExecutor

    from synth import writer as w
    n = 1 << 27
    workers = 16
    step = n // workers
    with ThreadPoolExecutor(workers) as pool:
        for slab in range(32):
            lead = slab & 1
            x = np.arange(slab * n, (slab + 1) * n, dtype=np.uint64).astype(np.uint32)
            head, _ = w.build_header([("lead", "U8", (lead,), lead), ("x", "F32", (n,), 4 * n)], None, 0)
            want = pool.map(lambda k: orc.cast_array(x[k * step:(k + 1) * step], "F32", dst), range(workers))
            size = len(head) + lead + 4 * n
            raw = device.device_bytes(size + 256)
            raw[:len(head) + lead].copy_(torch.from_numpy(np.frombuffer(head + bytes(lead), np.uint8).copy()))
            raw[len(head) + lead:size].copy_(torch.from_numpy(x.view(np.uint8)))
            plan = B.Plan([B.Header(head, size)], [0], ["x"], [(dst, -1, 1)], 0, 1)
            bufs, ptrs = device.alloc_outputs(plan)
            ws = device.device_bytes(plan.workspace_bytes())
            B.fst_materialize(raw.data_ptr(), size, plan, B.FST_ALL_GROUPS, ptrs, ws.data_ptr(), ws.numel(), 0)
            torch.cuda.synchronize()
            got = bufs[0][:2 * n].cpu().numpy().view(np.uint16)
            want = np.concatenate(list(want))
            # the oracle itself against torch's CPU conversion on every non-NaN input
            finite = (x & np.uint32(0x7FFFFFFF)) <= np.uint32(0x7F800000)
            tdt = torch.float16 if dst == "F16" else torch.bfloat16
            lib_bits = torch.from_numpy(x.view(np.float32)).to(tdt).view(torch.int16).numpy().view(np.uint16)
            off = np.nonzero((lib_bits != want) & finite)[0]
            assert len(off) == 0, f"oracle F32->{dst} differs from the library conversion at input {int(x[off[0]]):#010x}"
            bad = np.nonzero(got != want)[0]
            assert len(bad) == 0, (f"F32->{dst} slab {slab}: {len(bad)} differ, first input {int(x[bad[0]]):#010x} "
                                   f"got {int(got[bad[0]]):#06x} want {int(want[bad[0]]):#06x}")
            plan.close()
            if slab % 8 == 7:
                print(f"F32->{dst}: {slab + 1}/32 slabs equal", flush=True)


def test_all_ranks_in_one_pass():
    """Every rank's share of every tensor from one plan and one launch set (per-request rank)."""
    rng = np.random.default_rng(21)
    ts = [("q", "BF16", (512, 264), random_bits(rng, "BF16", (512, 264)).tobytes()),
          ("o", "F16", (264, 512), random_bits(rng, "F16", (264, 512)).tobytes()),
          ("qkv", "BF16", (3 * 128, 72), random_bits(rng, "BF16", (384, 72)).tobytes()),
          ("norm", "BF16", (264,), random_bits(rng, "BF16", (264,)).tobytes())]
    blob = writer.write_file(None, ts, None, 13)
    world = 8
    names, reqs = ["norm"], [("F32", -1, 1)]
    for r in range(world):
        names += ["q", "o", "qkv"]
        reqs += [(None, 0, 1, r), ("BF16", 1, 1, r), ("F32", 0, 3, r)]
    want = oracle_outputs([blob], names, reqs, 0, world)
    got, plan = materialize_resident([blob], names, reqs, 0, world)
    _check(got, want, names, reqs, "all ranks")
    assert b"".join(got[1 + 3 * r] for r in range(world)) == ts[0][3]       # q shares = stored q
    assert plan.read_bytes() == sum(len(t[3]) for t in ts)                    # every stored byte read once


def test_on_a_side_stream_and_empty_plan():
    rng = np.random.default_rng(3)
    blob, ts = make_file(rng, n_tensors=6, big=True)
    names = [n for n, _, _ in ts]
    reqs = [(None, -1, 1)] * len(names)
    s = torch.cuda.Stream()
    got, plan = materialize_resident([blob], names, reqs, stream=s)
    _check(got, oracle_outputs([blob], names, reqs), names, reqs, "side stream")
    # a plan whose outputs are all empty launches nothing
    e = writer.write_file(None, [("e", "F32", (0, 4), b""), ("f", "F16", (3, 0), b"")])
    got, plan = materialize_resident([e], ["e", "f"], [(None, -1, 1), ("F32", -1, 1)])
    assert got == [b"", b""] and plan.group_count() == 0

def test_thousands_of_small_tensors():
    """6000 tensors of 1 element .. 3 tiles, in four dtypes, a third of them converted: hint spans that hold
    dozens of pieces each, in every launch class, found by the bounded binary search."""
    rng = np.random.default_rng(55)
    ts, names, reqs = [], [], []
    for i in range(6000):
        dt = ("U8", "BF16", "F16", "F32")[int(rng.integers(4))]
        n = int(rng.integers(1, 2000)) if rng.random() < 0.9 else int(rng.integers(2000, 30000))
        ts.append((f"t{i}", dt, (n,), random_bits(rng, dt, (n,)).tobytes()))
        names.append(f"t{i}")
        targets = cast_targets(dt)
        reqs.append((targets[int(rng.integers(len(targets)))] if targets and rng.random() < 0.35 else None, -1, 1))
    blob = writer.write_file(None, ts, None, 5)
    want = oracle_outputs([blob], names, reqs)
    got, plan = materialize_resident([blob], names, reqs)
    _check(got, want, names, reqs, "one launch set")
    got, _ = materialize_resident([blob], names, reqs, max_group_bytes=1 << 20, per_group=True)
    _check(got, want, names, reqs, "groups of 1 MiB")


def test_degenerate_requests():
    """The corners of the request space: eight dimensions split on the first, a middle and the last one;
    as many ranks as the dimension has indices; one rank (the share is the whole tensor) with and without
    blocks; tensors with a zero dimension, split or not; scalars; a one-element tensor."""
    rng = np.random.default_rng(31)
    t8 = (2, 3, 2, 4, 2, 3, 2, 8)
    ts = [("lead", "U8", (1,), b"\x07"),
          ("t8", "BF16", t8, random_bits(rng, "BF16", t8).tobytes()),
          ("m", "F32", (12, 40), random_bits(rng, "F32", (12, 40)).tobytes()),
          ("z0", "F16", (0, 16), b""), ("z1", "F16", (16, 0), b""), ("z2", "I32", (4, 0, 8), b""),
          ("s", "F32", (), random_bits(rng, "F32", ()).tobytes()),
          ("one", "BF16", (1,), random_bits(rng, "BF16", (1,)).tobytes()),
          ("one2", "F64", (1, 1), random_bits(rng, "F64", (1, 1)).tobytes())]
    blob = writer.write_file(None, ts, None, 11)
    cases = [
        (2, 1, ["t8", "t8", "t8", "t8"], [(None, 0, 1), ("F16", 2, 1), ("F32", 4, 1), (None, 6, 1)]),
        (4, 3, ["t8", "t8"], [(None, 3, 1), ("F32", 7, 1)]),
        (8, 7, ["t8", "m"], [("F16", 7, 1), ("F64", 1, 1)]),                      # one index of dim 7 per rank
        (12, 11, ["m", "m"], [(None, 0, 1), ("BF16", 0, 1)]),                     # one row per rank
        (1, 0, ["m", "m", "m", "t8"], [(None, 0, 1), ("F16", 1, 1), (None, 0, 3), ("F32", 0, 2)]),   # one rank
        (4, 2, ["z0", "z1", "z1", "z2", "z2", "s", "one", "one2"],
         [(None, 1, 1), ("F32", 0, 1), (None, -1, 1), (None, 0, 1), (None, 2, 1), ("BF16", -1, 1), ("F32", -1, 1), ("F32", -1, 1)]),
    ]
    for world, rank, names, reqs in cases:
        print(f"world {world} rank {rank}: {list(zip(names, reqs))}", flush=True)
        want = oracle_outputs([blob], names, reqs, rank, world)
        got, plan = materialize_resident([blob], names, reqs, rank, world)
        _check(got, want, names, reqs, f"world {world} rank {rank}")
        got, _ = materialize_slots([blob], names, reqs, rank, world, 4096)
        _check(got, want, names, reqs, f"slots world {world} rank {rank}")


def test_prepare_once_launch_on_two_source_buffers():
    """The table is uploaded once; the kernels are then launched on two raw buffers of the same layout
    and different content, and once more per group after re-preparing group by group."""
    rng = np.random.default_rng(9)
    ts = [("pad", "U8", (3,), bytes(3)), ("w", "BF16", (520, 264), None), ("h", "F16", (264, 520), None),
          ("v", "F32", (1031,), None)]
    blobs = []
    for k in range(2):
        full = [(n, d, s, b if b is not None else random_bits(rng, d, s).tobytes()) for n, d, s, b in ts]
        blobs.append(writer.write_file(None, full, None, 5))
    names, reqs = ["w", "w", "h", "h", "v"], [(None, 0, 1), ("F16", 1, 1), ("F32", 0, 2), ("BF16", 1, 1), ("BF16", -1, 1)]
    world, rank = 4, 2
    hs = headers_of(blobs[:1])
    plan = B.Plan(hs, [0], names, reqs, rank, world)
    raws = [upload_resident([b]) for b in blobs]
    raw_len = raws[0][2]
    bufs, ptrs = device.alloc_outputs(plan)
    ws = device.device_bytes(plan.workspace_bytes())
    with pytest.raises(B.FstError) as e:
        B.fst_launch(plan, B.FST_ALL_GROUPS, raws[0][0].data_ptr(), raw_len, 0)
    assert e.value.name == "FST_E_ARG"
    B.fst_prepare(plan, B.FST_ALL_GROUPS, B.FST_LAYOUT_RESIDENT, raw_len, ptrs, ws.data_ptr(), ws.numel(), 0)
    with pytest.raises(B.FstError) as e:
        B.fst_launch(plan, B.FST_ALL_GROUPS, raws[0][0].data_ptr(), raw_len - 4, 0)
    assert e.value.name == "FST_E_RANGE"
    for k in (0, 1, 0):
        for b in bufs:
            b.fill_(0xC3)
        B.fst_launch(plan, B.FST_ALL_GROUPS, raws[k][0].data_ptr(), raw_len, 0)
        from util_gpu import fetch
        _check(fetch(bufs, plan), oracle_outputs([blobs[k]], names, reqs, rank, world), names, reqs, f"buffer {k}")
    # cut into small groups: each group prepared into its own part of a larger workspace, then launched
    ng = plan.set_groups(16384)
    assert ng > 3
    wss = [device.device_bytes(plan.workspace_bytes()) for _ in range(ng)]
    for b in bufs:
        b.fill_(0x3C)
    for g in range(ng):
        B.fst_prepare(plan, g, B.FST_LAYOUT_RESIDENT, raw_len, ptrs, wss[g].data_ptr(), wss[g].numel(), 0)
    for g in range(ng):
        B.fst_launch(plan, g, raws[1][0].data_ptr(), raw_len, 0)
    _check(fetch(bufs, plan), oracle_outputs([blobs[1]], names, reqs, rank, world), names, reqs, "per group")


def test_launch_half_replays_from_a_hip_graph():
    """fst_launch enqueues kernels only, so it can be recorded into a HIP graph once and replayed for every
    new set of raw bytes that lands in the same buffer (a checkpoint reloaded into place).  Eager work and
    synchronisations sit between the replays, and every replay is checked against the oracle."""
    rng = np.random.default_rng(12)
    shapes = [("w", "BF16", (520, 264)), ("h", "F16", (264, 520)), ("r", "BF16", (300, 1096)), ("v", "F32", (1031,))]
    names, reqs = ["w", "h", "h", "r", "v"], [(None, 0, 1), ("F32", 0, 2), ("BF16", 1, 1), ("F32", 1, 1), ("BF16", -1, 1)]
    world, rank = 4, 1
    blobs = [writer.write_file(None, [(n, d, s, random_bits(rng, d, s).tobytes()) for n, d, s in shapes], None, 3)
             for _ in range(3)]
    plan = B.Plan(headers_of(blobs[:1]), [0], names, reqs, rank, world)
    raw, _, raw_len = upload_resident(blobs[:1])
    bufs, ptrs = device.alloc_outputs(plan)
    ws = device.device_bytes(plan.workspace_bytes())
    s = torch.cuda.Stream()
    B.fst_prepare(plan, B.FST_ALL_GROUPS, B.FST_LAYOUT_RESIDENT, raw_len, ptrs, ws.data_ptr(), ws.numel(), s.cuda_stream)
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        B.fst_launch(plan, B.FST_ALL_GROUPS, raw.data_ptr(), raw_len, torch.cuda.current_stream().cuda_stream)
    from util_gpu import fetch
    for k in (1, 2, 0, 1):
        host = np.zeros(raw_len, np.uint8)
        host[:len(blobs[k])] = np.frombuffer(blobs[k], np.uint8)
        raw.copy_(torch.from_numpy(host))                   # eager work between the replays
        for b in bufs:
            b.fill_(0x77)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        _check(fetch(bufs, plan), oracle_outputs([blobs[k]], names, reqs, rank, world), names, reqs, f"replay of file {k}")


def test_operand_checks_reject_before_any_launch():
    rng = np.random.default_rng(4)
    blob, ts = make_file(rng, n_tensors=4, big=True)
    names = [n for n, _, shape in ts if int(np.prod(shape)) > 0]
    reqs = [(None, -1, 1)] * len(names)
    hs = headers_of([blob])
    raw, bases, raw_len = upload_resident([blob])
    plan = B.Plan(hs, bases, names, reqs)
    bufs, ptrs = device.alloc_outputs(plan)
    ws = device.device_bytes(plan.workspace_bytes())

    def err(**kw):
        a = dict(raw_ptr=raw.data_ptr(), raw_len=raw_len, group=B.FST_ALL_GROUPS, out_ptrs=ptrs,
                 workspace_ptr=ws.data_ptr(), workspace_len=ws.numel())
        a.update(kw)
        with pytest.raises(B.FstError) as e:
            B.fst_materialize(a["raw_ptr"], a["raw_len"], plan, a["group"], a["out_ptrs"], a["workspace_ptr"],
                              a["workspace_len"], 0)
        return e.value.name

    assert err(raw_ptr=raw.data_ptr() + 16) == "FST_E_ALIGN"
    assert err(out_ptrs=[ptrs[0] + 64] + ptrs[1:]) == "FST_E_ALIGN"
    assert err(out_ptrs=[0] + ptrs[1:]) == "FST_E_ARG"
    assert err(raw_len=len(blob) // 2) == "FST_E_RANGE"
    assert err(workspace_len=32) == "FST_E_RANGE"
    assert err(workspace_ptr=ws.data_ptr() + 8) == "FST_E_ALIGN"
    assert err(group=plan.group_count()) == "FST_E_RANGE"
    with pytest.raises(B.FstError):
        B.fst_materialize_slot(raw.data_ptr(), raw_len, plan, B.FST_ALL_GROUPS, ptrs, ws.data_ptr(), ws.numel(), 0)
    torch.cuda.synchronize()
