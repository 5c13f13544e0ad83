"""Cases for the CPU build of the library in which kernel launches go to the table interpreter
(cpu_kernels.cpp): run by tests/test_host_tables.py in a child process with FST_LIBRARY pointing at that
build.  "Device" buffers are 256-byte aligned numpy arrays.  Every case compares the outputs with the oracle
and relies on the interpreter's bounds checks (a launch that would touch a byte outside the registered source
and output ranges fails)."""
import ctypes
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2505_23072_amd import binding as B
from synth import writer
from util_cases import cast_targets, make_file, random_bits, random_request

assert os.environ.get("FST_LIBRARY"), "run through tests/test_host_tables.py"
L = B.lib()
L.fst_test_set_source.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
L.fst_test_add_output.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
L.fst_test_first_violation.restype = ctypes.c_char_p
L.fst_test_violations.restype = ctypes.c_uint64
L.fst_test_direct_tiles.restype = ctypes.c_uint64
L.fst_test_staged_tiles.restype = ctypes.c_uint64


def aligned(n, fill):
    store = np.full(n + 512, fill, np.uint8)
    off = (-store.ctypes.data) % 256
    return store, store[off:off + n]


def headers_of(blobs):
    return [B.Header(bytes(b[:8 + B.fst_header_len(bytes(b[:8]))]), len(b)) for b in blobs]


def oracle_outputs(blobs, names, reqs, rank, world):
    tabs = [orc.parse(bytes(b), len(b)) for b in blobs]
    res = []
    for nm, rq in zip(names, reqs):
        dst, dim, blocks = rq[:3]
        r = rq[3] if len(rq) > 3 and rq[3] >= 0 else rank
        for b, tab in zip(blobs, tabs):
            hit = [t for t in tab.tensors if t.name == nm]
            if hit:
                t = hit[0]
                stored = np.frombuffer(b, np.uint8, t.end - t.begin, tab.body_off + t.begin)
                res.append(orc.materialize(stored, t.dtype, t.shape, dst, dim, blocks, r, world)[0].tobytes())
                break
    return res


def slot_image(gi, blobs):
    host = np.full(gi["slot_bytes"], 0xEE, np.uint8)
    data = np.frombuffer(blobs[gi["file"]], np.uint8)
    for (lo, hi, off), (row_bytes, n_rows, stride) in zip(gi["extents"], gi["extent_rows"]):
        for r in range(n_rows):
            host[off + r * row_bytes:off + (r + 1) * row_bytes] = data[lo + r * stride:lo + r * stride + row_bytes]
    return host


def run(blobs, names, reqs, rank, world, layout, max_group_bytes=0, min_gap=None, min_seg=None, per_group=False,
        phases=None):
    """phases: per file, where its bytes sit modulo 256 (None: at their file offsets' residues; "aligned": tensor
    data on a 256-byte boundary; or a list)."""
    hs = headers_of(blobs)
    sizes = [len(b) for b in blobs]
    if phases is None:
        phases = [0] * len(blobs)
    elif phases == "aligned":
        phases = [h.aligned_phase() for h in hs]
    bases, at = [], 0
    for n, ph in zip(sizes, phases):
        bases.append(at + ph)
        at += (ph + n + 255) // 256 * 256
    plan = B.Plan(hs, bases if layout == B.FST_LAYOUT_RESIDENT else phases, names, reqs, rank, world)
    for g in range(plan.group_count()):
        gi = plan.group(g)
        for lo, hi, off in gi["extents"]:
            assert off % 256 == (lo + phases[gi["file"]]) % 256
    plan.set_groups(max_group_bytes, min_gap, min_seg)
    keep, outs, ptrs = [], [], []
    L.fst_test_clear_outputs()
    for i in range(plan.output_count()):
        n = plan.output(i)["nbytes"]
        st, o = aligned(max(n, 1), 0xA5)
        keep.append(st)
        outs.append(o[:n])
        ptrs.append(o.ctypes.data)
        L.fst_test_add_output(o.ctypes.data, n)
    wst, ws = aligned(plan.workspace_bytes(), 0)

    def launch(src, group, lay):
        L.fst_test_set_source(src.ctypes.data, len(src))
        B.fst_prepare(plan, group, lay, len(src), ptrs, ws.ctypes.data, len(ws), 0)
        B.fst_launch(plan, group, src.ctypes.data, len(src), 0)

    if layout == B.FST_LAYOUT_RESIDENT:
        _, raw = aligned(at, 0xDD)
        for g in range(plan.group_count()):
            gi = plan.group(g)
            for lo, hi, _ in gi["extents"]:
                raw[bases[gi["file"]] + lo:bases[gi["file"]] + hi] = np.frombuffer(blobs[gi["file"]], np.uint8)[lo:hi]
        # the raw buffer ends where the last file ends (up to the next multiple of 4 may be read)
        raw = raw[:bases[-1] + sizes[-1]]
        if per_group:
            for g in range(plan.group_count()):
                launch(raw, g, layout)
        else:
            launch(raw, B.FST_ALL_GROUPS, layout)
    elif layout == B.FST_LAYOUT_SLOT:
        for g in range(plan.group_count()):
            gi = plan.group(g)
            assert not max_group_bytes or gi["slot_bytes"] <= max_group_bytes
            _, slot = aligned(gi["slot_bytes"], 0)
            slot[:] = slot_image(gi, blobs)
            launch(slot, g, layout)
    else:
        _, packed = aligned(max(plan.packed_bytes(), 1), 0)
        for g in range(plan.group_count()):
            gi = plan.group(g)
            packed[gi["packed_offset"]:gi["packed_offset"] + gi["slot_bytes"]] = slot_image(gi, blobs)
        launch(packed[:plan.packed_bytes()], B.FST_ALL_GROUPS, layout)
    assert L.fst_test_violations() == 0, L.fst_test_first_violation()
    return [o.tobytes() for o in outs], plan


LAYOUTS = [
    dict(layout=B.FST_LAYOUT_RESIDENT),
    dict(layout=B.FST_LAYOUT_RESIDENT, max_group_bytes=8192, per_group=True),
    dict(layout=B.FST_LAYOUT_RESIDENT, max_group_bytes=0, min_gap=0),
    dict(layout=B.FST_LAYOUT_SLOT, max_group_bytes=16384),
    dict(layout=B.FST_LAYOUT_SLOT, max_group_bytes=32768, min_gap=300),
    dict(layout=B.FST_LAYOUT_SLOT, max_group_bytes=16384, min_gap=300, min_seg=2),
    dict(layout=B.FST_LAYOUT_PACKED, max_group_bytes=1 << 16, min_gap=0, min_seg=64),
    dict(layout=B.FST_LAYOUT_PACKED),
    dict(layout=B.FST_LAYOUT_PACKED, max_group_bytes=20000, min_seg=1),
]


def check_all(blobs, names, reqs, rank, world, layouts=LAYOUTS, tag=""):
    """Every layout with every file at its own residues, and again with the files shifted: tensor data aligned
    for the even layouts, an arbitrary phase per file for the odd ones."""
    want = oracle_outputs(blobs, names, reqs, rank, world)
    rng = np.random.default_rng(len(names) * 7919 + len(blobs[0]))
    for k, kw in enumerate(layouts):
        for phases in (None, "aligned" if k % 2 == 0 else [int(x) for x in rng.integers(0, 256, len(blobs))]):
            got, plan = run(blobs, names, reqs, rank, world, phases=phases, **kw)
            for i, (g, w) in enumerate(zip(got, want)):
                assert g == w, f"{tag} {kw} phases {phases} output {i} {names[i]} {reqs[i]}"
            plan.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_files(seed):
    rng = np.random.default_rng(2000 + seed)
    world = int(rng.choice([1, 2, 4, 8]))
    rank = int(rng.integers(world))
    blobs, names, reqs = [], [], []
    for f in range(int(rng.integers(1, 4))):
        blob, ts = make_file(rng, n_tensors=8, big=True, prefix=f"f{f}.")
        blobs.append(blob)
        names += [n for n, _, _ in ts]
        reqs += [random_request(rng, d, s, world) for _, d, s in ts]
    check_all(blobs, names, reqs, rank, world)


@pytest.mark.parametrize("residue", [0, 1, 2, 7])
def test_ragged_rows(residue):
    rng = np.random.default_rng(300 + residue)
    spec = [("a", "BF16", (60, 1096), 8), ("b", "F32", (70, 44), 4), ("c", "I8", (90, 100), 4), ("d", "F16", (129, 72), 8),
            ("e", "BF16", (6, 50, 21), 5), ("g", "F32", (131, 72), 8), ("h", "F64", (80, 44), 4), ("i", "F64", (129, 40), 8),
            ("m", "F8_E4M3", (90, 100), 4), ("n", "F8_E5M2", (129, 72), 8)]
    ts = [("lead", "U8", (residue % 3,), bytes(residue % 3))]
    ts += [(n, dt, shape, random_bits(rng, dt, shape).tobytes()) for n, dt, shape, _ in spec]
    ts.append(("qkv", "BF16", (120, 37), random_bits(rng, "BF16", (120, 37)).tobytes()))
    blob = writer.write_file(None, ts, None, residue)
    for world in (4, 5, 8):
        names, reqs = [], []
        for n, dt, shape, w in spec:
            if w == world:
                for dst in [None] + cast_targets(dt):
                    names.append(n)
                    reqs.append((dst, 1, 1))
        if world == 4:
            names += ["qkv", "qkv"]
            reqs += [(None, 0, 3), ("F32", 0, 3)]
        for rank in (0, world - 1):
            check_all([blob], names, reqs, rank, world, tag=f"world {world} rank {rank}")


@pytest.mark.parametrize("residue", [0, 1, 2, 4, 13])
def test_rows_shorter_than_a_chunk(residue):
    rng = np.random.default_rng(500 + residue)
    spec = [("a", "U8", (700, 24), 8), ("b", "U8", (301, 26), 2), ("c", "I16", (410, 12), 4), ("d", "BF16", (290, 8), 8),
            ("e", "F32", (150, 6), 2), ("f", "F16", (205, 14), 2), ("g", "F64", (90, 6), 2), ("h", "I64", (70, 2), 2),
            ("i", "BF16", (33, 7, 10), 5), ("j", "F32", (110, 9), 3), ("k", "U8", (200, 30), 2), ("l", "F64", (120, 3), 3),
            ("m", "F8_E4M3", (300, 12), 4), ("n", "F8_E5M2", (100, 14), 2)]
    ts = [("lead", "U8", (residue % 3,), bytes(residue % 3))]
    ts += [(n, dt, shape, random_bits(rng, dt, shape).tobytes()) for n, dt, shape, _ in spec]
    blob = writer.write_file(None, ts, None, residue)
    for world in (2, 3, 4, 5, 8):
        names, reqs = [], []
        for n, dt, shape, w in spec:
            if w == world:
                for dst in [None] + cast_targets(dt):
                    names.append(n)
                    reqs.append((dst, len(shape) - 1, 1))
        for rank in sorted({0, world - 1}):
            check_all([blob], names, reqs, rank, world, tag=f"world {world} rank {rank}")
            # shares of a half to a fifth of a short row go through the LDS area (an eighth's tiles span too much for it,
            # but for the conversions with two or four elements per chunk)
            got, plan = run([blob], names, reqs, rank, world, B.FST_LAYOUT_RESIDENT)
            assert world > 5 or L.fst_test_staged_tiles() > 0, (world, L.fst_test_staged_tiles())
            plan.close()


def test_many_small_tensors_and_all_ranks():
    rng = np.random.default_rng(55)
    ts, names, reqs = [], [], []
    for i in range(900):
        dt = ("U8", "BF16", "F16", "F32", "F64")[int(rng.integers(5))]
        n = int(rng.integers(1, 600)) if rng.random() < 0.9 else int(rng.integers(2000, 9000))
        ts.append((f"t{i}", dt, (n,), random_bits(rng, dt, (n,)).tobytes()))
        names.append(f"t{i}")
        targets = cast_targets(dt)
        reqs.append((targets[int(rng.integers(len(targets)))] if targets and rng.random() < 0.35 else None, -1, 1))
    blob = writer.write_file(None, ts, None, 5)
    check_all([blob], names, reqs, 0, 1, layouts=LAYOUTS[:2] + LAYOUTS[3:4] + LAYOUTS[7:8])
    ts = [("q", "BF16", (128, 264), random_bits(rng, "BF16", (128, 264)).tobytes()),
          ("o", "F16", (264, 136), random_bits(rng, "F16", (264, 136)).tobytes()),
          ("qkv", "BF16", (3 * 64, 72), random_bits(rng, "BF16", (192, 72)).tobytes())]
    blob = writer.write_file(None, ts, None, 13)
    names, reqs = [], []
    for r in range(8):
        names += ["q", "o", "qkv"]
        reqs += [(None, 0, 1, r), ("BF16", 1, 1, r), ("F32", 0, 3, r)]
    check_all([blob], names, reqs, 0, 8)


def test_staging_with_compacted_extents():
    """The stager on the synchronous stand-in runtime: packed and streamed loads of a plan whose strided shares are
    staged as row segments back to back, through ring slots smaller than the tensors."""
    rng = np.random.default_rng(77)
    ts = [("w", "BF16", (96, 1024), None), ("o", "BF16", (1024, 96), None), ("qkv", "F16", (3 * 64, 128), None),
          ("r", "F32", (300, 274), None), ("n", "BF16", (1024,), None), ("s", "U8", (400, 24), None)]
    ts = [(n, d, s, random_bits(rng, d, s).tobytes()) for n, d, s, _ in ts]
    blob = writer.write_file(None, ts, None, 7)
    names = ["w", "o", "qkv", "r", "r", "n", "s"]
    reqs = [(None, 0, 1), (None, 1, 1), ("F32", 0, 3), (None, 1, 1), ("BF16", 1, 1), ("F32", -1, 1), (None, 1, 1)]
    world, rank = 2, 1
    want = oracle_outputs([blob], names, reqs, rank, world)
    hs = headers_of([blob])
    mem = np.frombuffer(blob, np.uint8).copy()

    @ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_uint64)
    def read(ctx, fi, off, dst, n):
        if fi != 0 or off + n > len(mem):
            return -1
        ctypes.memmove(dst, mem.ctypes.data + off, n)
        return 0

    read_ptr = ctypes.cast(read, ctypes.c_void_p).value
    for mode, group_bytes, min_gap, min_seg in (("packed", 1 << 16, 0, 16), ("packed", 0, None, 1), ("streamed", 1 << 15, 512, 64),
                                                ("packed", 1 << 16, 1 << 20, None)):
        plan = B.Plan(hs, [0], names, reqs, rank, world)
        plan.set_groups(group_bytes, min_gap, min_seg)
        L.fst_test_clear_outputs()
        keep, outs, ptrs = [], [], []
        for i in range(plan.output_count()):
            n = plan.output(i)["nbytes"]
            st, o = aligned(n, 0xA5)
            keep.append(st)
            outs.append(o)
            ptrs.append(o.ctypes.data)
            L.fst_test_add_output(o.ctypes.data, n)
        _, ws = aligned(plan.workspace_bytes(), 0)
        stager = B.Stager(3, 4, 4096)
        if mode == "packed":
            _, buf = aligned(plan.packed_bytes(), 0xCC)
            L.fst_test_set_source(buf.ctypes.data, len(buf))
            stats = stager.stage_packed(plan, read_ptr, 0, buf.ctypes.data, len(buf), ptrs, ws.ctypes.data, len(ws))
            for g in range(plan.group_count()):
                gi = plan.group(g)
                img = slot_image(gi, [blob])
                have = buf[gi["packed_offset"]:gi["packed_offset"] + gi["slot_bytes"]]
                mask = img != 0xEE                      # bytes between the extents stay untouched
                assert np.array_equal(have[mask], img[mask])
        else:
            slots = [aligned(group_bytes, 0xCC)[1] for _ in range(2)]
            lo = min(s.ctypes.data for s in slots)
            hi = max(s.ctypes.data + len(s) for s in slots)
            L.fst_test_set_source(lo, hi - lo)
            stats = stager.stage_streamed(plan, read_ptr, 0, [s.ctypes.data for s in slots], group_bytes, ptrs,
                                          ws.ctypes.data, len(ws))
        stager.close()
        assert L.fst_test_violations() == 0, L.fst_test_first_violation()
        staged = sum(plan.group(g)["staged_bytes"] for g in range(plan.group_count()))
        assert stats["staged_bytes"] == staged
        if min_seg is not None and min_seg <= 16 and min_gap is not None:
            assert staged < plan.read_bytes() + 4096, "sparse and compacted: what is staged is what is read, and little more"
        for i, w in enumerate(want):
            assert outs[i].tobytes() == w, f"{mode} {group_bytes} {min_gap} {min_seg}: output {i} {names[i]} {reqs[i]}"
        plan.close()


def test_hint_spans_follow_the_piece_length():
    """512 tensors of 8 KiB (8 tiles each): the launch's hint spans are 8 tiles long, so every tile finds its
    piece with one search step at most; one large tensor keeps spans of 1024 tiles."""
    ts = [(f"t{i}", "BF16", (4096,), bytes(8192)) for i in range(512)]
    blob = writer.write_file(None, ts, None, 0)
    names = [t[0] for t in ts]
    got, plan = run([blob], names, [(None, -1, 1)] * len(names), 0, 1, layout=B.FST_LAYOUT_RESIDENT)
    assert L.fst_test_direct_tiles() == 512 * 8
    plan.close()
    blob = writer.write_file(None, [("big", "U8", (3 << 20,), bytes(3 << 20)), ("small", "U8", (100,), bytes(100))], None, 0)
    got, plan = run([blob], ["big", "small"], [(None, -1, 1)] * 2, 0, 1, layout=B.FST_LAYOUT_RESIDENT)
    assert L.fst_test_direct_tiles() >= 3072 - 1024
    plan.close()
