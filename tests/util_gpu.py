"""Helpers of the GPU parity tests: put file bytes into device memory, call the C ABI, fetch the
outputs.  All computing happens in the library; the oracle is only used for the expected values."""
import numpy as np
import torch

from oracle import oracle as orc
from paper_2505_23072_amd import binding as B
from paper_2505_23072_amd import device


def headers_of(blobs):
    hs = []
    for b in blobs:
        n = B.fst_header_len(bytes(b[:8]))
        hs.append(B.Header(bytes(b[:8 + n]), len(b)))
    return hs


def phases_of(blobs, phases):
    """Per file, where its bytes sit modulo 256 in device memory: None = at their file offsets' residues,
    "aligned" = tensor data on a 256-byte boundary, or a list."""
    if phases is None:
        return [0] * len(blobs)
    if phases == "aligned":
        return [h.aligned_phase() for h in headers_of(blobs)]
    return list(phases)


def bases_of(blobs, phases=None):
    bases, at = [], 0
    for b, ph in zip(blobs, phases_of(blobs, phases)):
        bases.append(at + ph)
        at += (ph + len(b) + 255) // 256 * 256
    return bases, max(at, 256)


def upload_resident(blobs, sparse_plan=None, phases=None):
    """Whole files in the raw buffer; with sparse_plan only that plan's extents (0xDD elsewhere)."""
    bases, raw_len = bases_of(blobs, phases)
    if sparse_plan is None:
        host = np.zeros(raw_len, np.uint8)
        for b, at in zip(blobs, bases):
            host[at:at + len(b)] = np.frombuffer(b, np.uint8)
    else:
        host = np.full(raw_len, 0xDD, np.uint8)
        for g in range(sparse_plan.group_count()):
            gi = sparse_plan.group(g)
            for lo, hi, _ in gi["extents"]:
                at = bases[gi["file"]]
                host[at + lo:at + hi] = np.frombuffer(blobs[gi["file"]], np.uint8)[lo:hi]
    raw = device.device_bytes(raw_len)
    raw.copy_(torch.from_numpy(host))
    return raw, bases, raw_len


def fetch(bufs, plan):
    torch.cuda.synchronize()
    return [bufs[i][:plan.output(i)["nbytes"]].cpu().numpy().tobytes() if plan.output(i)["nbytes"] else b""
            for i in range(plan.output_count())]


def materialize_resident(blobs, names, reqs, rank=0, world=1, max_group_bytes=None, per_group=False, stream=None,
                         min_gap_bytes=None, phases=None):
    """Resident layout; one call for all groups, or one call per group."""
    hs = headers_of(blobs)
    plan = B.Plan(hs, bases_of(blobs, phases)[0], names, reqs, rank, world)
    if max_group_bytes is not None:
        plan.set_groups(max_group_bytes, min_gap_bytes)
    raw, bases, raw_len = upload_resident(blobs, plan if min_gap_bytes is not None else None, phases)
    bufs, ptrs = device.alloc_outputs(plan)
    for b in bufs:
        b.fill_(0xA5)
    ws = device.device_bytes(plan.workspace_bytes())
    sp = stream.cuda_stream if stream is not None else 0
    torch.cuda.synchronize()
    if per_group:
        for g in range(plan.group_count()):
            B.fst_materialize(raw.data_ptr(), raw_len, plan, g, ptrs, ws.data_ptr(), ws.numel(), sp)
            torch.cuda.synchronize()      # the workspace is reused by the next call
    else:
        B.fst_materialize(raw.data_ptr(), raw_len, plan, B.FST_ALL_GROUPS, ptrs, ws.data_ptr(), ws.numel(), sp)
    return fetch(bufs, plan), plan


def slot_image(gi, blobs, fill=0xEE, phases=None):
    """The slot image of one group, built on the host from the file bytes: plain extents verbatim, compacted
    extents as their row segments back to back; bytes between the extents keep `fill`."""
    host = np.full(gi["slot_bytes"], fill, np.uint8)
    data = np.frombuffer(blobs[gi["file"]], np.uint8)
    phase = phases[gi["file"]] if phases is not None else 0
    for (lo, hi, off), (row_bytes, n_rows, stride) in zip(gi["extents"], gi["extent_rows"]):
        assert off % 256 == (lo + phase) % 256
        if n_rows == 1:
            assert row_bytes == hi - lo
            host[off:off + hi - lo] = data[lo:hi]
        else:
            assert hi == lo + (n_rows - 1) * stride + row_bytes
            for r in range(n_rows):
                host[off + r * row_bytes:off + (r + 1) * row_bytes] = data[lo + r * stride:lo + r * stride + row_bytes]
    return host


def materialize_slots(blobs, names, reqs, rank, world, max_group_bytes, min_gap_bytes=None, min_segment_bytes=None,
                      phases=None):
    """Slot layout: every group's extents alone in a slot buffer, each at its slot offset."""
    hs = headers_of(blobs)
    phases = phases_of(blobs, phases)
    plan = B.Plan(hs, phases, names, reqs, rank, world)
    plan.set_groups(max_group_bytes, min_gap_bytes, min_segment_bytes)
    bufs, ptrs = device.alloc_outputs(plan)
    for b in bufs:
        b.fill_(0x5A)
    ws = device.device_bytes(plan.workspace_bytes())
    slot = device.device_bytes(max_group_bytes + 512)
    for g in range(plan.group_count()):
        gi = plan.group(g)
        assert gi["slot_bytes"] <= max_group_bytes
        slot[:gi["slot_bytes"]].copy_(torch.from_numpy(slot_image(gi, blobs, phases=phases)))
        B.fst_materialize_slot(slot.data_ptr(), gi["slot_bytes"], plan, g, ptrs, ws.data_ptr(), ws.numel(), 0)
        torch.cuda.synchronize()
    return fetch(bufs, plan), plan


def materialize_packed(blobs, names, reqs, rank=0, world=1, max_group_bytes=0, min_gap_bytes=None,
                       min_segment_bytes=None, phases=None):
    """Packed layout: the slot images of all groups side by side in one buffer, one launch set for all."""
    hs = headers_of(blobs)
    phases = phases_of(blobs, phases)
    plan = B.Plan(hs, phases, names, reqs, rank, world)
    plan.set_groups(max_group_bytes, min_gap_bytes, min_segment_bytes)
    bufs, ptrs = device.alloc_outputs(plan)
    for b in bufs:
        b.fill_(0x69)
    ws = device.device_bytes(plan.workspace_bytes())
    n = plan.packed_bytes()
    host = np.full(max(n, 256), 0xEE, np.uint8)
    at = 0
    for g in range(plan.group_count()):
        gi = plan.group(g)
        assert gi["packed_offset"] == at and at % 256 == 0
        host[at:at + gi["slot_bytes"]] = slot_image(gi, blobs, phases=phases)
        at += gi["slot_bytes"]
    assert at == n
    packed = device.device_bytes(len(host))
    packed.copy_(torch.from_numpy(host))
    torch.cuda.synchronize()
    B.fst_prepare(plan, B.FST_ALL_GROUPS, B.FST_LAYOUT_PACKED, n, ptrs, ws.data_ptr(), ws.numel(), 0)
    B.fst_launch(plan, B.FST_ALL_GROUPS, packed.data_ptr(), n, 0)
    return fetch(bufs, plan), plan


def oracle_outputs(blobs, names, reqs, rank=0, world=1):
    tabs = [orc.parse(bytes(b), len(b)) for b in blobs]
    res = []
    for nm, rq in zip(names, reqs):
        dst, dim, blocks = rq[:3]
        r = rq[3] if len(rq) > 3 and rq[3] >= 0 else rank
        for b, tab in zip(blobs, tabs):
            hit = [t for t in tab.tensors if t.name == nm]
            if not hit:
                continue
            t = hit[0]
            stored = np.frombuffer(b, np.uint8, t.end - t.begin, tab.body_off + t.begin)
            out, shape = orc.materialize(stored, t.dtype, t.shape, dst, dim, blocks, r, world)
            res.append(out.tobytes())
            break
        else:
            raise KeyError(nm)
    return res


def first_diff(a: bytes, b: bytes) -> str:
    if len(a) != len(b):
        return f"length {len(a)} != {len(b)}"
    x, y = np.frombuffer(a, np.uint8), np.frombuffer(b, np.uint8)
    bad = np.nonzero(x != y)[0]
    return f"{len(bad)} bytes differ, first at {bad[0]}: got {x[bad[0]]:#x} want {y[bad[0]]:#x}" if len(bad) else "equal"
