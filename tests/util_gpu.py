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


def upload_resident(blobs, sparse_plan=None):
    """Whole files in the raw buffer; with sparse_plan only that plan's extents (0xDD elsewhere)."""
    bases, raw_len = device.file_bases([len(b) for b in blobs])
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
                         min_gap_bytes=None):
    """Resident layout; one call for all groups, or one call per group."""
    hs = headers_of(blobs)
    plan = B.Plan(hs, device.file_bases([len(b) for b in blobs])[0], names, reqs, rank, world)
    if max_group_bytes is not None:
        plan.set_groups(max_group_bytes, min_gap_bytes)
    raw, bases, raw_len = upload_resident(blobs, plan if min_gap_bytes is not None else None)
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


def materialize_slots(blobs, names, reqs, rank, world, max_group_bytes, min_gap_bytes=None):
    """Slot layout: every group's extents alone in a slot buffer, each at its slot offset."""
    hs = headers_of(blobs)
    plan = B.Plan(hs, [0] * len(blobs), names, reqs, rank, world)
    plan.set_groups(max_group_bytes, min_gap_bytes)
    bufs, ptrs = device.alloc_outputs(plan)
    for b in bufs:
        b.fill_(0x5A)
    ws = device.device_bytes(plan.workspace_bytes())
    slot = device.device_bytes(max_group_bytes + 512)
    for g in range(plan.group_count()):
        gi = plan.group(g)
        assert gi["slot_bytes"] <= max_group_bytes
        host = np.full(gi["slot_bytes"], 0xEE, np.uint8)
        for lo, hi, off in gi["extents"]:
            assert off % 256 == lo % 256
            host[off:off + hi - lo] = np.frombuffer(blobs[gi["file"]], np.uint8)[lo:hi]
        slot[:gi["slot_bytes"]].copy_(torch.from_numpy(host))
        B.fst_materialize_slot(slot.data_ptr(), gi["slot_bytes"], plan, g, ptrs, ws.data_ptr(), ws.numel(), 0)
        torch.cuda.synchronize()
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
