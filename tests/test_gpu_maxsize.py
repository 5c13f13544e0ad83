"""Tensors longer than one kernel piece (a piece holds at most 2^31 chunks = 32 GiB of 16-byte chunks):
the planner cuts them, and chunk indices stay below 2^31 inside every piece.  A launch class with more
workgroups than one dispatch can hold (4 194 048 workgroups = 64 GiB - 4 MiB of 16-byte chunks) goes out as
several dispatches.  The bytes come from the procedural source through the staging ring.  Every output byte is compared on the device with the raw
buffer itself (a whole-tensor copy and a column slice have plain definitions as array slices), and
windows around the cut, the start and the end are compared with the oracle on the host."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2505_23072_amd import binding as B
from paper_2505_23072_amd import device
from synth.source import ProceduralModel
from synth.specs import FileSpec, ModelSpec, TensorSpec

pytestmark = pytest.mark.gpu

GiB = 1 << 30


def _stage(spec, names, reqs, rank=0, world=1):
    model = ProceduralModel(spec)
    bases, raw_len = device.file_bases(model.sizes)
    hs = [B.Header(h, s) for h, s in zip(model.headers, model.sizes)]
    plan = B.Plan(hs, bases, names, reqs, rank, world)
    raw = device.device_bytes(raw_len)
    ws = device.device_bytes(plan.workspace_bytes())
    bufs, ptrs = device.alloc_outputs(plan)
    st = B.Stager(16, 14, 32 << 20)
    try:
        st.stage_resident(plan, model.read_fn, model.ctx, raw.data_ptr(), raw_len, ptrs, ws.data_ptr(), ws.numel(),
                          B.FST_STAGE_NO_KERNELS)
    finally:
        st.close()
    B.fst_materialize(raw.data_ptr(), raw_len, plan, B.FST_ALL_GROUPS, ptrs, ws.data_ptr(), ws.numel(), 0)
    torch.cuda.synchronize()
    return model, plan, raw, bufs


def test_one_row_of_65_gib_plus_a_ragged_tail():
    """Three pieces (cuts at 32 and 64 GiB) in one launch class that needs two dispatches."""
    n = 65 * GiB + 5
    spec = ModelSpec("one-long-vector", 41, [FileSpec("a.safetensors", [
        TensorSpec("lead", "U8", (3,), fill="bytes"), TensorSpec("big", "U8", (n,), fill="bytes")], 9)])
    print(f"{spec.name}: {n} bytes", flush=True)
    model, plan, raw, bufs = _stage(spec, ["big"], [(None, -1, 1)])
    assert plan.output(0)["nbytes"] == n and plan.read_bytes() == n
    begin = len(model.headers[0]) + 3
    out = bufs[0]
    for at in range(0, n, 4 * GiB):                         # every byte, on the device
        m = min(4 * GiB, n - at)
        assert torch.equal(out[at:at + m], raw[begin + at:begin + at + m]), f"bytes [{at}, {at + m}) differ"
    first_of_second_dispatch = 4194048 * 16384
    # around the piece cuts, around the first workgroup of the second dispatch, and the ragged end, against the oracle
    for at in (0, 32 * GiB - 4096, first_of_second_dispatch - 4096, 64 * GiB - 4096, n - 8192):
        stored = model.read(0, begin + at, 8192)
        want, _ = orc.materialize(stored, "U8", (8192,))
        assert out[at:at + 8192].cpu().numpy().tobytes() == want.tobytes(), f"window at {at}"


def test_column_share_longer_than_one_piece():
    rows, cols = 36864, 1 << 20                              # bf16 [36864, 1048576]: 72 GiB stored
    spec = ModelSpec("wide-matrix", 42, [FileSpec("a.safetensors", [TensorSpec("w", "BF16", (rows, cols))], 6)])
    world, rank = 2, 1                                       # share: 36864 rows of 1 MiB = 36 GiB
    print(f"{spec.name}: [{rows}, {cols}] bf16, rank {rank} of {world} on dim 1", flush=True)
    model, plan, raw, bufs = _stage(spec, ["w"], [(None, 1, 1)], rank, world)
    half = cols // world
    assert plan.output(0)["shape"] == (rows, half) and plan.output(0)["nbytes"] == rows * half * 2
    begin = len(model.headers[0])
    assert begin % 2 == 0
    stored = raw[begin:begin + rows * cols * 2].view(torch.int16).view(rows, cols)
    out = bufs[0][:rows * half * 2].view(torch.int16).view(rows, half)
    for r in range(0, rows, 4096):                           # every element, on the device
        assert torch.equal(out[r:r + 4096], stored[r:r + 4096, rank * half:(rank + 1) * half]), f"rows from {r}"
    for r in (0, 32767, 32768, rows - 1):                    # rows around the cut (2^31 chunks = 32768 rows)
        row = model.read(0, begin + r * cols * 2, cols * 2)
        want, shape = orc.materialize(row, "BF16", (1, cols), None, 1, 1, rank, world)
        assert shape == (1, half)
        assert out[r].cpu().numpy().tobytes() == want.tobytes(), f"row {r}"
