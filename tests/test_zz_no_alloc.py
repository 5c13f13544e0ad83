"""fst_materialize_static -- fst_materialize with the library's built-in workspace, for callers that
cannot allocate device memory -- against fst_materialize itself, bit for bit, on two calls in a row
(the second with a smaller input, so that the workspace still holds the longer table of the first),
and against the oracle.  Runs last: a failure here must not hide the other tests."""
import numpy as np
import pytest
import torch

from paper_2505_23072_amd import binding as B
from paper_2505_23072_amd import device
from util_cases import make_file, random_request
from util_gpu import first_diff, headers_of, oracle_outputs, upload_resident

pytestmark = pytest.mark.gpu


def _case(seed, n_tensors, world):
    rng = np.random.default_rng(seed)
    blob, ts = make_file(rng, n_tensors, residue=int(rng.integers(16)), big=True)
    names, reqs = [], []
    for n, dt, shape in ts:
        names.append(n)
        reqs.append(random_request(rng, dt, shape, world))
    return blob, names, reqs


def _both_ways(blob, names, reqs, rank, world):
    hs = headers_of([blob])
    raw, bases, raw_len = upload_resident([blob])
    plan = B.Plan(hs, bases, names, reqs, rank, world)
    plan.set_groups(1 << 16)                                   # several groups, merged by FST_ALL_GROUPS
    outs = []
    for static in (False, True):
        bufs, ptrs = device.alloc_outputs(plan)
        for b in bufs:
            b.fill_(0x3C)
        torch.cuda.synchronize()
        if static:
            B.fst_materialize_static(raw.data_ptr(), raw_len, plan, B.FST_ALL_GROUPS, ptrs, 0)
        else:
            ws = device.device_bytes(plan.workspace_bytes())
            B.fst_materialize(raw.data_ptr(), raw_len, plan, B.FST_ALL_GROUPS, ptrs, ws.data_ptr(), ws.numel(), 0)
        torch.cuda.synchronize()
        outs.append([bufs[i][:plan.output(i)["nbytes"]].cpu().numpy().tobytes() for i in range(plan.output_count())])
    return outs, plan


def test_static_workspace_matches_caller_workspace_twice_in_a_row():
    for step, (seed, n_tensors, world) in enumerate(((901, 40, 2), (902, 6, 2))):       # the second input is smaller
        blob, names, reqs = _case(seed, n_tensors, world)
        print(f"call {step}: {len(blob)} bytes, {len(names)} requests", flush=True)
        (plain, static), plan = _both_ways(blob, names, reqs, 1, world)
        want = oracle_outputs([blob], names, reqs, 1, world)
        for i, (a, b, w) in enumerate(zip(plain, static, want)):
            assert b == a, f"call {step}, {names[i]} {reqs[i]}: static vs workspace: {first_diff(b, a)}"
            assert b == w, f"call {step}, {names[i]} {reqs[i]}: static vs oracle: {first_diff(b, w)}"
        plan.close()


def test_static_workspace_per_group_and_size_limit():
    blob, names, reqs = _case(903, 12, 1)
    hs = headers_of([blob])
    raw, bases, raw_len = upload_resident([blob])
    plan = B.Plan(hs, bases, names, reqs, 0, 1)
    ng = plan.set_groups(1 << 14)
    assert ng > 2
    bufs, ptrs = device.alloc_outputs(plan)
    for g in range(ng):                                        # same stream: each call may overwrite the last table
        B.fst_materialize_static(raw.data_ptr(), raw_len, plan, g, ptrs, 0)
    torch.cuda.synchronize()
    want = oracle_outputs([blob], names, reqs, 0, 1)
    for i, w in enumerate(want):
        got = bufs[i][:plan.output(i)["nbytes"]].cpu().numpy().tobytes()
        assert got == w, f"{names[i]} {reqs[i]}: {first_diff(got, w)}"
    with pytest.raises(B.FstError) as e:
        B.fst_materialize_static(raw.data_ptr(), raw_len, plan, ng, ptrs, 0)
    assert e.value.name == "FST_E_RANGE"
    plan.close()
    # a plan whose tables cannot fit the built-in workspace is refused before anything is enqueued:
    # 70 000 one-element tensors need 70 000 pieces of 64 bytes
    from synth import writer
    n = 70_000
    ts = [(f"t{i}", "U8", (1,), bytes([i & 255])) for i in range(n)]
    big = writer.write_file(None, ts, None, 0)
    hs = headers_of([big])
    raw, bases, raw_len = upload_resident([big])
    names = [t[0] for t in ts]
    plan = B.Plan(hs, bases, names, [(None, -1, 1)] * n)
    assert plan.workspace_bytes() > B.FST_STATIC_WORKSPACE_BYTES
    out = device.device_bytes(256)
    with pytest.raises(B.FstError) as e:
        B.fst_materialize_static(raw.data_ptr(), raw_len, plan, B.FST_ALL_GROUPS, [out.data_ptr()] * n, 0)
    assert e.value.name == "FST_E_RANGE" and "built-in workspace" in str(e.value)
    plan.close()
