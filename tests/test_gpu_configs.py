"""Full-size parity on the five configurations (synthetic stand-ins for the paper's Table I models:
same tensor names, shapes, dtypes and file splits; values N(0, 0.02) from a seeded pool).  The
procedural source produces the file bytes on the fly for the staging ring, and again, independently,
for the oracle, tensor by tensor.  EVERY output of every configuration is compared with the oracle,
bit for bit, in batches that bound host memory; the additional launch configurations of a test (one
merged call, per-file prepare + launch) are checked on sampled layers."""
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2505_23072_amd import binding as B
from paper_2505_23072_amd import device
from synth import specs
from synth.source import ProceduralModel
from util_gpu import first_diff

pytestmark = pytest.mark.gpu

GB = 1 << 30


def _plan(model, spec, bases):
    hs = [B.Header(h, s) for h, s in zip(model.headers, model.sizes)]
    names = [t.name for f in spec.files for t in f.tensors]
    reqs = [(t.dst_dtype, t.shard_dim, t.blocks) for f in spec.files for t in f.tensors]
    return B.Plan(hs, bases, names, reqs, spec.rank, spec.world), names, reqs


def _check_sample(model, spec, plan, bufs, names, reqs, picks, threads=16):
    """Oracle over the picked outputs (batched on plain threads), compared with the device results."""
    tabs = [orc.parse(h, s) for h, s in zip(model.headers, model.sizes)]
    jobs, meta = [], []
    for i in picks:
        info = plan.output(i)
        fi = info["file"]
        t = tabs[fi].find(names[i])
        stored = model.read(fi, tabs[fi].body_off + t.begin, t.end - t.begin)
        dst, dim, blocks = reqs[i]
        shape, nb = orc.result_info(t.dtype, t.shape, dst, dim, blocks, spec.rank, spec.world)
        assert shape == info["shape"] and nb == info["nbytes"] and (dst or t.dtype) == info["dtype"], names[i]
        jobs.append(dict(stored=stored, dtype=t.dtype, shape=t.shape, dst_dtype=dst, shard_dim=dim, blocks=blocks,
                         rank=spec.rank, world=spec.world, out=np.empty(nb, np.uint8)))
        meta.append(i)
    orc.materialize_jobs(jobs, threads)
    for i, j in zip(meta, jobs):
        got = bufs[i][:j["out"].nbytes].cpu().numpy()
        assert got.tobytes() == j["out"].tobytes(), f"{names[i]} {reqs[i]}: {first_diff(got.tobytes(), j['out'].tobytes())}"


def _check_all(model, spec, plan, bufs, names, reqs, batch_bytes=6 << 30, threads=16):
    """Every output against the oracle.  Outputs are taken in plan order in batches of about batch_bytes of
    stored tensor bytes: the stored bytes are regenerated from the byte source (a thread per tensor), the
    oracle runs over the batch on plain threads, each device result is fetched and compared, then everything
    of the batch is dropped."""
    t0 = time.time()
    tabs = [orc.parse(h, s) for h, s in zip(model.headers, model.sizes)]
    order = list(range(plan.output_count()))
    n_bytes = 0
    with ThreadPoolExecutor(threads) as pool:
        at = 0
        while at < len(order):
            batch, size = [], 0
            while at < len(order) and (not batch or size < batch_bytes):
                i = order[at]
                info = plan.output(i)
                t = tabs[info["file"]].find(names[i])
                batch.append((i, info, t))
                size += t.end - t.begin
                at += 1

            def make(item):
                i, info, t = item
                fi = info["file"]
                stored = model.read(fi, tabs[fi].body_off + t.begin, t.end - t.begin)
                dst, dim, blocks = reqs[i]
                shape, nb = orc.result_info(t.dtype, t.shape, dst, dim, blocks, spec.rank, spec.world)
                assert shape == info["shape"] and nb == info["nbytes"] and (dst or t.dtype) == info["dtype"], names[i]
                return dict(stored=stored, dtype=t.dtype, shape=t.shape, dst_dtype=dst, shard_dim=dim, blocks=blocks,
                            rank=spec.rank, world=spec.world, out=np.empty(nb, np.uint8))

            jobs = list(pool.map(make, batch))
            orc.materialize_jobs(jobs, threads)

            def compare(pair):
                (i, info, t), j = pair
                got = bufs[i][:j["out"].nbytes].cpu().numpy()
                if not np.array_equal(got, j["out"]):
                    return f"{names[i]} {reqs[i]}: {first_diff(got.tobytes(), j['out'].tobytes())}"
                return None

            bad = [b for b in pool.map(compare, zip(batch, jobs)) if b]
            assert not bad, bad[:3]
            n_bytes += sum(j["out"].nbytes for j in jobs)
            del jobs
    assert n_bytes == plan.write_bytes()
    print(f"{spec.name}: all {len(order)} outputs ({n_bytes / 1e9:.2f} GB) equal the oracle's, {time.time() - t0:.1f}s", flush=True)


def _picks(spec, names, layers):
    """Non-layer tensors plus every tensor of the given layers."""
    keep = []
    for i, n in enumerate(names):
        parts = n.split(".")
        idx = [int(p) for p in parts if p.isdigit()]
        if not idx or idx[0] in layers:
            keep.append(i)
    return keep


def _headers(model):
    return [B.Header(h, s) for h, s in zip(model.headers, model.sizes)]


def _run_resident(spec, layers, group_bytes=GB, aligned=False):
    """aligned: every file shifted so that its tensor data starts on a 256-byte boundary of the raw buffer (what
    bench.py and the loader do); otherwise every byte at its file offset's residue."""
    t0 = time.time()
    model = ProceduralModel(spec)
    bases, raw_len = device.file_bases(model.sizes, _headers(model) if aligned else None)
    plan, names, reqs = _plan(model, spec, bases)
    plan.set_groups(group_bytes)
    raw = device.device_bytes(raw_len)
    ws = device.device_bytes(plan.workspace_bytes())
    bufs, ptrs = device.alloc_outputs(plan)
    st = B.Stager(8, 12, 128 << 20)          # the ring bench.py uses
    try:
        stats = st.stage_resident(plan, model.read_fn, model.ctx, raw.data_ptr(), raw_len, ptrs, ws.data_ptr(), ws.numel())
    finally:
        st.close()
    print(f"{spec.name}: staged {stats['staged_bytes'] / 1e9:.2f} GB in {stats['seconds_total']:.2f}s "
          f"({plan.group_count()} groups), setup {time.time() - t0:.1f}s", flush=True)
    assert plan.write_bytes() == sum(plan.output(i)["nbytes"] for i in range(plan.output_count()))
    _check_all(model, spec, plan, bufs, names, reqs)
    # the launch configuration the benchmark times: one call for everything, raw bytes resident
    for b in bufs:
        b.zero_()
    B.fst_materialize(raw.data_ptr(), raw_len, plan, B.FST_ALL_GROUPS, ptrs, ws.data_ptr(), ws.numel(), 0)
    torch.cuda.synchronize()
    _check_sample(model, spec, plan, bufs, names, reqs, _picks(spec, names, layers[:1]))
    # and the way bench.py launches it: one group per file, tables uploaded first (fst_prepare), then the
    # kernels of each file by themselves (fst_launch)
    for b in bufs:
        b.zero_()
    ng = plan.set_groups(0)
    assert ng == len(spec.files)
    wss = [device.device_bytes(plan.workspace_bytes()) for _ in range(ng)]
    for g in range(ng):
        B.fst_prepare(plan, g, B.FST_LAYOUT_RESIDENT, raw_len, ptrs, wss[g].data_ptr(), wss[g].numel(), 0)
    for g in range(ng):
        B.fst_launch(plan, g, raw.data_ptr(), raw_len, 0)
    torch.cuda.synchronize()
    _check_sample(model, spec, plan, bufs, names, reqs, _picks(spec, names, layers[-1:]))
    return plan


def _run_streamed(spec, dev_slots, slot_bytes, min_gap=None, min_seg=None):
    t0 = time.time()
    model = ProceduralModel(spec)
    # the compacted staging is the one bench.py times: like it, with every file's tensor data aligned
    phases = device.file_phases(_headers(model)) if min_seg is not None else [0] * len(model.sizes)
    plan, names, reqs = _plan(model, spec, phases)
    ng = plan.set_groups(slot_bytes, min_gap, min_seg)
    slots = [device.device_bytes(slot_bytes) for _ in range(dev_slots)]
    ws = device.device_bytes(plan.workspace_bytes())
    bufs, ptrs = device.alloc_outputs(plan)
    st = B.Stager(8, 12, 128 << 20)          # the ring bench.py uses
    try:
        stats = st.stage_streamed(plan, model.read_fn, model.ctx, [s.data_ptr() for s in slots], slot_bytes, ptrs,
                                  ws.data_ptr(), ws.numel())
    finally:
        st.close()
    kind = ("compacted " if min_seg is not None else "") + ("sparse " if min_gap is not None else "")
    print(f"{spec.name}: {kind}streamed {stats['staged_bytes'] / 1e9:.2f} GB in {stats['seconds_total']:.2f}s through "
          f"{dev_slots}x{slot_bytes / GB:.1f} GiB device slots ({ng} groups), outputs {plan.write_bytes() / 1e9:.2f} GB, "
          f"setup {time.time() - t0:.1f}s", flush=True)
    assert stats["staged_bytes"] == sum(plan.group(g)["staged_bytes"] for g in range(ng))
    _check_all(model, spec, plan, bufs, names, reqs)
    return plan, stats


@pytest.mark.parametrize("aligned", [False, True])
def test_config2_llama7b_resident(aligned):
    spec = specs.config2_llama7b()
    plan = _run_resident(spec, layers=[0, 23, 24, 31], aligned=aligned)
    assert plan.output_count() == 291 and plan.read_bytes() == plan.write_bytes() == 13_476_831_232


@pytest.mark.parametrize("aligned", [False, True])
def test_config3_llama13b_fp16_to_bf16(aligned):
    spec = specs.config3_llama13b()
    plan = _run_resident(spec, layers=[0, 13, 39], aligned=aligned)
    assert plan.output_count() == 363 and plan.read_bytes() == plan.write_bytes() == 26_031_728_640
    assert plan.output(5)["dtype"] == "BF16"


# how the tensor-parallel configurations are staged: whole groups (first to last needed byte); sparse (unread
# ranges above 1 MiB left out; the kernels take dim-1 shares with strided reads); sparse and compacted (row
# segments of 2 KiB and more read one by one and staged back to back: what is staged is what the rank reads)
STAGINGS = [(None, None), (1 << 20, None), (1 << 20, 2048)]


@pytest.mark.parametrize("min_gap,min_seg", STAGINGS)
def test_config4_llama70b_tp8_rank0_streamed(min_gap, min_seg):
    spec = specs.config4_llama70b()
    plan, stats = _run_streamed(spec, dev_slots=3, slot_bytes=4 * GB, min_gap=min_gap, min_seg=min_seg)
    assert plan.output_count() == 723
    assert plan.write_bytes() == 18_163_974_144 == plan.read_bytes()
    if min_seg is not None:
        assert stats["staged_bytes"] <= 1.1 * plan.read_bytes()


@pytest.mark.parametrize("min_gap,min_seg", STAGINGS)
def test_config5_bloom176b_tp8_rank0_streamed(min_gap, min_seg):
    spec = specs.config5_bloom176b()
    plan, stats = _run_streamed(spec, dev_slots=3, slot_bytes=4 * GB, min_gap=min_gap, min_seg=min_seg)
    assert plan.output_count() == 845
    assert plan.write_bytes() == 50_374_675_456
    # layer norms are widened to fp32: they read 2 bytes and write 4 per element
    assert plan.write_bytes() - plan.read_bytes() == 16_285_696 // 2
    if min_seg is not None:
        assert stats["staged_bytes"] <= 1.1 * plan.read_bytes()


def _run_as_benchmarked(spec, layers):
    """The two launch configurations bench.py times for a tensor-parallel configuration, files placed with their
    tensor data aligned.  End to end: what the rank reads, sparse and compacted, staged into the packed layout and
    materialized group by group while it is staged; every output is compared.  Kernel leg: all staged bytes
    in device memory first (whole files resident when they fit beside the outputs, else the sparse packed layout
    with row-split tensors whole), then one merged launch set over every group; sampled layers are compared."""
    import gc
    gc.collect()
    torch.cuda.empty_cache()            # the buffers below need most of the device
    model = ProceduralModel(spec)
    hs = _headers(model)
    phases = device.file_phases(hs)
    st = B.Stager(8, 12, 128 << 20)
    try:
        # end to end
        plan, names, reqs = _plan(model, spec, phases)
        plan.set_groups(GB, 1 << 20, 2048)
        n = plan.packed_bytes()
        packed = device.device_bytes(n)
        ws = device.device_bytes(plan.workspace_bytes())
        bufs, ptrs = device.alloc_outputs(plan)
        stats = st.stage_packed(plan, model.read_fn, model.ctx, packed.data_ptr(), n, ptrs, ws.data_ptr(), ws.numel())
        assert stats["staged_bytes"] <= 1.01 * plan.read_bytes()
        print(f"{spec.name}: packed, sparse + compacted: staged {stats['staged_bytes'] / 1e9:.2f} GB in {stats['seconds_total']:.2f}s, "
              f"{plan.group_count()} groups", flush=True)
        _check_all(model, spec, plan, bufs, names, reqs)
        plan.close()
        del packed, ws
        for b in bufs:
            b.zero_()
        gc.collect()
        torch.cuda.empty_cache()
        # kernel leg
        bases, raw_len = device.file_bases(model.sizes, hs)
        resident = raw_len + sum(b.numel() for b in bufs) <= 230 * GB
        plan, names, reqs = _plan(model, spec, bases if resident else phases)
        plan.set_groups(GB, None if resident else 1 << 20)
        n = raw_len if resident else plan.packed_bytes()
        src = device.device_bytes(n)
        ws = device.device_bytes(plan.workspace_bytes())
        fn = st.stage_resident if resident else st.stage_packed
        fn(plan, model.read_fn, model.ctx, src.data_ptr(), n, ptrs, ws.data_ptr(), ws.numel(), B.FST_STAGE_NO_KERNELS)
        layout = B.FST_LAYOUT_RESIDENT if resident else B.FST_LAYOUT_PACKED
        B.fst_prepare(plan, B.FST_ALL_GROUPS, layout, n, ptrs, ws.data_ptr(), ws.numel(), 0)
        B.fst_launch(plan, B.FST_ALL_GROUPS, src.data_ptr(), n, 0)
        torch.cuda.synchronize()
        print(f"{spec.name}: kernel leg from the {'resident' if resident else 'packed sparse'} layout, {n / 1e9:.1f} GB staged, "
              f"{plan.group_count()} groups in one launch set", flush=True)
        _check_sample(model, spec, plan, bufs, names, reqs, _picks(spec, names, layers))
        plan.close()
        del src, ws, bufs
    finally:
        st.close()
        gc.collect()
        torch.cuda.empty_cache()


def test_config4_llama70b_as_benchmarked():
    _run_as_benchmarked(specs.config4_llama70b(), layers=[0, 41, 79])


def test_config5_bloom176b_as_benchmarked():
    _run_as_benchmarked(specs.config5_bloom176b(), layers=[0, 35, 69])


def test_falcon40b_tp2_rank0_streamed_sparse():
    """A second workload from the paper's Table I (Falcon-40B, 9 files, loaded on two GPUs there)."""
    spec = specs.config_falcon40b()
    assert spec.n_tensors == 60 * 8 + 4 and abs(spec.body_bytes / 2 ** 30 - 78) < 1.0
    plan, _ = _run_streamed(spec, dev_slots=3, slot_bytes=4 * GB, min_gap=1 << 20)
    whole = sum(t.nbytes for f in spec.files for t in f.tensors if t.shard_dim < 0)
    split = sum(t.nbytes for f in spec.files for t in f.tensors if t.shard_dim >= 0)
    assert plan.write_bytes() == whole + split // 2 == plan.read_bytes()


def test_config4_through_the_loader_api(tmp_path):
    """Llama-70B rank 0 of 8 through the paper-shaped Python API with the requests declared first: what crosses the
    bus is what the sparse, compacted plan stages, every tensor equals the oracle's, and a loop of get_sharded /
    get_tensor over all 723 keys costs microseconds per key.  The checkpoint is written to tmpfs three layers at a
    time (files of 138 GB do not fit), so the loader runs once per slice of files."""
    import os
    import shutil
    import tempfile

    from paper_2505_23072_amd.loader import LocalShard, SafeTensorsFileLoader
    spec = specs.config4_llama70b()
    model = ProceduralModel(spec)
    base = "/dev/shm" if os.path.isdir("/dev/shm") else str(tmp_path)
    tabs = [orc.parse(h, s) for h, s in zip(model.headers, model.sizes)]
    ld = SafeTensorsFileLoader(LocalShard(spec.rank, spec.world), torch.device("cuda:0"))
    total_staged = total_read = n_keys = 0
    t_fetch = 0.0
    try:
        for f0 in range(0, len(spec.files), 3):
            work = tempfile.mkdtemp(prefix="fst_loader_", dir=base)
            try:
                fis = list(range(f0, min(f0 + 3, len(spec.files))))
                paths = []
                for fi in fis:
                    p = os.path.join(work, spec.files[fi].filename)
                    model.write_file(fi, p, 16)
                    paths.append(p)
                reqs = {t.name: (t.dst_dtype, t.shard_dim, t.blocks) for fi in fis for t in spec.files[fi].tensors}
                ld.add_filenames({0: paths})
                ld.add_requests(reqs)
                fb = ld.copy_files_to_device()
                probe = B.Plan([B.Header(model.headers[fi], model.sizes[fi]) for fi in fis], [0] * len(fis), list(reqs),
                               list(reqs.values()), spec.rank, spec.world)
                probe.set_groups(1 << 30, 1 << 20, 2048)
                want_staged = sum(probe.group(g)["staged_bytes"] for g in range(probe.group_count()))
                assert fb.staged_bytes == want_staged <= 1.01 * probe.read_bytes()
                total_staged += fb.staged_bytes
                total_read += probe.read_bytes()
                probe.close()
                t = time.perf_counter()
                got = {n: (fb.get_sharded(n, rq[1], rq[0], rq[2]) if rq[1] >= 0 else fb.get_tensor(n, rq[0])) for n, rq in reqs.items()}
                t_fetch += time.perf_counter() - t
                n_keys += len(got)
                jobs, keys = [], []
                for fi in fis:
                    for ts in spec.files[fi].tensors:
                        t_ = tabs[fi].find(ts.name)
                        stored = model.read(fi, tabs[fi].body_off + t_.begin, t_.end - t_.begin)
                        dst, dim, blocks = reqs[ts.name]
                        shape, nb = orc.result_info(t_.dtype, t_.shape, dst, dim, blocks, spec.rank, spec.world)
                        assert tuple(got[ts.name].shape) == shape
                        jobs.append(dict(stored=stored, dtype=t_.dtype, shape=t_.shape, dst_dtype=dst, shard_dim=dim, blocks=blocks,
                                         rank=spec.rank, world=spec.world, out=np.empty(nb, np.uint8)))
                        keys.append(ts.name)
                orc.materialize_jobs(jobs, 16)
                for k, j in zip(keys, jobs):
                    g = got[k].contiguous().view(-1).view(torch.uint8).cpu().numpy()
                    assert np.array_equal(g, j["out"]), k
                fb.close()
                del got, jobs
            finally:
                shutil.rmtree(work, ignore_errors=True)
    finally:
        ld.close()
    assert n_keys == 723 and total_read == 18_163_974_144 and total_staged <= 1.01 * total_read
    print(f"loader API, llama-70b rank 0/8: staged {total_staged / 1e9:.2f} GB for {total_read / 1e9:.2f} GB read; "
          f"{n_keys} keys fetched in {t_fetch * 1e3:.2f} ms ({t_fetch / n_keys * 1e6:.1f} us per key)", flush=True)


def test_config2_per_key_fetches_through_the_loader_api(tmp_path):
    """Llama-7B the paper's way: whole files staged verbatim, then one get_tensor per key.  A fetch only
    enqueues (tables in the library's built-in workspace, no wait), so the loop over all 291 keys is timed
    separately from the kernels it queues; every tensor is then compared with the oracle."""
    import os
    import shutil
    import tempfile

    from paper_2505_23072_amd.loader import SafeTensorsFileLoader, SingleGroup
    spec = specs.config2_llama7b()
    model = ProceduralModel(spec)
    base = "/dev/shm" if os.path.isdir("/dev/shm") else str(tmp_path)
    work = tempfile.mkdtemp(prefix="fst_loader_", dir=base)
    try:
        paths = model.write_all(work, threads=16)
        ld = SafeTensorsFileLoader(SingleGroup(), torch.device("cuda:0"))
        ld.add_filenames({0: paths})
        t = time.perf_counter()
        fb = ld.copy_files_to_device()
        t_copy = time.perf_counter() - t
        names = [ts.name for f in spec.files for ts in f.tensors]
        torch.cuda.synchronize()
        t = time.perf_counter()
        got = {n: fb.get_tensor(n) for n in names}
        t_loop = time.perf_counter() - t
        torch.cuda.synchronize()
        t_all = time.perf_counter() - t
        print(f"loader API, llama-7b: copy_files_to_device {t_copy:.3f}s; {len(names)} get_tensor calls enqueued in "
              f"{t_loop * 1e3:.1f} ms ({t_loop / len(names) * 1e6:.0f} us per key), kernels done after {t_all * 1e3:.1f} ms", flush=True)
        tabs = [orc.parse(h, s) for h, s in zip(model.headers, model.sizes)]
        for fi, f in enumerate(spec.files):
            jobs = []
            for ts in f.tensors:
                t_ = tabs[fi].find(ts.name)
                stored = model.read(fi, tabs[fi].body_off + t_.begin, t_.end - t_.begin)
                jobs.append(dict(stored=stored, dtype=t_.dtype, shape=t_.shape, dst_dtype=None, shard_dim=-1, blocks=1, rank=0,
                                 world=1, out=np.empty(t_.end - t_.begin, np.uint8)))
            orc.materialize_jobs(jobs, 16)
            for ts, j in zip(f.tensors, jobs):
                g = got[ts.name].contiguous().view(-1).view(torch.uint8).cpu().numpy()
                assert np.array_equal(g, j["out"]), ts.name
        fb.close()
        ld.close()
    finally:
        shutil.rmtree(work, ignore_errors=True)
