"""GPU tests of the staging ring (paper Section III-A: pinned bounce buffer + host-to-device copies)
together with the kernels: tiny ring slots force every wrap and split case; results must equal the
oracle's and the staged bytes must equal the file bytes."""
import ctypes
import os

import numpy as np
import pytest
import torch

from paper_2505_23072_amd import binding as B
from paper_2505_23072_amd import device
from synth import specs
from synth.source import ProceduralModel
from synth import writer
from util_cases import make_file, random_bits, random_request
from util_gpu import bases_of, first_diff, headers_of, oracle_outputs, phases_of

pytestmark = pytest.mark.gpu


def _case(seed, tmp_path, nfiles=3):
    rng = np.random.default_rng(seed)
    world = int(rng.choice([1, 2, 4]))
    rank = int(rng.integers(world))
    blobs, names, reqs, paths = [], [], [], []
    for f in range(nfiles):
        blob, ts = make_file(rng, n_tensors=8, big=True, prefix=f"f{f}.")
        p = str(tmp_path / f"f{f}.safetensors")
        open(p, "wb").write(blob)
        blobs.append(blob)
        paths.append(p)
        names += [n for n, _, _ in ts]
        reqs += [random_request(rng, d, s, world) for _, d, s in ts]
    return blobs, paths, names, reqs, rank, world


class Fds:
    def __init__(self, paths):
        self.fds = [os.open(p, os.O_RDONLY) for p in paths]
        self.arr = (ctypes.c_int * len(self.fds))(*self.fds)

    @property
    def ctx(self):
        return ctypes.addressof(self.arr)

    def close(self):
        for fd in self.fds:
            os.close(fd)


@pytest.mark.parametrize("seed,slots,threads,slot_bytes,group_bytes,gap", [
    (0, 3, 4, 4096, 16384, None), (1, 2, 1, 4096, 4096, None), (2, 8, 8, 65536, 1 << 20, None), (3, 1, 3, 8192, 0, None),
    (4, 5, 2, 4096, 50000, None), (5, 3, 4, 4096, 16384, 0), (6, 4, 2, 8192, 0, 1000),
    # slots of many parts: several reader threads fill one slot together
    (7, 3, 8, 131072, 1 << 20, None), (8, 2, 16, 262144, 0, 500), (9, 1, 12, 65536, 0, None)])
def test_resident_ring(seed, slots, threads, slot_bytes, group_bytes, gap, tmp_path):
    blobs, paths, names, reqs, rank, world = _case(seed, tmp_path)
    print(f"seed {seed} ring {slots}x{slot_bytes} threads {threads} groups {group_bytes}", flush=True)
    want = oracle_outputs(blobs, names, reqs, rank, world)
    hs = headers_of(blobs)
    # the files at their own residues, with their tensor data on a 256-byte boundary, or at any phase
    phases = (None, "aligned", [(37 * seed + 11 * f) % 256 for f in range(len(blobs))])[seed % 3]
    bases, raw_len = bases_of(blobs, phases)
    plan = B.Plan(hs, bases, names, reqs, rank, world)
    plan.set_groups(group_bytes, gap)
    raw = device.device_bytes(raw_len)
    raw.fill_(0xCC)
    ws = device.device_bytes(plan.workspace_bytes())
    bufs, ptrs = device.alloc_outputs(plan)
    st = B.Stager(slots, threads, slot_bytes)
    fds = Fds(paths)
    try:
        stats = st.stage_resident(plan, B.read_fds_fn(), fds.ctx, raw.data_ptr(), raw_len, ptrs, ws.data_ptr(), ws.numel())
        staged = sum(plan.group(g)["staged_bytes"] for g in range(plan.group_count()))
        assert stats["staged_bytes"] == staged and stats["n_copies"] >= plan.group_count()
        host = raw.cpu().numpy()
        covered = np.zeros(raw_len, bool)
        for g in range(plan.group_count()):                     # staged bytes == file bytes
            gi = plan.group(g)
            at = bases[gi["file"]]
            for lo, hi, _ in gi["extents"]:
                assert host[at + lo:at + hi].tobytes() == blobs[gi["file"]][lo:hi]
                covered[at + lo:at + hi] = True
        assert np.all(host[~covered] == 0xCC)                   # nothing else was written
        for i, w in enumerate(want):
            got = bufs[i][:len(w)].cpu().numpy().tobytes() if len(w) else b""
            assert got == w, f"{names[i]} {reqs[i]}: {first_diff(got, w)}"
        # copy-only modes run the same ring without kernels / without reads
        for flags in (B.FST_STAGE_NO_KERNELS, B.FST_STAGE_NO_KERNELS | B.FST_STAGE_NO_READ):
            s2 = st.stage_resident(plan, B.read_fds_fn(), fds.ctx, raw.data_ptr(), raw_len, ptrs, ws.data_ptr(),
                                   ws.numel(), flags)
            assert s2["staged_bytes"] == staged
    finally:
        fds.close()
        st.close()


@pytest.mark.parametrize("seed,dev_slots,group_bytes,gap", [(10, 2, 32768, None), (11, 1, 8192, None), (12, 3, 100000, None),
                                                            (13, 4, 4096, None), (14, 2, 32768, 0), (15, 3, 65536, 2000)])
def test_streamed_ring(seed, dev_slots, group_bytes, gap, tmp_path):
    """Raw buffer = ring of device slots smaller than the files: groups are cut to fit."""
    blobs, paths, names, reqs, rank, world = _case(seed, tmp_path)
    print(f"seed {seed} device slots {dev_slots}x{group_bytes}", flush=True)
    want = oracle_outputs(blobs, names, reqs, rank, world)
    hs = headers_of(blobs)
    phases = phases_of(blobs, (None, "aligned", [(37 * seed + 11 * f) % 256 for f in range(len(blobs))])[seed % 3])
    plan = B.Plan(hs, phases, names, reqs, rank, world)
    ng = plan.set_groups(group_bytes, gap)
    assert ng > len(blobs)
    slots = [device.device_bytes(group_bytes) for _ in range(dev_slots)]
    ws = device.device_bytes(plan.workspace_bytes())
    bufs, ptrs = device.alloc_outputs(plan)
    st = B.Stager(4, 3, 4096)
    fds = Fds(paths)
    try:
        st.stage_streamed(plan, B.read_fds_fn(), fds.ctx, [s.data_ptr() for s in slots], group_bytes, ptrs,
                          ws.data_ptr(), ws.numel())
        for i, w in enumerate(want):
            got = bufs[i][:len(w)].cpu().numpy().tobytes() if len(w) else b""
            assert got == w, f"{names[i]} {reqs[i]}: {first_diff(got, w)}"
        with pytest.raises(B.FstError) as e:      # slots smaller than a group are refused up front
            st.stage_streamed(plan, B.read_fds_fn(), fds.ctx, [s.data_ptr() for s in slots], group_bytes // 2, ptrs,
                              ws.data_ptr(), ws.numel())
        assert e.value.name == "FST_E_RANGE"
    finally:
        fds.close()
        st.close()


def test_read_failure_is_reported(tmp_path):
    blobs, paths, names, reqs, rank, world = _case(20, tmp_path, nfiles=1)
    short = str(tmp_path / "short.safetensors")
    open(short, "wb").write(blobs[0][:len(blobs[0]) // 2])       # the file ends before its header says
    hs = headers_of(blobs)
    plan = B.Plan(hs, [0], names, reqs, rank, world)
    plan.set_groups(8192)
    raw = device.device_bytes(len(blobs[0]) + 256)
    ws = device.device_bytes(plan.workspace_bytes())
    bufs, ptrs = device.alloc_outputs(plan)
    st = B.Stager(2, 2, 4096)
    fds = Fds([short])
    try:
        with pytest.raises(B.FstError) as e:
            st.stage_resident(plan, B.read_fds_fn(), fds.ctx, raw.data_ptr(), raw.numel(), ptrs, ws.data_ptr(), ws.numel())
        assert e.value.name == "FST_E_IO"
        with pytest.raises(B.FstError) as e:      # raw buffer too small for the plan
            st.stage_resident(plan, B.read_fds_fn(), fds.ctx, raw.data_ptr(), 1024, ptrs, ws.data_ptr(), ws.numel())
        assert e.value.name == "FST_E_RANGE"
        torch.cuda.synchronize()
    finally:
        fds.close()
        st.close()


def test_tiny_checkpoint_end_to_end(tmp_path):
    """The tiny configuration (2-layer Llama-like model plus int8[37] and bool[13] tensors that push the
    weights to odd offsets): files -> tensors, every tensor against the oracle."""
    from oracle import oracle as orc
    spec = specs.config1_tiny()
    model = ProceduralModel(spec)
    paths = model.write_all(str(tmp_path))
    blob = open(paths[0], "rb").read()
    table = orc.parse(blob, len(blob))
    offs = {t.name: (table.body_off + t.begin) % 16 for t in table.tensors}
    assert offs["model.embed_tokens.weight"] % 2 == (table.body_off + 37) % 2     # odd shift from int8[37]
    out = device.load_files(paths, group_bytes=1 << 20)
    assert len(out) == spec.n_tensors == 23
    for t in table.tensors:
        stored = np.frombuffer(blob, np.uint8, t.end - t.begin, table.body_off + t.begin)
        want, shape = orc.materialize(stored, t.dtype, t.shape)
        got = out[t.name]
        assert tuple(got.shape) == shape and got.dtype == device.TORCH_DTYPE[t.dtype]
        gb = got.contiguous().view(-1).view(torch.uint8).cpu().numpy().tobytes()
        assert gb == want.tobytes(), f"{t.name}: {first_diff(gb, want.tobytes())}"
    # norm weights are ones, as the configuration says
    assert torch.all(out["model.norm.weight"].float() == 1.0)


def test_smoke_entry_point():
    import __graft_entry__
    __graft_entry__.smoke()


def test_loader_api(tmp_path):
    """The paper-shaped Python API (Figs. 8/9) over the C ABI: whole tensors, shards, conversions."""
    from oracle import oracle as orc
    from paper_2505_23072_amd.loader import FilesBufferOnDevice, LocalShard, SafeTensorsFileLoader, SingleGroup
    blobs, paths, names, reqs, rank, world = _case(30, tmp_path, nfiles=2)
    loader = SafeTensorsFileLoader(SingleGroup(), torch.device("cuda:0"))
    loader.add_filenames({0: paths})
    fb = loader.copy_files_to_device()
    assert sorted(fb.keys()) == sorted(names)
    want = oracle_outputs(blobs, names, [(None, -1, 1)] * len(names))
    for n, w in zip(names, want):
        t = fb.get_tensor(n)
        assert t.contiguous().view(-1).view(torch.uint8).cpu().numpy().tobytes() == w if len(w) else t.numel() == 0
    fb.close()
    with pytest.raises(RuntimeError):
        fb.get_tensor(names[0])
    # rank 1 of 2: shards and conversions in one launch set; auto release after the last key
    sh = SafeTensorsFileLoader(LocalShard(1, 2), torch.device("cuda:0"), auto_release=True)
    sh.add_filenames({0: paths[:1], 1: paths[1:]})
    fb = sh.copy_files_to_device()
    rq = {n: r for n, r in zip(names, [random_request(np.random.default_rng(i), d, s, 2)
                                       for i, (n_, d, s) in enumerate(_specs_of(blobs))])}
    got = fb.get_many(rq)
    want = oracle_outputs(blobs, list(rq), list(rq.values()), 1, 2)
    for (n, t), w in zip(got.items(), want):
        gb = t.contiguous().view(-1).view(torch.uint8).cpu().numpy().tobytes() if t.numel() else b""
        assert gb == w, n
    with pytest.raises(RuntimeError):      # every key fetched: the raw buffer is gone
        fb.get_tensor(names[0])
    loader.close()
    sh.close()


def test_loader_with_declared_requests_stages_sparsely(tmp_path):
    """Requests declared before copy_files_to_device: only the rank's bytes cross the bus (gaps skipped, row
    segments compacted), resident-packed and streamed through small device slots; per-key fetches on two
    streams in turn (they share the library's built-in workspace) without a wait in between."""
    from paper_2505_23072_amd.loader import LocalShard, SafeTensorsFileLoader
    rng = np.random.default_rng(61)
    ts = [("emb", "BF16", (512, 256)), ("q", "BF16", (1024, 256)), ("o", "BF16", (256, 2048)), ("qkv", "F16", (3 * 256, 128)),
          ("n", "BF16", (256,)), ("r", "F32", (300, 274)), ("u", "BF16", (4096, 256)), ("d", "BF16", (256, 4096))]
    full = [(n, d, s, random_bits(rng, d, s).tobytes()) for n, d, s in ts]
    path = str(tmp_path / "m.safetensors")
    blob = writer.write_file(path, full, None, 9)
    reqs = {"emb": (None, -1, 1), "q": (None, 0, 1), "o": (None, 1, 1), "qkv": ("F32", 0, 3), "n": ("F32", -1, 1),
            "r": ("BF16", 1, 1), "u": (None, 0, 1), "d": (None, 1, 1)}
    world, rank = 2, 1
    want = oracle_outputs([blob], list(reqs), list(reqs.values()), rank, world)
    probe = B.Plan(headers_of([blob]), [0], list(reqs), list(reqs.values()), rank, world)
    read_bytes = probe.read_bytes()
    probe.close()
    for slots in (None, (2, 1 << 18)):
        ld = SafeTensorsFileLoader(LocalShard(rank, world), torch.device("cuda:0"), bounce_buffer_bytes=1 << 16,
                                   min_gap_bytes=4096, min_segment_bytes=256, group_bytes=1 << 20)
        ld.add_filenames({0: [path]})
        ld.add_requests(reqs)
        fb = ld.copy_files_to_device(stream_slots=slots)
        # what crossed the bus is what the rank reads (plus nothing: every gap here is above min_gap, every
        # row segment above min_segment)
        assert fb.staged_bytes == read_bytes, (fb.staged_bytes, read_bytes, slots)
        assert fb.staged_bytes < 0.6 * len(blob)
        for (n, rq), w in zip(reqs.items(), want):
            t = fb.get_sharded(n, rq[1], rq[0], rq[2]) if rq[1] >= 0 else fb.get_tensor(n, rq[0])
            assert t.contiguous().view(-1).view(torch.uint8).cpu().numpy().tobytes() == w, (n, slots)
        with pytest.raises(RuntimeError):       # not declared, and the raw bytes were never resident
            fb.get_sharded("q", 1)
        fb.close()
        ld.close()
    # undeclared: whole files resident; fetches alternate between two streams and never wait
    ld = SafeTensorsFileLoader(LocalShard(rank, world), torch.device("cuda:0"))
    ld.add_filenames({0: [path]})
    fb = ld.copy_files_to_device()
    assert fb.staged_bytes == len(blob) - headers_of([blob])[0].body_offset()      # every tensor byte, once
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = {}
    for rep in range(3):
        for k, (n, rq) in enumerate(reqs.items()):
            with torch.cuda.stream(streams[(k + rep) % 2]):
                got[n] = fb.get_many({n: rq})[n]
    torch.cuda.synchronize()
    for (n, rq), w in zip(reqs.items(), want):
        assert got[n].contiguous().view(-1).view(torch.uint8).cpu().numpy().tobytes() == w, n
    fb.close()
    ld.close()


def test_files_written_by_the_safetensors_package(tmp_path):
    """Interoperation with the format's own implementation: checkpoints written by the `safetensors`
    package (its header sizes, key order and padding, whatever they are) are loaded through the staging
    ring and the kernels and must equal, bit for bit, what the package's own loader returns; slices and
    conversions are compared with torch indexing / torch CPU conversions of the package's tensors."""
    import safetensors.torch as st
    from paper_2505_23072_amd.loader import LocalShard, SafeTensorsFileLoader, SingleGroup
    g = torch.Generator().manual_seed(5)
    files = {}
    for f in range(2):
        files[f] = {
            f"l{f}.q.weight": (torch.randn(96, 64, generator=g) * 0.02).to(torch.bfloat16),
            f"l{f}.o.weight": (torch.randn(64, 96, generator=g) * 0.02).to(torch.float16),
            f"l{f}.norm.weight": torch.ones(64, dtype=torch.float32),
            f"l{f}.ids": torch.arange(37, dtype=torch.int64),
            f"l{f}.mask": torch.arange(13) % 2 == 0,
            f"l{f}.bytes": torch.arange(7, dtype=torch.uint8),
            f"l{f}.scalar": torch.tensor(3.25, dtype=torch.float64),
        }
    paths = []
    for f, tensors in files.items():
        p = str(tmp_path / f"pkg{f}.safetensors")
        st.save_file(tensors, p, metadata={"format": "pt"} if f else None)
        paths.append(p)
    ref = {}
    for p in paths:
        ref.update(st.load_file(p))          # the package's own loader, on the CPU

    def bits(t):
        return t.contiguous().view(-1).view(torch.uint8).cpu().numpy().tobytes() if t.numel() else b""

    loader = SafeTensorsFileLoader(SingleGroup(), torch.device("cuda:0"))
    loader.add_filenames({0: paths})
    fb = loader.copy_files_to_device()
    assert sorted(fb.keys()) == sorted(ref)
    for k, want in ref.items():
        got = fb.get_tensor(k)
        assert got.dtype == want.dtype and tuple(got.shape) == tuple(want.shape), k
        assert bits(got) == bits(want), k
    # conversions of finite values: torch's CPU conversion is a second opinion
    assert bits(fb.get_tensor("l0.q.weight", "F16")) == bits(ref["l0.q.weight"].to(torch.float16))
    assert bits(fb.get_tensor("l1.o.weight", "BF16")) == bits(ref["l1.o.weight"].to(torch.bfloat16))
    assert bits(fb.get_tensor("l0.norm.weight", "F64")) == bits(ref["l0.norm.weight"].to(torch.float64))
    assert bits(fb.get_tensor("l1.scalar", "F32")) == bits(ref["l1.scalar"].to(torch.float32))
    fb.close()
    loader.close()
    sh = SafeTensorsFileLoader(LocalShard(2, 4), torch.device("cuda:0"))
    sh.add_filenames({0: paths})
    fb = sh.copy_files_to_device()
    assert bits(fb.get_sharded("l1.q.weight", 0)) == bits(ref["l1.q.weight"][48:72])          # rows of rank 2 of 4
    assert bits(fb.get_sharded("l0.o.weight", 1)) == bits(ref["l0.o.weight"][:, 48:72])       # columns of rank 2 of 4
    assert bits(fb.get_sharded("l0.q.weight", 0, blocks=3)) == bits(torch.cat([ref["l0.q.weight"][b * 32 + 16:b * 32 + 24]
                                                                              for b in range(3)]))
    assert bits(fb.get_sharded("l1.o.weight", 1, "F32")) == bits(ref["l1.o.weight"][:, 48:72].to(torch.float32))
    fb.close()
    sh.close()


def _specs_of(blobs):
    from oracle import oracle as orc
    out = []
    for b in blobs:
        for t in orc.parse(b, len(b)).tensors:
            out.append((t.name, t.dtype, t.shape))
    # same order as `names` in _case: file by file, in on-disk order
    return out
