"""Pins of the oracle's partition step (paper Section II-A: input projections split column-wise,
output projections row-wise; Section III-B: partitions of the same shape along one dimension) and of
the row-major addressing rule (Section III-A).  Reference: numpy indexing on index-encoded tensors."""
import itertools

import numpy as np
import pytest
import torch

from oracle import oracle as orc

NP = {"U8": np.uint8, "I16": np.int16, "F16": np.float16, "F32": np.float32, "I32": np.int32,
      "I64": np.int64, "F64": np.float64}


def _index_tensor(shape, dt):
    n = int(np.prod(shape)) if len(shape) else 1
    return (np.arange(n, dtype=np.int64) % (250 if dt == "U8" else 30000)).astype(NP[dt]).reshape(shape)


@pytest.mark.parametrize("dt", ["U8", "I16", "F32", "I64"])
@pytest.mark.parametrize("shape", [(24,), (24, 6), (6, 24), (4, 6, 48), (2, 3, 4, 24), (48, 1), (1, 48)])
def test_partition_equals_numpy_indexing(dt, shape):
    a = _index_tensor(shape, dt)
    for d in range(len(shape)):
        for w in (1, 2, 3, 8):
            if shape[d] % w:
                with pytest.raises(orc.OracleError) as e:
                    orc.materialize(a, dt, shape, shard_dim=d, rank=0, world=w)
                assert e.value.kind == "SHARD"
                continue
            per = shape[d] // w
            parts = []
            for r in range(w):
                out, oshape = orc.materialize(a, dt, shape, shard_dim=d, rank=r, world=w)
                sl = [slice(None)] * len(shape)
                sl[d] = slice(r * per, (r + 1) * per)
                ref = np.ascontiguousarray(a[tuple(sl)])
                assert oshape == ref.shape and out.tobytes() == ref.tobytes()
                parts.append(out.view(NP[dt]).reshape(oshape))
            # all ranks together give back the stored tensor
            assert np.array_equal(np.concatenate(parts, axis=d), a)


def test_row_split_element_rule():
    """out[i][j] == T[i][r*C/w + j] on a tensor whose value is its own linear index."""
    R, C, w = 5, 32, 4
    t = np.arange(R * C, dtype=np.int32).reshape(R, C)
    for r in range(w):
        out, oshape = orc.materialize(t, "I32", (R, C), shard_dim=1, rank=r, world=w)
        o = out.view(np.int32).reshape(oshape)
        for i, j in itertools.product(range(R), range(C // w)):
            assert o[i, j] == i * C + r * (C // w) + j


@pytest.mark.parametrize("blocks,world", [(3, 2), (3, 8), (2, 4), (3, 1)])
def test_blocked_partition_is_per_block_partitions_concatenated(blocks, world):
    rows, cols = blocks * world * 2, 5
    a = _index_tensor((rows, cols), "I32")
    subs = np.split(a, blocks, axis=0)
    for r in range(world):
        out, oshape = orc.materialize(a, "I32", (rows, cols), shard_dim=0, blocks=blocks, rank=r, world=world)
        pieces = []
        for s in subs:
            o, _ = orc.materialize(np.ascontiguousarray(s), "I32", s.shape, shard_dim=0, rank=r, world=world)
            pieces.append(o)
        assert out.tobytes() == b"".join(p.tobytes() for p in pieces)
        ref = np.concatenate([np.split(s, world, axis=0)[r] for s in subs], axis=0)
        assert oshape == ref.shape and out.tobytes() == ref.tobytes()
    # 1-D (a fused bias) works the same way
    b = _index_tensor((rows,), "I16")
    out, oshape = orc.materialize(b, "I16", (rows,), shard_dim=0, blocks=blocks, rank=world - 1, world=world)
    ref = np.concatenate([np.split(s, world)[world - 1] for s in np.split(b, blocks)])
    assert out.tobytes() == ref.tobytes() and oshape == ref.shape


def test_cast_and_partition_commute():
    rng = np.random.default_rng(5)
    a = (rng.standard_normal((16, 24)) * 3).astype(np.float32)
    for dst in ("F16", "BF16"):
        whole, _ = orc.materialize(a, "F32", a.shape, dst_dtype=dst)
        for d, w in ((0, 4), (1, 3)):
            for r in range(w):
                cs, oshape = orc.materialize(a, "F32", a.shape, dst_dtype=dst, shard_dim=d, rank=r, world=w)
                sc, oshape2 = orc.materialize(whole.view(np.uint16).reshape(a.shape), dst, a.shape,
                                              shard_dim=d, rank=r, world=w)
                assert oshape == oshape2 and cs.tobytes() == sc.tobytes()
    # and the fused result equals library cast of the library slice
    out, _ = orc.materialize(a, "F32", a.shape, dst_dtype="BF16", shard_dim=1, rank=1, world=2)
    ref = torch.from_numpy(np.ascontiguousarray(a[:, 12:])).to(torch.bfloat16).view(torch.int16).numpy()
    assert out.tobytes() == ref.tobytes()


def test_partition_argument_errors():
    a = _index_tensor((8, 8), "I16")
    bad = [dict(shard_dim=2), dict(shard_dim=0, world=0), dict(shard_dim=0, rank=2, world=2),
           dict(shard_dim=0, rank=-1, world=2), dict(shard_dim=1, blocks=2, world=2),
           dict(shard_dim=-1, blocks=2), dict(shard_dim=0, blocks=3, world=2), dict(shard_dim=0, blocks=0)]
    for kw in bad:
        with pytest.raises(orc.OracleError) as e:
            orc.materialize(a, "I16", (8, 8), **kw)
        assert e.value.kind == "SHARD", kw
    with pytest.raises(orc.OracleError) as e:           # dim 1 of a vector
        orc.materialize(_index_tensor((8,), "I16"), "I16", (8,), shard_dim=1, world=2)
    assert e.value.kind == "SHARD"
    with pytest.raises(orc.OracleError) as e:
        orc.materialize(a, "I16", (8, 8), dst_dtype="F16")
    assert e.value.kind == "CAST"


def test_scalars_and_empty():
    s = np.array(2.5, np.float32)
    out, oshape = orc.materialize(s, "F32", (), dst_dtype="F16")
    assert oshape == () and out.view(np.float16)[0] == np.float16(2.5)
    out, oshape = orc.materialize(np.zeros(0, np.uint8), "F32", (4, 0), shard_dim=0, rank=1, world=2)
    assert oshape == (2, 0) and out.size == 0


def test_threaded_fan_out_matches_single_calls():
    rng = np.random.default_rng(9)
    jobs, refs = [], []
    for i in range(12):
        a = rng.integers(0, 1 << 16, (16, 40), dtype=np.uint16)
        kw = dict(dtype="F16", shape=(16, 40), dst_dtype="BF16", shard_dim=i % 2, rank=i % 4, world=4)
        ref, _ = orc.materialize(a, **kw)
        jobs.append(dict(stored=a.view(np.uint8).reshape(-1), out=np.zeros(ref.nbytes, np.uint8), **kw))
        refs.append(ref)
    orc.materialize_jobs(jobs, 4)
    for j, r in zip(jobs, refs):
        assert j["out"].tobytes() == r.tobytes()


def test_hand_derived_partitions_and_conversions():
    """Partitions and conversions worked out by hand (tests/golden/handmade_partition.txt)."""
    from util_golden import load_fixture
    g = load_fixture("handmade_partition.txt")
    blob = g["file"]
    tab = orc.parse(blob, len(blob))
    assert len(g["parts"]) >= 9
    for nm, dst, dim, blocks, rank, world, shape, want in g["parts"]:
        t = tab.find(nm)
        stored = np.frombuffer(blob, np.uint8, t.end - t.begin, tab.body_off + t.begin)
        out, got_shape = orc.materialize(stored, t.dtype, t.shape, dst, dim, blocks, rank, world)
        assert got_shape == shape and out.tobytes() == want, (nm, dst, dim, blocks, rank, world)
