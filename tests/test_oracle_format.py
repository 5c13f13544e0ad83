"""Pins of the CPU oracle's container reader (paper Section II-A, Fig. 1): hand-typed files, files
made and read by the independent `safetensors` package, the definition "tensor bytes == file bytes at
the stated offsets", and malformed files."""
import json
import os
import struct

import numpy as np
import pytest

from oracle import oracle as orc
from synth import writer
from util_golden import load_fixture


def _name_of(fixture_name: str) -> str:
    # fixture names that are pure hex are byte strings of the decoded key
    try:
        return bytes.fromhex(fixture_name).decode("utf-8") if len(fixture_name) > 4 else fixture_name
    except ValueError:
        return fixture_name


@pytest.mark.parametrize("fx", ["handmade_two.txt", "handmade_odd.txt", "handmade_partition.txt"])
def test_handmade_fixture(fx, tmp_path):
    g = load_fixture(fx)
    blob = g["file"]
    tab = orc.parse(blob, len(blob))
    assert tab.n_json == g["n_json"] and tab.body_off == g["body_off"]
    assert tab.metadata == g["meta"]
    assert len(tab.tensors) == len(g["expect"])
    p = tmp_path / "f.safetensors"
    p.write_bytes(blob)
    for nm, dt, shp, b, e, data in g["expect"]:
        t = tab.find(_name_of(nm))
        assert (t.dtype, t.shape, t.begin, t.end) == (dt, shp, b, e)
        out, oshape, odt = orc.load(str(p), _name_of(nm))
        assert out.tobytes() == data and oshape == shp and odt == dt


def test_header_len_is_little_endian():
    assert orc.header_len(bytes([1, 2, 0, 0, 0, 0, 0, 0])) == 0x0201
    assert orc.header_len(bytes([0, 0, 0, 0, 0, 0, 0, 0x80])) == 1 << 63
    with pytest.raises(orc.OracleError) as e:
        orc.header_len(b"\x01\x02\x03")
    assert e.value.kind == "TRUNCATED"


def _rand_tensors(rng, n=6):
    dts = [("U8", np.uint8), ("I8", np.int8), ("I16", np.int16), ("F16", np.float16), ("F32", np.float32),
           ("I32", np.int32), ("F64", np.float64), ("I64", np.int64), ("BOOL", np.bool_), ("U16", np.uint16)]
    out = []
    for i in range(n):
        nm, npdt = dts[rng.integers(len(dts))]
        shape = tuple(int(x) for x in rng.integers(0, 6, rng.integers(0, 4)))
        a = (rng.standard_normal(shape) * 50).astype(npdt) if npdt != np.bool_ else rng.integers(0, 2, shape).astype(npdt)
        out.append((f"t{i}.w", nm, shape, np.ascontiguousarray(a)))
    return out


@pytest.mark.parametrize("residue", range(16))
def test_bytes_equal_file_bytes_at_every_header_residue(residue, tmp_path):
    """Definition: a materialized tensor (no partition, no conversion) is body[begin:end]."""
    rng = np.random.default_rng(residue)
    ts = _rand_tensors(rng)
    p = str(tmp_path / "r.safetensors")
    blob = writer.write_file(p, [(n, d, s, a.tobytes()) for n, d, s, a in ts], {"k": "v"}, residue)
    tab = orc.parse(blob, len(blob))
    assert tab.body_off % 16 == residue and tab.body_off == 8 + tab.n_json
    assert tab.body_off + tab.body_len == len(blob)
    at = 0
    for t in tab.tensors:                      # contiguous, ordered by offset, exact tiling
        assert t.begin == at
        at = t.end
    assert at == tab.body_len
    for n, d, s, a in ts:
        t = tab.find(n)
        assert (t.dtype, t.shape) == (d, s)
        out, oshape, odt = orc.load(p, n)
        assert out.tobytes() == blob[tab.body_off + t.begin: tab.body_off + t.end] == a.tobytes()


def test_cross_check_with_safetensors_package(tmp_path):
    """An independent implementation writes; the oracle must read what that implementation reads back."""
    st_np = pytest.importorskip("safetensors.numpy")
    st_t = pytest.importorskip("safetensors.torch")
    import torch
    from safetensors import safe_open
    rng = np.random.default_rng(7)
    arrs = {n: a for n, _, _, a in _rand_tensors(rng, 12)}
    p = str(tmp_path / "pkg.safetensors")
    st_np.save_file(arrs, p, metadata={"who": "pkg"})
    blob = open(p, "rb").read()
    tab = orc.parse(blob, len(blob))
    assert tab.metadata == {"who": "pkg"}
    with safe_open(p, framework="np") as f:
        assert sorted(f.keys()) == sorted(t.name for t in tab.tensors)
        for k in f.keys():
            ref = f.get_tensor(k)
            out, oshape, odt = orc.load(p, k)
            assert oshape == tuple(ref.shape)
            assert out.tobytes() == np.ascontiguousarray(ref).tobytes()
    # bfloat16 goes through the torch flavour of the package
    tt = {"x.bf16": torch.randn(5, 7).to(torch.bfloat16), "y.f16": torch.randn(3).to(torch.float16)}
    p2 = str(tmp_path / "pkg2.safetensors")
    st_t.save_file(tt, p2)
    for k, v in tt.items():
        out, oshape, odt = orc.load(p2, k)
        assert odt == {"x.bf16": "BF16", "y.f16": "F16"}[k] and oshape == tuple(v.shape)
        assert out.tobytes() == v.contiguous().view(torch.uint8).numpy().tobytes()


def test_writer_output_is_readable_by_safetensors_package(tmp_path):
    """Pins the test-only writer: the independent package must read back what it wrote."""
    pytest.importorskip("safetensors")
    from safetensors import safe_open
    rng = np.random.default_rng(11)
    ts = [t for t in _rand_tensors(rng, 10)]
    p = str(tmp_path / "w.safetensors")
    writer.write_file(p, [(n, d, s, a.tobytes()) for n, d, s, a in ts], {"a": "b"}, body_residue=5)
    with safe_open(p, framework="np") as f:
        assert f.metadata() == {"a": "b"}
        for n, d, s, a in ts:
            ref = f.get_tensor(n)
            assert ref.shape == s and ref.tobytes() == a.tobytes()


def test_round_trip_writer_oracle_writer(tmp_path):
    rng = np.random.default_rng(3)
    ts = _rand_tensors(rng, 9)
    p = str(tmp_path / "a.safetensors")
    blob = writer.write_file(p, [(n, d, s, a.tobytes()) for n, d, s, a in ts], {"m": "1"}, 9)
    tab = orc.parse(blob, len(blob))
    again = []
    for t in tab.tensors:                         # already in offset order
        out, _, _ = orc.load(p, t.name)
        again.append((t.name, t.dtype, t.shape, out.tobytes()))
    blob2 = writer.write_file(None, again, tab.metadata, 9,
                              order=[[t.name for t in tab.tensors].index(n) for n, _, _, _ in ts])
    assert blob2 == blob


def _file(json_text: bytes, body: bytes = b"", n=None) -> bytes:
    return struct.pack("<Q", len(json_text) if n is None else n) + json_text + body


def _kind(blob, size=None):
    with pytest.raises(orc.OracleError) as e:
        orc.parse(blob, len(blob) if size is None else size)
    return e.value.kind


def test_malformed_files():
    ok = b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}'
    assert orc.parse(_file(ok, b"xy"), len(ok) + 10).tensors[0].name == "a"
    assert _kind(b"\x05\x00\x00") == "TRUNCATED"
    assert _kind(_file(ok, b"xy")[:20], size=len(ok) + 10) == "TRUNCATED"
    assert _kind(_file(ok, b"xy", n=1)) == "HEADER_SIZE"
    assert _kind(_file(ok, b"xy", n=len(ok) + 100)) == "HEADER_SIZE"           # header beyond the file
    assert _kind(_file(ok, b"xy", n=100_000_001), size=1 << 40) == "HEADER_SIZE"
    assert _kind(_file(b' ' + ok, b"xy")) == "JSON"                             # must start with {
    assert _kind(_file(ok[:-1] + b',}', b"xy")) == "JSON"
    assert _kind(_file(ok + b'x', b"xy")) == "JSON"                             # junk after the object
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[02],"data_offsets":[0,2]}}', b"xy")) == "JSON"
    assert _kind(_file(b'{"a\x01":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}', b"xy")) == "JSON"
    assert _kind(_file(b'{"a\xff":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}', b"xy")) == "JSON"
    assert _kind(_file(b'{"a\\ud800":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}', b"xy")) == "JSON"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[-2],"data_offsets":[0,2]}}', b"xy")) == "SCHEMA"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[2.0],"data_offsets":[0,2]}}', b"xy")) == "SCHEMA"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[2e0],"data_offsets":[0,2]}}', b"xy")) == "SCHEMA"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[18446744073709551616],"data_offsets":[0,2]}}', b"xy")) == "SCHEMA"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2],"x":1}}', b"xy")) == "SCHEMA"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[2]}}', b"xy")) == "SCHEMA"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,1,2]}}', b"xy")) == "SCHEMA"
    assert _kind(_file(b'{"a":[1]}', b"")) == "SCHEMA"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[[2]],"data_offsets":[0,2]}}', b"xy")) == "SCHEMA"  # too deep
    assert _kind(_file(b'{"__metadata__":{"k":1}}', b"")) == "SCHEMA"
    assert _kind(_file(b'{"a":{"dtype":"U9","shape":[2],"data_offsets":[0,2]}}', b"xy")) == "DTYPE"
    assert _kind(_file(b'{"a":{"dtype":"I16","shape":[2],"data_offsets":[0,2]}}', b"xy")) == "SIZE_MISMATCH"
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}', b"xyz")) == "OFFSETS"   # tail hole
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[1,3]}}', b"xyz")) == "OFFSETS"   # head hole
    two = b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]},"b":{"dtype":"U8","shape":[2],"data_offsets":[%d,%d]}}'
    assert _kind(_file(two % (1, 3), b"xyz")) == "OFFSETS"                      # overlap
    assert _kind(_file(two % (3, 5), b"xyzvw")) == "OFFSETS"                    # hole
    assert len(orc.parse(_file(two % (2, 4), b"xyzv"), len(two % (2, 4)) + 12).tensors) == 2
    assert _kind(_file(b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[2,0]}}', b"xy")) == "OFFSETS"
    dup = b'{"a":{"dtype":"U8","shape":[1],"data_offsets":[0,1]},"\\u0061":{"dtype":"U8","shape":[1],"data_offsets":[1,2]}}'
    assert _kind(_file(dup, b"xy")) == "DUPLICATE"                              # equal after decoding
    assert _kind(_file(b'{"a":{"dtype":"U8","dtype":"U8","shape":[2],"data_offsets":[0,2]}}', b"xy")) == "DUPLICATE"
    nine = b'{"a":{"dtype":"U8","shape":[1,1,1,1,1,1,1,1,1],"data_offsets":[0,1]}}'
    assert _kind(_file(nine, b"x")) == "RANGE"
    # an empty table is a valid file with an empty body
    assert orc.parse(_file(b"{}"), 10).tensors == []
    assert _kind(_file(b"{}", b"x")) == "OFFSETS"


def test_zero_byte_tensors_sit_on_any_boundary():
    js = (b'{"z0":{"dtype":"F32","shape":[0],"data_offsets":[0,0]},'
          b'"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]},'
          b'"z1":{"dtype":"I64","shape":[3,0,2],"data_offsets":[2,2]}}')
    tab = orc.parse(_file(js, b"xy"), len(js) + 10)
    assert [t.name for t in tab.tensors] == ["z0", "a", "z1"]


def test_load_errors(tmp_path):
    p = tmp_path / "x.safetensors"
    p.write_bytes(_file(b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}', b"xy"))
    with pytest.raises(orc.OracleError) as e:
        orc.load(str(p), "missing")
    assert e.value.kind == "NOT_FOUND"
    with pytest.raises(orc.OracleError) as e:
        orc.load(str(tmp_path / "nope"), "a")
    assert e.value.kind == "IO"
