"""The library's own header parser (host code, no GPU): hand-typed fixtures, agreement with the CPU
oracle on generated and on malformed files (paper Section II-A, Fig. 1)."""
import struct

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2505_23072_amd import binding as B
from synth import writer
from test_oracle_format import _file, _name_of, _rand_tensors
from util_golden import load_fixture

# oracle result class -> library status name
CLASS = {"TRUNCATED": "FST_E_TRUNCATED", "HEADER_SIZE": "FST_E_HEADER_SIZE", "JSON": "FST_E_JSON",
         "SCHEMA": "FST_E_SCHEMA", "DTYPE": "FST_E_DTYPE", "SIZE_MISMATCH": "FST_E_SIZE_MISMATCH",
         "OFFSETS": "FST_E_OFFSETS", "DUPLICATE": "FST_E_DUP_NAME", "RANGE": "FST_E_RANGE"}


@pytest.mark.parametrize("fx", ["handmade_two.txt", "handmade_odd.txt", "handmade_partition.txt"])
def test_handmade_fixture(fx):
    g = load_fixture(fx)
    h = B.Header(g["file"], len(g["file"]))
    assert h.body_offset() == g["body_off"] and h.file_size() == len(g["file"])
    assert h.metadata() == g["meta"]
    assert h.count() == len(g["expect"])
    for nm, dt, shp, b, e, data in g["expect"]:
        t = h.tensor(h.find(_name_of(nm)))
        assert (t["dtype"], t["shape"], t["begin"], t["end"]) == (dt, shp, b, e)
        assert g["file"][g["body_off"] + b: g["body_off"] + e] == data


def test_header_len():
    assert B.fst_header_len(bytes([1, 2, 0, 0, 0, 0, 0, 0])) == 0x0201
    assert B.fst_header_len(bytes([0] * 7 + [0x80])) == 1 << 63
    with pytest.raises(B.FstError) as e:
        B.fst_header_len(b"\x01")
    assert e.value.name == "FST_E_TRUNCATED"


@pytest.mark.parametrize("seed", range(8))
def test_same_table_as_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    ts = _rand_tensors(rng, 10)
    order = list(rng.permutation(len(ts)))
    blob = writer.write_file(None, [(n, d, s, a.tobytes()) for n, d, s, a in ts], {"s": str(seed)},
                             body_residue=int(rng.integers(16)), order=order)
    tab = orc.parse(blob, len(blob))
    h = B.Header(blob[:tab.body_off], len(blob))
    assert h.body_offset() == tab.body_off and h.metadata() == tab.metadata
    mine = h.tensors()
    assert [(t["name"], t["dtype"], t["shape"], t["begin"], t["end"]) for t in mine] == \
           [(t.name, t.dtype, t.shape, t.begin, t.end) for t in tab.tensors]
    for t in tab.tensors:
        assert mine[h.find(t.name)]["name"] == t.name
    with pytest.raises(B.FstError) as e:
        h.find("no such tensor")
    assert e.value.name == "FST_E_NOT_FOUND"


def _both(blob, size=None):
    size = len(blob) if size is None else size
    try:
        orc.parse(blob, size)
        o = "OK"
    except orc.OracleError as e:
        o = e.kind
    try:
        B.Header(blob, size)
        m = "OK"
    except B.FstError as e:
        m = e.name
    return o, m


BAD_JSON = [
    b' {"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]},}',
    b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}x',
    b'{"a":{"dtype":"U8","shape":[02],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2.],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2e],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[-],"data_offsets":[0,2]}}',
    b'{"a\x01":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a\xff":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a\xc0\x80":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a\xed\xa0\x80":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a\xf4\x90\x80\x80":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a\\ud800":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a\\udc00":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a\\x":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}',
    b'{"a" {"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{a:{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8" "shape":[2],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2 3],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2,],"data_offsets":[0,2]}}',
]
BAD_SCHEMA = [
    b'{"a":{"dtype":"U8","shape":[-2],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2.0],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2e0],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[18446744073709551616],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2],"x":1}}',
    b'{"a":{"dtype":"U8","shape":[2]}}',
    b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,1,2]}}',
    b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0]}}',
    b'{"a":[1]}',
    b'{"a":"x"}',
    b'{"a":7}',
    b'{"a":null}',
    b'{"a":{}}',
    b'{"a":{"dtype":7,"shape":[2],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":2,"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":["2"],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[true],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[[2]],"data_offsets":[0,2]}}',
    b'{"a":{"dtype":"U8","shape":[{}],"data_offsets":[0,2]}}',
    b'{"__metadata__":{"k":1}}',
    b'{"__metadata__":["k"]}',
]
OTHER = [
    (b'{"a":{"dtype":"U9","shape":[2],"data_offsets":[0,2]}}', b"xy", "DTYPE"),
    (b'{"a":{"dtype":"","shape":[2],"data_offsets":[0,2]}}', b"xy", "DTYPE"),
    (b'{"a":{"dtype":"I16","shape":[2],"data_offsets":[0,2]}}', b"xy", "SIZE_MISMATCH"),
    (b'{"a":{"dtype":"U8","shape":[4294967296,4294967296],"data_offsets":[0,2]}}', b"xy", "SIZE_MISMATCH"),
    (b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}', b"xyz", "OFFSETS"),
    (b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[1,3]}}', b"xyz", "OFFSETS"),
    (b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[2,0]}}', b"xy", "OFFSETS"),
    (b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]},"b":{"dtype":"U8","shape":[2],"data_offsets":[1,3]}}', b"xyz", "OFFSETS"),
    (b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]},"b":{"dtype":"U8","shape":[2],"data_offsets":[3,5]}}', b"xyzvw", "OFFSETS"),
    (b'{}', b"x", "OFFSETS"),
    (b'{"a":{"dtype":"U8","shape":[1],"data_offsets":[0,1]},"\\u0061":{"dtype":"U8","shape":[1],"data_offsets":[1,2]}}', b"xy", "DUPLICATE"),
    (b'{"a":{"dtype":"U8","dtype":"U8","shape":[2],"data_offsets":[0,2]}}', b"xy", "DUPLICATE"),
    (b'{"__metadata__":{"k":"1","k":"2"}}', b"", "DUPLICATE"),
    (b'{"__metadata__":{},"__metadata__":{}}', b"", "DUPLICATE"),
    (b'{"a":{"dtype":"U8","shape":[1,1,1,1,1,1,1,1,1],"data_offsets":[0,1]}}', b"x", "RANGE"),
]


def test_malformed_files_get_the_same_class_as_the_oracle():
    for js in BAD_JSON:
        assert _both(_file(js, b"xy")) == ("JSON", "FST_E_JSON"), js
    for js in BAD_SCHEMA:
        assert _both(_file(js, b"xy")) == ("SCHEMA", "FST_E_SCHEMA"), js
    for js, body, kind in OTHER:
        assert _both(_file(js, body)) == (kind, CLASS[kind]), js
    ok = b'{"a":{"dtype":"U8","shape":[2],"data_offsets":[0,2]}}'
    assert _both(_file(ok, b"xy")) == ("OK", "OK")
    assert _both(b"\x05\x00\x00") == ("TRUNCATED", "FST_E_TRUNCATED")
    assert _both(_file(ok, b"xy")[:20], len(ok) + 10) == ("TRUNCATED", "FST_E_TRUNCATED")
    assert _both(_file(ok, b"xy", n=1)) == ("HEADER_SIZE", "FST_E_HEADER_SIZE")
    assert _both(_file(ok, b"xy", n=len(ok) + 100)) == ("HEADER_SIZE", "FST_E_HEADER_SIZE")
    assert _both(_file(ok, b"xy", n=100_000_001), 1 << 40) == ("HEADER_SIZE", "FST_E_HEADER_SIZE")
    assert _both(_file(ok, b"xy", n=(1 << 64) - 4), 1 << 40) == ("HEADER_SIZE", "FST_E_HEADER_SIZE")
    assert _both(_file(b"{}")) == ("OK", "OK")
    # valid corner cases both accept: white space everywhere, escapes, empty shape
    js = b'{ "a\\n\\t\\u00e9\\ud83d\\ude00" : { "shape" : [ ] , "data_offsets" : [ 0 , 4 ] , "dtype" : "F32" } }  \n'
    assert _both(_file(js, b"abcd")) == ("OK", "OK")
    h = B.Header(_file(js, b"abcd"), len(js) + 12)
    assert h.tensor(0)["name"] == "a\n\té\U0001F600" == orc.parse(_file(js, b"abcd"), len(js) + 12).tensors[0].name


def test_random_mutations_never_crash_and_agree_on_acceptance():
    """Byte flips of a valid header: both readers must agree on accept / reject."""
    rng = np.random.default_rng(42)
    ts = _rand_tensors(rng, 5)
    blob = bytearray(writer.write_file(None, [(n, d, s, a.tobytes()) for n, d, s, a in ts], {"k": "v"}, 4))
    n = struct.unpack("<Q", blob[:8])[0]
    agree = 0
    for _ in range(3000):
        b2 = bytearray(blob)
        for _ in range(int(rng.integers(1, 3))):
            b2[8 + int(rng.integers(n))] = int(rng.integers(256))
        o, m = _both(bytes(b2))
        assert (o == "OK") == (m == "OK"), bytes(b2[8:8 + n])
        agree += 1
    assert agree == 3000
