"""The C-ABI library loads without a GPU and exports every symbol include/fst.h declares."""
import ctypes
import os
import re

from paper_2505_23072_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "fst.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(fst_[a-z0-9_]+)\s*\(", text))
    names.discard("fst_read_fn")
    return sorted(names)


def test_every_declared_symbol_is_exported():
    L = ctypes.CDLL(B.LIB_PATH)
    names = _declared_functions()
    assert len(names) >= 30
    for n in names:
        assert hasattr(L, n), f"{n} is declared in fst.h but not exported"


def test_binding_covers_every_declared_symbol():
    assert sorted(B._SIGNATURES) == _declared_functions()
    B.lib()


def test_struct_sizes_match_the_header():
    # sizes follow from the field lists in fst.h (natural alignment, 8-byte max)
    assert ctypes.sizeof(B.fst_tensor_info) == 8 + 8 + 4 + 4 + 64 + 8 + 8
    assert ctypes.sizeof(B.fst_request) == 16
    assert ctypes.sizeof(B.fst_output_info) == 4 + 4 + 64 + 8 + 4 + 4
    assert ctypes.sizeof(B.fst_group_info) == 4 * 4 + 8 * 7
    assert ctypes.sizeof(B.fst_extent) == 48
    assert ctypes.sizeof(B.fst_descriptor) == 12 + 8 + 4 + 8 * 5
    assert ctypes.sizeof(B.fst_stager_config) == 16
    assert ctypes.sizeof(B.fst_stage_stats) == 32


def test_dtype_table():
    L = B.lib()
    sizes = {"F64": 8, "F32": 4, "F16": 2, "BF16": 2, "F8_E5M2": 1, "F8_E4M3": 1, "I64": 8, "I32": 4, "I16": 2,
             "I8": 1, "U64": 8, "U32": 4, "U16": 2, "U8": 1, "BOOL": 1}
    for i, n in enumerate(B.DTYPE_NAMES):
        assert L.fst_dtype_name(i).decode() == n
        assert L.fst_dtype_size(i) == sizes[n]
        assert L.fst_dtype_from_name(n.encode(), len(n)) == i
    assert L.fst_dtype_from_name(b"F12", 3) < 0
    assert L.fst_dtype_name(99) is None and L.fst_dtype_size(-1) == 0
    assert L.fst_status_name(-10).decode() == "FST_E_SHARD"
