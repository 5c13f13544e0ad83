"""ctypes access to the CPU oracle (liboracle.so built from fst_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's CPU-baseline
leg.  The GPU path never imports this module.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

MAX_DIMS = 8
DTYPES = ["BOOL", "U8", "I8", "F8_E5M2", "F8_E4M3", "I16", "U16", "F16", "BF16",
          "I32", "U32", "F32", "I64", "U64", "F64"]
ERR = {0: "OK", 1: "TRUNCATED", 2: "HEADER_SIZE", 3: "JSON", 4: "SCHEMA", 5: "DTYPE",
       6: "SIZE_MISMATCH", 7: "OFFSETS", 8: "DUPLICATE", 9: "NOT_FOUND", 10: "SHARD", 11: "CAST",
       12: "RANGE", 13: "IO", 14: "NOMEM"}


class OracleError(Exception):
    def __init__(self, code: int):
        super().__init__(ERR.get(code, str(code)))
        self.code = code
        self.kind = ERR.get(code, str(code))


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "fst_oracle.c")
    hdr = os.path.join(_HERE, "fst_oracle.h")
    newest = max(os.path.getmtime(src), os.path.getmtime(hdr))
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < newest:
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-pthread", "-o", _LIB_PATH, src])
    return _LIB_PATH


class _Tensor(ctypes.Structure):
    _fields_ = [("name", ctypes.c_void_p), ("name_len", ctypes.c_size_t), ("dtype", ctypes.c_int),
                ("ndim", ctypes.c_int), ("shape", ctypes.c_uint64 * MAX_DIMS),
                ("begin", ctypes.c_uint64), ("end", ctypes.c_uint64)]


class _Table(ctypes.Structure):
    _fields_ = [("n_json", ctypes.c_uint64), ("body_off", ctypes.c_uint64), ("body_len", ctypes.c_uint64),
                ("count", ctypes.c_size_t), ("tensors", ctypes.POINTER(_Tensor)),
                ("n_meta", ctypes.c_size_t), ("meta_keys", ctypes.POINTER(ctypes.c_void_p)),
                ("meta_vals", ctypes.POINTER(ctypes.c_void_p))]


class _Job(ctypes.Structure):
    _fields_ = [("stored", ctypes.c_void_p), ("src_dtype", ctypes.c_int), ("ndim", ctypes.c_int),
                ("shape", ctypes.c_uint64 * MAX_DIMS), ("dst_dtype", ctypes.c_int),
                ("shard_dim", ctypes.c_int), ("blocks", ctypes.c_int), ("rank", ctypes.c_int),
                ("world", ctypes.c_int), ("out", ctypes.c_void_p), ("out_cap", ctypes.c_uint64),
                ("rc", ctypes.c_int)]


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        L.orc_parse.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                ctypes.POINTER(ctypes.POINTER(_Table))]
        L.orc_table_free.argtypes = [ctypes.POINTER(_Table)]
        L.orc_header_len.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint64)]
        for fn, a, r in [("orc_bf16_to_f32", ctypes.c_uint16, ctypes.c_uint32),
                         ("orc_f16_to_f32", ctypes.c_uint16, ctypes.c_uint32),
                         ("orc_f32_to_bf16", ctypes.c_uint32, ctypes.c_uint16),
                         ("orc_f32_to_f16", ctypes.c_uint32, ctypes.c_uint16),
                         ("orc_f32_to_f64", ctypes.c_uint32, ctypes.c_uint64),
                         ("orc_f64_to_f32", ctypes.c_uint64, ctypes.c_uint32),
                         ("orc_f64_to_f16", ctypes.c_uint64, ctypes.c_uint16),
                         ("orc_f64_to_bf16", ctypes.c_uint64, ctypes.c_uint16),
                         ("orc_f16_to_f64", ctypes.c_uint16, ctypes.c_uint64),
                         ("orc_bf16_to_f64", ctypes.c_uint16, ctypes.c_uint64),
                         ("orc_f8e5m2_to_f32", ctypes.c_uint8, ctypes.c_uint32),
                         ("orc_f8e4m3_to_f32", ctypes.c_uint8, ctypes.c_uint32)]:
            getattr(L, fn).argtypes = [a]
            getattr(L, fn).restype = r
        L.orc_cast_array.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_void_p]
        L.orc_materialize.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]
        L.orc_result_info.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_void_p]
        L.orc_load.argtypes = [ctypes.c_char_p, ctypes.c_char_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                               ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p,
                               ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int),
                               ctypes.POINTER(ctypes.c_uint64)]
        L.orc_free.argtypes = [ctypes.c_void_p]
        L.orc_materialize_jobs.argtypes = [ctypes.POINTER(_Job), ctypes.c_size_t, ctypes.c_int]
        _lib = L
    return _lib


def dtype_id(name: Optional[str]) -> int:
    return -1 if name is None else DTYPES.index(name)


@dataclass
class TensorEntry:
    name: str
    dtype: str
    shape: Tuple[int, ...]
    begin: int
    end: int


@dataclass
class Table:
    n_json: int
    body_off: int
    body_len: int
    tensors: List[TensorEntry]
    metadata: Dict[str, str]

    def find(self, name: str) -> TensorEntry:
        for t in self.tensors:
            if t.name == name:
                return t
        raise OracleError(9)


def header_len(first8: bytes) -> int:
    n = ctypes.c_uint64()
    rc = lib().orc_header_len(bytes(first8), len(first8), ctypes.byref(n))
    if rc:
        raise OracleError(rc)
    return n.value


def parse(head: bytes, file_size: int) -> Table:
    """head = (at least) the first 8+N bytes of the file."""
    head = bytes(head)
    p = ctypes.POINTER(_Table)()
    rc = lib().orc_parse(head, len(head), file_size, ctypes.byref(p))
    if rc:
        raise OracleError(rc)
    t = p.contents
    ents = []
    for i in range(t.count):
        e = t.tensors[i]
        nm = ctypes.string_at(e.name, e.name_len).decode("utf-8")
        ents.append(TensorEntry(nm, DTYPES[e.dtype], tuple(e.shape[d] for d in range(e.ndim)), e.begin, e.end))
    meta = {}
    for i in range(t.n_meta):
        meta[ctypes.string_at(t.meta_keys[i]).decode("utf-8")] = ctypes.string_at(t.meta_vals[i]).decode("utf-8")
    tab = Table(t.n_json, t.body_off, t.body_len, ents, meta)
    lib().orc_table_free(p)
    return tab


def cast_array(src: np.ndarray, src_dtype: str, dst_dtype: str) -> np.ndarray:
    """src: uint8/uint16/uint32 array of bit patterns; returns the converted bit patterns."""
    src = np.ascontiguousarray(src)
    ss = {"F64": 8, "F32": 4, "F16": 2, "BF16": 2}.get(src_dtype, src.itemsize)
    ds = {"F64": 8, "F32": 4, "F16": 2, "BF16": 2}.get(dst_dtype, ss)
    n = src.nbytes // ss
    out = np.empty(n * ds, np.uint8)
    rc = lib().orc_cast_array(src.ctypes.data, n, dtype_id(src_dtype), dtype_id(dst_dtype), out.ctypes.data)
    if rc:
        raise OracleError(rc)
    return out.view({1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[ds])


def result_info(dtype: str, shape: Sequence[int], dst_dtype: Optional[str] = None, shard_dim: int = -1,
                blocks: int = 1, rank: int = 0, world: int = 1) -> Tuple[Tuple[int, ...], int]:
    sh = (ctypes.c_uint64 * MAX_DIMS)(*shape)
    osh = (ctypes.c_uint64 * MAX_DIMS)()
    nb = ctypes.c_uint64()
    rc = lib().orc_result_info(dtype_id(dtype), len(shape), sh, dtype_id(dst_dtype), shard_dim, blocks,
                               rank, world, osh, ctypes.byref(nb))
    if rc:
        raise OracleError(rc)
    return tuple(osh[d] for d in range(len(shape))), nb.value


def materialize(stored: np.ndarray, dtype: str, shape: Sequence[int], dst_dtype: Optional[str] = None,
                shard_dim: int = -1, blocks: int = 1, rank: int = 0, world: int = 1
                ) -> Tuple[np.ndarray, Tuple[int, ...]]:
    """stored: uint8 array holding the tensor's bytes as they are in the file.  Returns (uint8 array of
    the result, result shape)."""
    if len(shape) > MAX_DIMS:
        raise OracleError(12)
    stored = np.ascontiguousarray(stored).view(np.uint8)
    oshape, nb = result_info(dtype, shape, dst_dtype, shard_dim, blocks, rank, world)
    out = np.empty(nb, np.uint8)
    sh = (ctypes.c_uint64 * MAX_DIMS)(*shape)
    rc = lib().orc_materialize(stored.ctypes.data, dtype_id(dtype), len(shape), sh, dtype_id(dst_dtype),
                               shard_dim, blocks, rank, world, out.ctypes.data, nb, None, None)
    if rc:
        raise OracleError(rc)
    return out, oshape


def load(path: str, name: str, dst_dtype: Optional[str] = None, shard_dim: int = -1, blocks: int = 1,
         rank: int = 0, world: int = 1) -> Tuple[np.ndarray, Tuple[int, ...], str]:
    """The plain reader: file -> one materialized tensor (uint8 bytes, shape, dtype name)."""
    out = ctypes.c_void_p()
    osh = (ctypes.c_uint64 * MAX_DIMS)()
    nd = ctypes.c_int()
    dt = ctypes.c_int()
    nb = ctypes.c_uint64()
    rc = lib().orc_load(path.encode(), name.encode("utf-8"), dtype_id(dst_dtype), shard_dim, blocks, rank,
                        world, ctypes.byref(out), osh, ctypes.byref(nd), ctypes.byref(dt), ctypes.byref(nb))
    if rc:
        raise OracleError(rc)
    arr = np.ctypeslib.as_array(ctypes.cast(out, ctypes.POINTER(ctypes.c_uint8)), shape=(max(nb.value, 1),))
    res = arr[:nb.value].copy()
    lib().orc_free(out)
    return res, tuple(osh[d] for d in range(nd.value)), DTYPES[dt.value]


def materialize_jobs(jobs: Sequence[dict], threads: int) -> None:
    """jobs: dicts with stored (uint8 array), dtype, shape, dst_dtype, shard_dim, blocks, rank, world,
    out (uint8 array).  Runs the scalar oracle over the jobs on `threads` plain threads."""
    arr = (_Job * len(jobs))()
    for j, d in zip(arr, jobs):
        j.stored = d["stored"].ctypes.data
        j.src_dtype = dtype_id(d["dtype"])
        j.ndim = len(d["shape"])
        for i, s in enumerate(d["shape"]):
            j.shape[i] = s
        j.dst_dtype = dtype_id(d.get("dst_dtype"))
        j.shard_dim = d.get("shard_dim", -1)
        j.blocks = d.get("blocks", 1)
        j.rank = d.get("rank", 0)
        j.world = d.get("world", 1)
        j.out = d["out"].ctypes.data
        j.out_cap = d["out"].nbytes
    rc = lib().orc_materialize_jobs(arr, len(jobs), threads)
    if rc:
        raise OracleError(rc)
