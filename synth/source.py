"""Python side of the procedural file source: builds the value pools with a seeded generator and
hands the layout of every file of a ModelSpec to libsynth (source.c)."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional

import numpy as np

from .specs import DTYPE_SIZE, ModelSpec
from .writer import build_header

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
POOL_PRIME = 8388593          # number of elements of every value pool (largest prime < 2^23)
_lib = None


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "source.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-pthread", "-o", _LIB_PATH, src])
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        L.syn_create.restype = ctypes.c_void_p
        L.syn_create.argtypes = [ctypes.c_int32]
        L.syn_set_pool.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_uint64]
        L.syn_set_file.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_uint64,
                                   ctypes.c_int64] + [ctypes.c_void_p] * 7
        L.syn_file_size.restype = ctypes.c_uint64
        L.syn_file_size.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        L.syn_read.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint64, ctypes.c_void_p,
                               ctypes.c_uint64]
        L.syn_write_file.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_char_p, ctypes.c_int32]
        L.syn_free.argtypes = [ctypes.c_void_p]
        _lib = L
    return _lib


def _normal_pool(dtype: str, seed: int) -> np.ndarray:
    """POOL_PRIME samples of N(0, 0.02) stored as `dtype`, as raw bytes (the 8-bit floats: N(0, 1), as weights
    quantized with a scale that brings them into the format's range would look)."""
    import torch
    g = torch.Generator().manual_seed(seed * 1000003 + 17)
    x = torch.randn(POOL_PRIME, generator=g, dtype=torch.float32)
    tdt = {"BF16": torch.bfloat16, "F16": torch.float16, "F32": torch.float32, "F64": torch.float64,
           "F8_E5M2": torch.float8_e5m2, "F8_E4M3": torch.float8_e4m3fn}[dtype]
    if not dtype.startswith("F8_"):
        x = x * 0.02
    return x.to(tdt).view(torch.uint8).numpy().copy()


_ONE = {"BF16": bytes([0x80, 0x3F]), "F16": bytes([0x00, 0x3C]), "F32": bytes([0, 0, 0x80, 0x3F]),
        "F64": bytes([0, 0, 0, 0, 0, 0, 0xF0, 0x3F])}


class ProceduralModel:
    """All files of a ModelSpec as a pure function (file, offset) -> bytes."""

    def __init__(self, spec: ModelSpec):
        L = lib()
        self.spec = spec
        self.handle = ctypes.c_void_p(L.syn_create(len(spec.files)))
        self._pools = {}           # key -> pool id
        self._keep = []
        rng = np.random.default_rng(spec.seed)
        k = 0                      # global tensor index
        self.headers: List[bytes] = []
        self.sizes: List[int] = []
        for fi, fs in enumerate(spec.files):
            entries = [(t.name, t.dtype, t.shape, t.nbytes) for t in fs.tensors]
            head, offs = build_header(entries, None, fs.body_residue)
            n = len(fs.tensors)
            begin = np.zeros(n, np.uint64); end = np.zeros(n, np.uint64)
            kind = np.zeros(n, np.int32); pool = np.zeros(n, np.int32)
            pstart = np.zeros(n, np.uint64); pat = np.zeros(8 * max(n, 1), np.uint8)
            patlen = np.ones(n, np.int32)
            for i, t in enumerate(fs.tensors):
                begin[i] = len(head) + offs[i][0]
                end[i] = len(head) + offs[i][1]
                es = DTYPE_SIZE[t.dtype]
                if t.fill == "ones":
                    kind[i] = 1
                    one = _ONE[t.dtype]
                    pat[8 * i:8 * i + len(one)] = np.frombuffer(one, np.uint8)
                    patlen[i] = len(one)
                else:
                    kind[i] = 0
                    pool[i] = self._pool_id(t.fill, t.dtype, spec.seed, rng)
                    plen_elems = POOL_PRIME if t.fill == "normal" else POOL_PRIME * 1
                    # start inside the pool: a different, element-aligned phase per tensor
                    step = 1299709  # prime
                    unit = es if t.fill == "normal" else 1
                    pstart[i] = ((k * step) % plen_elems) * unit
                k += 1
            rc = L.syn_set_file(self.handle, fi, head, len(head), n, begin.ctypes.data, end.ctypes.data,
                                kind.ctypes.data, pool.ctypes.data, pstart.ctypes.data, pat.ctypes.data,
                                patlen.ctypes.data)
            if rc:
                raise RuntimeError(f"syn_set_file failed: {rc}")
            self.headers.append(head)
            self.sizes.append(int(L.syn_file_size(self.handle, fi)))
        self.read_fn = ctypes.cast(L.syn_read, ctypes.c_void_p).value   # C function pointer
        self.ctx = self.handle.value

    def _pool_id(self, fill: str, dtype: str, seed: int, rng) -> int:
        key = (fill, dtype if fill == "normal" else "")
        if key not in self._pools:
            pid = len(self._pools)
            if fill == "normal":
                b = _normal_pool(dtype, seed)
            elif fill == "bytes":
                b = rng.integers(0, 256, POOL_PRIME, dtype=np.uint8)
            elif fill == "bool":
                b = rng.integers(0, 2, POOL_PRIME, dtype=np.uint8)
            else:
                raise ValueError(fill)
            b = np.ascontiguousarray(b)
            if lib().syn_set_pool(self.handle, pid, b.ctypes.data, b.nbytes):
                raise RuntimeError("syn_set_pool failed")
            self._pools[key] = pid
        return self._pools[key]

    def read(self, fi: int, off: int, length: int, out: Optional[np.ndarray] = None) -> np.ndarray:
        if out is None:
            out = np.empty(length, np.uint8)
        assert out.nbytes >= length and out.flags.c_contiguous
        if lib().syn_read(self.handle, fi, off, out.ctypes.data, length):
            raise ValueError(f"read out of range: file {fi} off {off} len {length}")
        return out[:length]

    def write_file(self, fi: int, path: str, threads: int = 8) -> None:
        if lib().syn_write_file(self.handle, fi, path.encode(), threads):
            raise OSError(f"could not write {path}")

    def write_all(self, directory: str, threads: int = 8) -> List[str]:
        os.makedirs(directory, exist_ok=True)
        paths = []
        for fi, fs in enumerate(self.spec.files):
            p = os.path.join(directory, fs.filename)
            self.write_file(fi, p, threads)
            paths.append(p)
        return paths

    def close(self) -> None:
        if self.handle:
            lib().syn_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
