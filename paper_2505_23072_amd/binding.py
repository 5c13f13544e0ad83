"""Thin ctypes binding of libfst.so: the same names as include/fst.h, argument marshalling only.

Every step of the path (header parsing, planning, staging, the kernels) runs inside the library;
PyTorch appears only in `device.py`, for device memory and streams.  If the library is missing the
import fails loudly: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char_p, c_double, c_int, c_int32, c_int64, c_size_t,
                    c_uint32, c_uint64, c_void_p)
from typing import Dict, List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
# FST_LIBRARY names another build of the same ABI (the tests use it for a sanitizer build of the host parts)
LIB_PATH = os.environ.get("FST_LIBRARY") or os.path.join(_HERE, "libfst.so")

FST_MAX_DIMS = 8
FST_OUTPUT_ALIGN = 256
FST_RAW_ALIGN = 256
FST_ALL_GROUPS = ctypes.c_size_t(-1).value
FST_KEEP = -1
FST_STAGE_NO_KERNELS = 1
FST_STAGE_NO_READ = 2

DTYPE_NAMES = ["F64", "F32", "F16", "BF16", "F8_E5M2", "F8_E4M3", "I64", "I32", "I16", "I8",
               "U64", "U32", "U16", "U8", "BOOL"]


class fst_tensor_info(Structure):
    _fields_ = [("name", c_void_p), ("name_len", c_size_t), ("dtype", c_int32), ("ndim", c_int32),
                ("shape", c_uint64 * FST_MAX_DIMS), ("begin", c_uint64), ("end", c_uint64)]


class fst_request(Structure):
    _fields_ = [("dst_dtype", c_int32), ("shard_dim", c_int32), ("blocks", c_int32), ("rank", c_int32)]


class fst_output_info(Structure):
    _fields_ = [("dtype", c_int32), ("ndim", c_int32), ("shape", c_uint64 * FST_MAX_DIMS),
                ("nbytes", c_uint64), ("align", c_uint32), ("file", c_uint32)]


class fst_group_info(Structure):
    _fields_ = [("file", c_uint32), ("n_descriptors", c_uint32), ("n_extents", c_uint32), ("reserved", c_uint32),
                ("lo", c_uint64), ("hi", c_uint64), ("slot_bytes", c_uint64), ("staged_bytes", c_uint64),
                ("read_bytes", c_uint64), ("write_bytes", c_uint64), ("packed_offset", c_uint64)]


class fst_extent(Structure):
    _fields_ = [("lo", c_uint64), ("hi", c_uint64), ("slot_offset", c_uint64), ("row_bytes", c_uint64),
                ("n_rows", c_uint64), ("stride", c_uint64)]


class fst_descriptor(Structure):
    _fields_ = [("output", c_uint32), ("file", c_uint32), ("group", c_uint32), ("src_dtype", c_int32),
                ("dst_dtype", c_int32), ("src_file_off", c_uint64), ("src_stride", c_uint64),
                ("dst_off", c_uint64), ("row_elems", c_uint64), ("n_rows", c_uint64)]


class fst_stager_config(Structure):
    _fields_ = [("n_slots", c_uint32), ("n_threads", c_uint32), ("slot_bytes", c_uint64)]


class fst_stage_stats(Structure):
    _fields_ = [("staged_bytes", c_uint64), ("n_copies", c_uint64), ("seconds_total", c_double),
                ("seconds_read", c_double)]


fst_read_fn = ctypes.CFUNCTYPE(c_int, c_void_p, c_int32, c_uint64, c_void_p, c_uint64)

_SIGNATURES = {
    "fst_last_error": (c_char_p, []),
    "fst_status_name": (c_char_p, [c_int]),
    "fst_dtype_name": (c_char_p, [c_int]),
    "fst_dtype_from_name": (c_int, [c_char_p, c_size_t]),
    "fst_dtype_size": (c_size_t, [c_int]),
    "fst_header_len": (c_int, [c_void_p, c_size_t, POINTER(c_uint64)]),
    "fst_parse_header": (c_int, [c_void_p, c_size_t, c_uint64, POINTER(c_void_p)]),
    "fst_header_count": (c_size_t, [c_void_p]),
    "fst_header_tensor": (c_int, [c_void_p, c_size_t, POINTER(fst_tensor_info)]),
    "fst_header_find": (c_int64, [c_void_p, c_char_p]),
    "fst_header_body_offset": (c_uint64, [c_void_p]),
    "fst_aligned_phase": (c_uint64, [c_void_p]),
    "fst_header_file_size": (c_uint64, [c_void_p]),
    "fst_header_metadata_count": (c_size_t, [c_void_p]),
    "fst_header_metadata": (c_int, [c_void_p, c_size_t, POINTER(c_char_p), POINTER(c_char_p)]),
    "fst_header_free": (None, [c_void_p]),
    "fst_plan_create": (c_int, [POINTER(c_void_p), POINTER(c_uint64), c_size_t, POINTER(c_char_p),
                                POINTER(fst_request), c_size_t, c_int32, c_int32, POINTER(c_void_p)]),
    "fst_plan_uniform": (c_int, [POINTER(c_void_p), POINTER(c_uint64), c_size_t, POINTER(c_char_p), c_size_t,
                                 c_int32, c_int32, c_int32, c_int32, POINTER(c_void_p)]),
    "fst_plan_output_count": (c_size_t, [c_void_p]),
    "fst_plan_output": (c_int, [c_void_p, c_size_t, POINTER(fst_output_info)]),
    "fst_plan_set_groups": (c_int, [c_void_p, c_uint64, POINTER(c_size_t)]),
    "fst_plan_set_groups_sparse": (c_int, [c_void_p, c_uint64, c_uint64, POINTER(c_size_t)]),
    "fst_plan_set_groups_compact": (c_int, [c_void_p, c_uint64, c_uint64, c_uint64, POINTER(c_size_t)]),
    "fst_plan_packed_bytes": (c_uint64, [c_void_p]),
    "fst_plan_group_extent": (c_int, [c_void_p, c_size_t, c_size_t, POINTER(fst_extent)]),
    "fst_plan_group_count": (c_size_t, [c_void_p]),
    "fst_plan_group": (c_int, [c_void_p, c_size_t, POINTER(fst_group_info)]),
    "fst_plan_descriptor_count": (c_size_t, [c_void_p]),
    "fst_plan_descriptor": (c_int, [c_void_p, c_size_t, POINTER(fst_descriptor)]),
    "fst_plan_read_bytes": (c_uint64, [c_void_p]),
    "fst_plan_write_bytes": (c_uint64, [c_void_p]),
    "fst_plan_workspace_bytes": (c_size_t, [c_void_p]),
    "fst_plan_free": (None, [c_void_p]),
    "fst_materialize": (c_int, [c_void_p, c_size_t, c_void_p, c_size_t, POINTER(c_void_p), c_void_p, c_size_t,
                                c_void_p]),
    "fst_materialize_slot": (c_int, [c_void_p, c_size_t, c_void_p, c_size_t, POINTER(c_void_p), c_void_p,
                                     c_size_t, c_void_p]),
    "fst_materialize_static": (c_int, [c_void_p, c_size_t, c_void_p, c_size_t, POINTER(c_void_p), c_void_p]),
    "fst_prepare": (c_int, [c_void_p, c_size_t, c_int32, c_size_t, POINTER(c_void_p), c_void_p, c_size_t, c_void_p]),
    "fst_launch": (c_int, [c_void_p, c_size_t, c_void_p, c_size_t, c_void_p]),
    "fst_stager_create": (c_int, [POINTER(fst_stager_config), POINTER(c_void_p)]),
    "fst_stager_destroy": (None, [c_void_p]),
    "fst_read_fds": (c_int, [c_void_p, c_int32, c_uint64, c_void_p, c_uint64]),
    "fst_stage_resident": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, POINTER(c_void_p),
                                   c_void_p, c_size_t, c_uint32, POINTER(fst_stage_stats)]),
    "fst_stage_packed": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, POINTER(c_void_p),
                                 c_void_p, c_size_t, c_uint32, POINTER(fst_stage_stats)]),
    "fst_stage_streamed": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, POINTER(c_void_p), c_size_t, c_size_t,
                                   POINTER(c_void_p), c_void_p, c_size_t, c_uint32, POINTER(fst_stage_stats)]),
}

_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Loads what is built; builds only if nothing is."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)      # AttributeError here = the library misses a declared symbol
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


class FstError(RuntimeError):
    def __init__(self, status: int):
        L = lib()
        self.status = status
        self.name = L.fst_status_name(status).decode()
        super().__init__(f"{self.name}: {L.fst_last_error().decode(errors='replace')}")


def _check(status: int) -> None:
    if status != 0:
        raise FstError(status)


def fst_dtype(name: Optional[str]) -> int:
    return FST_KEEP if name is None else DTYPE_NAMES.index(name)


def fst_header_len(first8: bytes) -> int:
    n = c_uint64()
    _check(lib().fst_header_len(bytes(first8), len(first8), byref(n)))
    return n.value


class Header:
    """Owner of one fst_header."""

    def __init__(self, head: bytes, file_size: int):
        self._h = c_void_p()
        head = bytes(head)
        _check(lib().fst_parse_header(head, len(head), file_size, byref(self._h)))

    @property
    def handle(self) -> c_void_p:
        return self._h

    def count(self) -> int:
        return lib().fst_header_count(self._h)

    def tensor(self, i: int) -> dict:
        ti = fst_tensor_info()
        _check(lib().fst_header_tensor(self._h, i, byref(ti)))
        return dict(name=ctypes.string_at(ti.name, ti.name_len).decode("utf-8"), dtype=DTYPE_NAMES[ti.dtype],
                    shape=tuple(ti.shape[d] for d in range(ti.ndim)), begin=ti.begin, end=ti.end)

    def tensors(self) -> List[dict]:
        return [self.tensor(i) for i in range(self.count())]

    def find(self, name: str) -> int:
        r = lib().fst_header_find(self._h, name.encode("utf-8"))
        if r < 0:
            raise FstError(int(r))
        return int(r)

    def body_offset(self) -> int:
        return lib().fst_header_body_offset(self._h)

    def aligned_phase(self) -> int:
        return lib().fst_aligned_phase(self._h)

    def file_size(self) -> int:
        return lib().fst_header_file_size(self._h)

    def metadata(self) -> Dict[str, str]:
        out = {}
        for i in range(lib().fst_header_metadata_count(self._h)):
            k, v = c_char_p(), c_char_p()
            _check(lib().fst_header_metadata(self._h, i, byref(k), byref(v)))
            out[k.value.decode("utf-8")] = v.value.decode("utf-8")
        return out

    def close(self) -> None:
        if self._h:
            lib().fst_header_free(self._h)
            self._h = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# (dst dtype name or None, shard_dim, blocks) or (dst dtype, shard_dim, blocks, rank of this request)
Request = Tuple


class Requests:
    """Names and requests marshalled once into the C arrays fst_plan_create takes: a caller that plans the same
    request set again (every step of a benchmark, every reload of a model) passes this instead of the lists."""

    def __init__(self, names: Sequence[str], requests: Sequence[Request]):
        n = len(names)
        self.names = list(names)
        self.n = n
        self.name_array = (c_char_p * max(n, 1))(*[s.encode("utf-8") for s in names])
        self.request_array = (fst_request * max(n, 1))()
        for i, r in enumerate(requests):
            self.request_array[i] = fst_request(fst_dtype(r[0]), r[1], r[2], r[3] if len(r) > 3 else -1)


class Plan:
    """Owner of one fst_plan."""

    def __init__(self, headers: Sequence[Header], raw_base: Sequence[int], names, requests: Optional[Sequence[Request]] = None,
                 rank: int = 0, world: int = 1):
        """names: a sequence of tensor names with `requests` beside it, or a Requests object holding both."""
        m = names if isinstance(names, Requests) else Requests(names, requests)
        n_files = len(headers)
        hs = (c_void_p * n_files)(*[h.handle for h in headers])
        rb = (c_uint64 * n_files)(*raw_base)
        self._p = c_void_p()
        _check(lib().fst_plan_create(hs, rb, n_files, m.name_array, m.request_array, m.n, rank, world, byref(self._p)))
        self.names = m.names

    @classmethod
    def uniform(cls, headers: Sequence[Header], raw_base: Sequence[int], names: Sequence[str],
                dst_dtype: Optional[str] = None, shard_dim: int = -1, rank: int = 0, world: int = 1) -> "Plan":
        self = cls.__new__(cls)
        n_files, n = len(headers), len(names)
        hs = (c_void_p * n_files)(*[h.handle for h in headers])
        rb = (c_uint64 * n_files)(*raw_base)
        nm = (c_char_p * max(n, 1))(*[s.encode("utf-8") for s in names])
        self._p = c_void_p()
        _check(lib().fst_plan_uniform(hs, rb, n_files, nm, n, fst_dtype(dst_dtype), shard_dim, rank, world,
                                      byref(self._p)))
        self.names = list(names)
        return self

    @property
    def handle(self) -> c_void_p:
        return self._p

    def output_count(self) -> int:
        return lib().fst_plan_output_count(self._p)

    def output(self, i: int) -> dict:
        oi = fst_output_info()
        _check(lib().fst_plan_output(self._p, i, byref(oi)))
        return dict(dtype=DTYPE_NAMES[oi.dtype], shape=tuple(oi.shape[d] for d in range(oi.ndim)),
                    nbytes=oi.nbytes, align=oi.align, file=oi.file)

    def set_groups(self, max_group_bytes: int, min_gap_bytes: Optional[int] = None,
                   min_segment_bytes: Optional[int] = None) -> int:
        """min_gap_bytes given: do not stage unread file ranges longer than that.  min_segment_bytes given:
        stage the row segments of strided shares one by one, back to back, when they are at least that long."""
        n = c_size_t()
        if min_segment_bytes is not None:
            gap = ctypes.c_uint64(-1).value if min_gap_bytes is None else min_gap_bytes
            _check(lib().fst_plan_set_groups_compact(self._p, max_group_bytes, gap, min_segment_bytes, byref(n)))
        elif min_gap_bytes is None:
            _check(lib().fst_plan_set_groups(self._p, max_group_bytes, byref(n)))
        else:
            _check(lib().fst_plan_set_groups_sparse(self._p, max_group_bytes, min_gap_bytes, byref(n)))
        return n.value

    def packed_bytes(self) -> int:
        return lib().fst_plan_packed_bytes(self._p)

    def group_count(self) -> int:
        return lib().fst_plan_group_count(self._p)

    def group(self, g: int) -> dict:
        gi = fst_group_info()
        _check(lib().fst_plan_group(self._p, g, byref(gi)))
        out = {k: getattr(gi, k) for k, _ in fst_group_info._fields_}
        out["extents"] = []           # (lo, hi, slot_offset)
        out["extent_rows"] = []       # (row_bytes, n_rows, stride): n_rows > 1 = compacted
        for i in range(gi.n_extents):
            e = fst_extent()
            _check(lib().fst_plan_group_extent(self._p, g, i, byref(e)))
            out["extents"].append((e.lo, e.hi, e.slot_offset))
            out["extent_rows"].append((e.row_bytes, e.n_rows, e.stride))
        return out

    def descriptor_count(self) -> int:
        return lib().fst_plan_descriptor_count(self._p)

    def descriptor(self, i: int) -> dict:
        d = fst_descriptor()
        _check(lib().fst_plan_descriptor(self._p, i, byref(d)))
        out = {k: getattr(d, k) for k, _ in fst_descriptor._fields_}
        out["src_dtype"] = DTYPE_NAMES[d.src_dtype]
        out["dst_dtype"] = DTYPE_NAMES[d.dst_dtype]
        return out

    def read_bytes(self) -> int:
        return lib().fst_plan_read_bytes(self._p)

    def write_bytes(self) -> int:
        return lib().fst_plan_write_bytes(self._p)

    def workspace_bytes(self) -> int:
        return lib().fst_plan_workspace_bytes(self._p)

    def close(self) -> None:
        if self._p:
            lib().fst_plan_free(self._p)
            self._p = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _ptr_array(ptrs: Sequence[int]):
    return (c_void_p * max(len(ptrs), 1))(*[c_void_p(p) for p in ptrs])


def fst_materialize(raw_ptr: int, raw_len: int, plan: Plan, group: int, out_ptrs: Sequence[int], workspace_ptr: int,
                    workspace_len: int, stream: int = 0) -> None:
    """raw_ptr / out_ptrs / workspace_ptr: device addresses; stream: a hipStream_t as an integer."""
    _check(lib().fst_materialize(c_void_p(raw_ptr), raw_len, plan.handle, group, _ptr_array(out_ptrs),
                                 c_void_p(workspace_ptr), workspace_len, c_void_p(stream)))


def fst_materialize_slot(slot_ptr: int, slot_len: int, plan: Plan, group: int, out_ptrs: Sequence[int],
                         workspace_ptr: int, workspace_len: int, stream: int = 0) -> None:
    _check(lib().fst_materialize_slot(c_void_p(slot_ptr), slot_len, plan.handle, group, _ptr_array(out_ptrs),
                                      c_void_p(workspace_ptr), workspace_len, c_void_p(stream)))


FST_STATIC_WORKSPACE_BYTES = 4 << 20


def fst_materialize_static(raw_ptr: int, raw_len: int, plan: Plan, group: int, out_ptrs: Sequence[int],
                           stream: int = 0) -> None:
    """fst_materialize with the library's built-in workspace: no device allocation anywhere."""
    _check(lib().fst_materialize_static(c_void_p(raw_ptr), raw_len, plan.handle, group, _ptr_array(out_ptrs),
                                        c_void_p(stream)))


FST_LAYOUT_RESIDENT, FST_LAYOUT_SLOT, FST_LAYOUT_PACKED = 0, 1, 2


def fst_prepare(plan: Plan, group: int, layout: int, src_len: int, out_ptrs: Sequence[int], workspace_ptr: int,
                workspace_len: int, stream: int = 0) -> None:
    _check(lib().fst_prepare(plan.handle, group, layout, src_len, _ptr_array(out_ptrs), c_void_p(workspace_ptr),
                             workspace_len, c_void_p(stream)))


def fst_launch(plan: Plan, group: int, src_ptr: int, src_len: int, stream: int = 0) -> None:
    _check(lib().fst_launch(plan.handle, group, c_void_p(src_ptr), src_len, c_void_p(stream)))


class Stager:
    """Owner of one fst_stager (pinned ring + two streams)."""

    def __init__(self, n_slots: int = 0, n_threads: int = 0, slot_bytes: int = 0):
        cfg = fst_stager_config(n_slots, n_threads, slot_bytes)
        self._s = c_void_p()
        _check(lib().fst_stager_create(byref(cfg), byref(self._s)))

    def stage_resident(self, plan: Plan, read_fn: int, read_ctx: int, raw_ptr: int, raw_len: int,
                       out_ptrs: Sequence[int], workspace_ptr: int, workspace_len: int, flags: int = 0) -> dict:
        """read_fn: address of a C function with the fst_read_fn signature (0 with FST_STAGE_NO_READ)."""
        st = fst_stage_stats()
        _check(lib().fst_stage_resident(self._s, plan.handle, c_void_p(read_fn), c_void_p(read_ctx),
                                        c_void_p(raw_ptr), raw_len, _ptr_array(out_ptrs), c_void_p(workspace_ptr),
                                        workspace_len, flags, byref(st)))
        return {k: getattr(st, k) for k, _ in fst_stage_stats._fields_}

    def stage_packed(self, plan: Plan, read_fn: int, read_ctx: int, packed_ptr: int, packed_len: int,
                     out_ptrs: Sequence[int], workspace_ptr: int, workspace_len: int, flags: int = 0) -> dict:
        st = fst_stage_stats()
        _check(lib().fst_stage_packed(self._s, plan.handle, c_void_p(read_fn), c_void_p(read_ctx),
                                      c_void_p(packed_ptr), packed_len, _ptr_array(out_ptrs), c_void_p(workspace_ptr),
                                      workspace_len, flags, byref(st)))
        return {k: getattr(st, k) for k, _ in fst_stage_stats._fields_}

    def stage_streamed(self, plan: Plan, read_fn: int, read_ctx: int, slot_ptrs: Sequence[int], slot_bytes: int,
                       out_ptrs: Sequence[int], workspace_ptr: int, workspace_len: int, flags: int = 0) -> dict:
        st = fst_stage_stats()
        _check(lib().fst_stage_streamed(self._s, plan.handle, c_void_p(read_fn), c_void_p(read_ctx),
                                        _ptr_array(slot_ptrs), len(slot_ptrs), slot_bytes, _ptr_array(out_ptrs),
                                        c_void_p(workspace_ptr), workspace_len, flags, byref(st)))
        return {k: getattr(st, k) for k, _ in fst_stage_stats._fields_}

    def close(self) -> None:
        if self._s:
            lib().fst_stager_destroy(self._s)
            self._s = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def read_fds_fn() -> int:
    """Address of the library's pread callback; its ctx is a C array of file descriptors."""
    return ctypes.cast(lib().fst_read_fds, c_void_p).value
