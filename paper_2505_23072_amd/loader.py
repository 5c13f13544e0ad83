"""Loader API in the shape of the paper's (Section III-C, Figs. 8 and 9):

    loader = SafeTensorsFileLoader(SingleGroup(), torch.device("cuda:0"))
    loader.add_filenames({0: ["a.safetensors"]})
    fb = loader.copy_files_to_device()
    t = fb.get_tensor("a0")
    s = fb.get_sharded("b0", dim=1)
    fb.close(); loader.close()

Two ways to use it.

*As in the paper*: `copy_files_to_device` stages the files verbatim into one raw HBM buffer through the
pinned ring; `get_tensor` / `get_sharded` / `get_many` then run the materialize kernels on that buffer
and return aligned tensors of their own.  A call only enqueues work on the current stream (tables go
into the library's built-in workspace, so nothing but the outputs is allocated) and does not wait: the
tensors are ordered on that stream like the results of any other kernel.  The raw buffer is released by
`close`, or automatically once every key has been fetched.

*With the requests declared first* (`add_requests`): the loader then knows which bytes this rank reads, so
it stages only those (the other ranks' shares stay on the host side of the bus; row segments of
partitions along an inner dimension are read one by one and staged back to back) and materializes every
group as soon as its bytes have landed, overlapped with the copies of the next.  `get_tensor` /
`get_sharded` then return the finished tensors.  With `stream_slots=(n, bytes)` the staged bytes pass
through a ring of n device slots instead of staying resident, which loads a checkpoint larger than device
memory.

One GPU only: a group says which rank's share this GPU takes, nothing is sent anywhere.  This module only
marshals; parsing, planning, staging and the kernels are in libfst.so.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import binding as B
from . import device as D

Request = Tuple[Optional[str], int, int]      # (target dtype name or None, shard dim or -1, blocks)

# The library's built-in workspace is one per GPU: calls that use it must not overlap.  Calls on one
# stream are ordered by the stream; a call on another stream first waits for the previous one.
_last_static_call: Dict[int, Tuple[int, "torch.cuda.Event"]] = {}


def _order_static_call(stream: "torch.cuda.Stream") -> None:
    last = _last_static_call.get(stream.device.index or 0)
    if last is not None and last[0] != stream.cuda_stream:
        stream.wait_event(last[1])


class SingleGroup:
    """The one-GPU process group of Fig. 8: rank 0 of 1."""

    def rank(self) -> int:
        return 0

    def size(self) -> int:
        return 1


class LocalShard(SingleGroup):
    """Take rank `rank`'s share of a `world`-way tensor-parallel split on this GPU (no communication)."""

    def __init__(self, rank: int, world: int):
        if not 0 <= rank < world:
            raise ValueError("rank must be inside world")
        self._rank, self._world = rank, world

    def rank(self) -> int:
        return self._rank

    def size(self) -> int:
        return self._world


class FilesBufferOnDevice:
    """What `copy_files_to_device` returns: the lookup from key to tensor (Section III-C), over the raw
    bytes of the files in HBM and/or the tensors already materialized from declared requests."""

    def __init__(self, headers, bases, raw, raw_len, group, auto_release, ready=None, ready_requests=None,
                 staged_bytes=0):
        self._headers, self._bases = headers, bases
        self._raw, self._raw_len, self._group = raw, raw_len, group
        self._auto = auto_release
        self._ready: Dict[str, torch.Tensor] = ready or {}
        self._ready_requests: Dict[str, Request] = ready_requests or {}
        self._pending = {t["name"] for h in headers for t in h.tensors()} - set(self._ready)
        self._in_flight: List[Tuple[B.Plan, torch.cuda.Event, Optional[torch.Tensor]]] = []
        self.key_to_file = {t["name"]: i for i, h in enumerate(headers) for t in h.tensors()}
        self.staged_bytes = staged_bytes          # bytes that crossed the bus for this buffer

    def keys(self) -> List[str]:
        return list(self.key_to_file)

    def _reap(self, wait: bool = False) -> None:
        """Plans (and the tables they own) may go once the stream has passed their kernels."""
        keep = []
        for plan, ev, ws in self._in_flight:
            if wait:
                ev.synchronize()
            if wait or ev.query():
                plan.close()
            else:
                keep.append((plan, ev, ws))
        self._in_flight = keep

    def get_many(self, requests: Dict[str, Request]) -> Dict[str, torch.Tensor]:
        """requests: key -> (target dtype name or None, shard dim or -1, blocks).  Keys whose declared request
        was already materialized are returned as they are; the others go out as one launch set on the current
        stream, without waiting for it."""
        out: Dict[str, torch.Tensor] = {}
        todo: Dict[str, Request] = {}
        for k, rq in requests.items():
            rq = (rq[0], rq[1], rq[2])
            if k in self._ready and self._ready_requests.get(k) == rq:
                out[k] = self._ready[k]
            else:
                todo[k] = rq
        if todo:
            if self._raw is None:
                raise RuntimeError("the device buffer has been released (or was streamed): only the requests "
                                   "declared before copy_files_to_device can be fetched")
            self._reap()
            names = list(todo)
            plan = B.Plan(self._headers, self._bases, names, [todo[n] for n in names], self._group.rank(),
                          self._group.size())
            try:
                bufs, ptrs = D.alloc_outputs(plan, self._raw.device)
                stream = torch.cuda.current_stream(self._raw.device)
                ws = None
                if plan.workspace_bytes() <= B.FST_STATIC_WORKSPACE_BYTES:
                    # no workspace to allocate: the tables go into the library's own
                    _order_static_call(stream)
                    B.fst_materialize_static(self._raw.data_ptr(), self._raw_len, plan, B.FST_ALL_GROUPS, ptrs,
                                             stream.cuda_stream)
                else:
                    ws = D.device_bytes(plan.workspace_bytes(), self._raw.device)
                    B.fst_materialize(self._raw.data_ptr(), self._raw_len, plan, B.FST_ALL_GROUPS, ptrs, ws.data_ptr(),
                                      ws.numel(), stream.cuda_stream)
                ev = torch.cuda.Event()
                ev.record(stream)
                if ws is None:
                    _last_static_call[stream.device.index or 0] = (stream.cuda_stream, ev)
                for i, n in enumerate(names):
                    out[n] = D.as_tensor(bufs[i], plan.output(i))
                self._in_flight.append((plan, ev, ws))
            except BaseException:
                plan.close()
                raise
        self._pending.difference_update(requests)
        if self._auto and not self._pending:
            self.close()
        return {k: out[k] for k in requests}

    def get_tensor(self, key: str, dtype: Optional[str] = None) -> torch.Tensor:
        return self.get_many({key: (dtype, -1, 1)})[key]

    def get_sharded(self, key: str, dim: int, dtype: Optional[str] = None, blocks: int = 1) -> torch.Tensor:
        return self.get_many({key: (dtype, dim, blocks)})[key]

    def close(self) -> None:
        """Releases the raw bytes.  Waits for the kernels still reading them."""
        self._reap(wait=True)
        self._raw = None


class SafeTensorsFileLoader:
    def __init__(self, pg=None, device: Optional[torch.device] = None, auto_release: bool = False,
                 max_threads: int = 12, bounce_buffer_bytes: int = 128 << 20, bounce_buffers: int = 8,
                 min_gap_bytes: int = 1 << 20, min_segment_bytes: int = 2048, group_bytes: int = 1 << 30):
        self._group = pg or SingleGroup()
        self._device = device or D.require_gpu()
        if self._device.type != "cuda":
            raise ValueError("this loader materializes on the GPU only")
        self._auto = auto_release
        self._files: List[str] = []
        self._requests: Dict[str, Request] = {}
        self._stager_cfg = (bounce_buffers, max_threads, bounce_buffer_bytes)
        self._stager: Optional[B.Stager] = None
        self._min_gap, self._min_seg, self._group_bytes = min_gap_bytes, min_segment_bytes, group_bytes

    def add_filenames(self, filemap: Dict[int, Sequence[str]]) -> None:
        """rank -> files, as in the paper; with one GPU every listed file is loaded here."""
        for rank in sorted(filemap):
            self._files += list(filemap[rank])

    def add_requests(self, requests: Dict[str, Request]) -> None:
        """Declare what will be fetched: key -> (target dtype name or None, shard dim or -1, blocks).  The next
        `copy_files_to_device` then stages only the bytes these requests read, and materializes them while it
        stages."""
        for k, rq in requests.items():
            self._requests[k] = (rq[0], rq[1], rq[2])

    def _stage(self, fn, plan, buf_ptr, buf_len, ptrs, ws, flags=0):
        if self._stager is None:
            self._stager = B.Stager(*self._stager_cfg)
        fds = [os.open(p, os.O_RDONLY) for p in self._files]
        try:
            arr = (ctypes.c_int * len(fds))(*fds)
            torch.cuda.current_stream(self._device).synchronize()    # the stager's streams are its own
            return fn(self._stager, plan, B.read_fds_fn(), ctypes.addressof(arr), buf_ptr, buf_len, ptrs,
                      ws.data_ptr() if ws is not None else 0, ws.numel() if ws is not None else 0, flags)
        finally:
            for fd in fds:
                os.close(fd)

    def copy_files_to_device(self, stream_slots: Optional[Tuple[int, int]] = None) -> FilesBufferOnDevice:
        headers, sizes = [], []
        for p in self._files:
            h, s = D.read_header(p)
            headers.append(h)
            sizes.append(s)
        if not self._requests:
            # the paper's way: whole files, verbatim, resident
            bases, raw_len = D.file_bases(sizes, headers)        # every file's tensor data on a 256-byte boundary
            names = [t["name"] for h in headers for t in h.tensors()]
            plan = B.Plan(headers, bases, names, [(None, -1, 1)] * len(names))
            plan.set_groups(self._group_bytes)
            raw = D.device_bytes(raw_len, self._device)
            try:
                st = self._stage(B.Stager.stage_resident, plan, raw.data_ptr(), raw_len, [0] * len(names), None,
                                 B.FST_STAGE_NO_KERNELS)
            finally:
                plan.close()
            fb = FilesBufferOnDevice(headers, bases, raw, raw_len, self._group, self._auto, staged_bytes=st["staged_bytes"])
        else:
            names = list(self._requests)
            reqs = [self._requests[n] for n in names]
            plan = B.Plan(headers, D.file_phases(headers), names, reqs, self._group.rank(), self._group.size())
            try:
                slot_bytes = stream_slots[1] if stream_slots else self._group_bytes
                plan.set_groups(slot_bytes, self._min_gap, self._min_seg)
                bufs, ptrs = D.alloc_outputs(plan, self._device)
                ws = D.device_bytes(plan.workspace_bytes(), self._device)
                if stream_slots:
                    slots = [D.device_bytes(slot_bytes, self._device) for _ in range(stream_slots[0])]
                    if self._stager is None:
                        self._stager = B.Stager(*self._stager_cfg)
                    fds = [os.open(p, os.O_RDONLY) for p in self._files]
                    try:
                        arr = (ctypes.c_int * len(fds))(*fds)
                        torch.cuda.current_stream(self._device).synchronize()
                        st = self._stager.stage_streamed(plan, B.read_fds_fn(), ctypes.addressof(arr),
                                                         [s.data_ptr() for s in slots], slot_bytes, ptrs, ws.data_ptr(), ws.numel())
                    finally:
                        for fd in fds:
                            os.close(fd)
                else:
                    n = plan.packed_bytes()
                    packed = D.device_bytes(n, self._device)
                    st = self._stage(B.Stager.stage_packed, plan, packed.data_ptr(), n, ptrs, ws)
                ready = {n: D.as_tensor(bufs[i], plan.output(i)) for i, n in enumerate(names)}
            finally:
                plan.close()
            fb = FilesBufferOnDevice(headers, [0] * len(headers), None, 0, self._group, self._auto, ready=ready,
                                     ready_requests=dict(self._requests), staged_bytes=st["staged_bytes"])
        self._files = []
        self._requests = {}
        return fb

    def close(self) -> None:
        if self._stager is not None:
            self._stager.close()
            self._stager = None
