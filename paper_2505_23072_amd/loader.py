"""Loader API in the shape of the paper's (Section III-C, Figs. 8 and 9):

    loader = SafeTensorsFileLoader(SingleGroup(), torch.device("cuda:0"))
    loader.add_filenames({0: ["a.safetensors"]})
    fb = loader.copy_files_to_device()
    t = fb.get_tensor("a0")
    s = fb.get_sharded("b0", dim=1)
    fb.close(); loader.close()

`copy_files_to_device` stages the files verbatim into one raw HBM buffer through the pinned ring;
`get_tensor` / `get_sharded` / `get_many` run the materialize kernels on that buffer and return
aligned tensors of their own, so the raw buffer can be released (`close`, or automatically once every
key has been fetched).  One GPU only: a group says which rank's share this GPU takes, nothing is sent
anywhere.  This module only marshals; parsing, planning, staging and the kernels are in libfst.so.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import torch

from . import binding as B
from . import device as D


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
    """The raw bytes of the loaded files in HBM plus the lookup from key to tensor (Section III-C)."""

    def __init__(self, headers, paths, bases, raw, raw_len, group, auto_release):
        self._headers, self._paths, self._bases = headers, paths, bases
        self._raw, self._raw_len, self._group = raw, raw_len, group
        self._auto = auto_release
        self._pending = {t["name"] for h in headers for t in h.tensors()}
        self.key_to_file = {t["name"]: i for i, h in enumerate(headers) for t in h.tensors()}

    def keys(self) -> List[str]:
        return list(self.key_to_file)

    def get_many(self, requests: Dict[str, Tuple[Optional[str], int, int]]) -> Dict[str, torch.Tensor]:
        """requests: key -> (target dtype name or None, shard dim or -1, blocks).  One launch set."""
        if self._raw is None:
            raise RuntimeError("the device buffer has been released")
        names = list(requests)
        plan = B.Plan(self._headers, self._bases, names, [requests[n] for n in names], self._group.rank(),
                      self._group.size())
        try:
            bufs, ptrs = D.alloc_outputs(plan, self._raw.device)
            ws = D.device_bytes(plan.workspace_bytes(), self._raw.device)
            stream = torch.cuda.current_stream(self._raw.device)
            B.fst_materialize(self._raw.data_ptr(), self._raw_len, plan, B.FST_ALL_GROUPS, ptrs, ws.data_ptr(),
                              ws.numel(), stream.cuda_stream)
            out = {n: D.as_tensor(bufs[i], plan.output(i)) for i, n in enumerate(names)}
            stream.synchronize()       # the plan and its table may go once the kernels have run
        finally:
            plan.close()
        self._pending.difference_update(names)
        if self._auto and not self._pending:
            self.close()
        return out

    def get_tensor(self, key: str, dtype: Optional[str] = None) -> torch.Tensor:
        return self.get_many({key: (dtype, -1, 1)})[key]

    def get_sharded(self, key: str, dim: int, dtype: Optional[str] = None, blocks: int = 1) -> torch.Tensor:
        return self.get_many({key: (dtype, dim, blocks)})[key]

    def close(self) -> None:
        self._raw = None


class SafeTensorsFileLoader:
    def __init__(self, pg=None, device: Optional[torch.device] = None, auto_release: bool = False,
                 max_threads: int = 12, bounce_buffer_bytes: int = 32 << 20, bounce_buffers: int = 16):
        self._group = pg or SingleGroup()
        self._device = device or D.require_gpu()
        if self._device.type != "cuda":
            raise ValueError("this loader materializes on the GPU only")
        self._auto = auto_release
        self._files: List[str] = []
        self._stager_cfg = (bounce_buffers, max_threads, bounce_buffer_bytes)
        self._stager: Optional[B.Stager] = None

    def add_filenames(self, filemap: Dict[int, Sequence[str]]) -> None:
        """rank -> files, as in the paper; with one GPU every listed file is loaded here."""
        for rank in sorted(filemap):
            self._files += list(filemap[rank])

    def copy_files_to_device(self) -> FilesBufferOnDevice:
        headers, sizes = [], []
        for p in self._files:
            h, s = D.read_header(p)
            headers.append(h)
            sizes.append(s)
        bases, raw_len = D.file_bases(sizes)
        names = [t["name"] for h in headers for t in h.tensors()]
        plan = B.Plan(headers, bases, names, [(None, -1, 1)] * len(names))     # whole files
        plan.set_groups(1 << 30)
        raw = D.device_bytes(raw_len, self._device)
        if self._stager is None:
            self._stager = B.Stager(*self._stager_cfg)
        fds = [os.open(p, os.O_RDONLY) for p in self._files]
        try:
            arr = (ctypes.c_int * len(fds))(*fds)
            torch.cuda.current_stream(self._device).synchronize()    # the stager's streams are its own
            self._stager.stage_resident(plan, B.read_fds_fn(), ctypes.addressof(arr), raw.data_ptr(), raw_len, [0] * len(names),
                                        0, 0, B.FST_STAGE_NO_KERNELS)
        finally:
            for fd in fds:
                os.close(fd)
            plan.close()
        fb = FilesBufferOnDevice(headers, list(self._files), bases, raw, raw_len, self._group, self._auto)
        self._files = []
        return fb

    def close(self) -> None:
        if self._stager is not None:
            self._stager.close()
            self._stager = None
