"""PyTorch plumbing around the C ABI: device buffers, streams, and tensor views of the outputs.
Nothing here computes: it allocates, passes pointers and reinterprets the bytes the kernels wrote."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import binding as B

TORCH_DTYPE = {
    "F64": torch.float64, "F32": torch.float32, "F16": torch.float16, "BF16": torch.bfloat16,
    "I64": torch.int64, "I32": torch.int32, "I16": torch.int16, "I8": torch.int8,
    "U8": torch.uint8, "BOOL": torch.bool,
    "U16": getattr(torch, "uint16", None), "U32": getattr(torch, "uint32", None),
    "U64": getattr(torch, "uint64", None),
    "F8_E5M2": getattr(torch, "float8_e5m2", None), "F8_E4M3": getattr(torch, "float8_e4m3fn", None),
}


def require_gpu() -> torch.device:
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: this library has no CPU path")
    return torch.device("cuda:0")


def device_bytes(n: int, dev: Optional[torch.device] = None) -> torch.Tensor:
    """n bytes of device memory (torch allocations are 512-byte aligned)."""
    t = torch.empty(max(int(n), 1), dtype=torch.uint8, device=dev or require_gpu())
    assert t.data_ptr() % 256 == 0
    return t


def read_header(path: str) -> Tuple[B.Header, int]:
    size = os.path.getsize(path)
    with open(path, "rb") as f:
        first = f.read(8)
        n = B.fst_header_len(first)
        head = first + f.read(min(n, max(size - 8, 0)))
    return B.Header(head, size), size


def file_bases(sizes: Sequence[int], headers: Optional[Sequence[B.Header]] = None) -> Tuple[List[int], int]:
    """Offsets at which whole files sit in one raw buffer, and its length.  Without headers every file starts on a
    multiple of 256; with them every file is shifted so that its tensor data (the first byte after the header)
    starts on one, which lets the kernels read most tensors with aligned loads."""
    bases, at = [], 0
    for i, s in enumerate(sizes):
        phase = headers[i].aligned_phase() if headers is not None else 0
        bases.append(at + phase)
        at += (phase + s + 255) // 256 * 256
    return bases, max(at, 256)


def file_phases(headers: Sequence[B.Header]) -> List[int]:
    """raw_base values for plans that are only staged into slots or packed: just the phase that aligns each file's
    tensor data."""
    return [h.aligned_phase() for h in headers]


def alloc_outputs(plan: B.Plan, dev: Optional[torch.device] = None) -> Tuple[List[torch.Tensor], List[int]]:
    """One uint8 device tensor per output, and their addresses."""
    bufs = [device_bytes(plan.output(i)["nbytes"], dev) for i in range(plan.output_count())]
    return bufs, [b.data_ptr() for b in bufs]


def as_tensor(buf: torch.Tensor, info: dict) -> torch.Tensor:
    """View an output buffer as a tensor of the output's dtype and shape (no copy)."""
    dt = TORCH_DTYPE.get(info["dtype"])
    if dt is None:
        raise TypeError(f"this PyTorch build has no dtype for {info['dtype']}")
    n = info["nbytes"]
    if n == 0:
        return torch.empty(info["shape"], dtype=dt, device=buf.device)
    return buf[:n].view(dt).reshape(info["shape"])


def load_files(paths: Sequence[str], requests: Optional[Dict[str, B.Request]] = None, rank: int = 0, world: int = 1,
               group_bytes: int = 1 << 30, stager: Optional[B.Stager] = None) -> Dict[str, torch.Tensor]:
    """Files -> tensors on the GPU, through the staging ring and the materialize kernels.
    requests: name -> (dst dtype or None, shard_dim, blocks); default: every tensor, unchanged."""
    dev = require_gpu()
    headers, sizes = [], []
    for p in paths:
        h, s = read_header(p)
        headers.append(h)
        sizes.append(s)
    bases, raw_len = file_bases(sizes, headers)
    if requests is None:
        requests = {t["name"]: (None, -1, 1) for h in headers for t in h.tensors()}
    names = list(requests)
    plan = B.Plan(headers, bases, names, [requests[n] for n in names], rank, world)
    plan.set_groups(group_bytes)
    raw = device_bytes(raw_len, dev)
    ws = device_bytes(plan.workspace_bytes(), dev)
    bufs, ptrs = alloc_outputs(plan, dev)
    own = stager is None
    st = stager or B.Stager()
    fds = [os.open(p, os.O_RDONLY) for p in paths]
    try:
        arr = (ctypes.c_int * len(fds))(*fds)
        # the stager's streams are not ordered with torch's: the allocator may have handed out blocks that
        # earlier work on the current stream still uses
        torch.cuda.current_stream(dev).synchronize()
        st.stage_resident(plan, B.read_fds_fn(), ctypes.addressof(arr), raw.data_ptr(), raw_len, ptrs,
                          ws.data_ptr(), ws.numel())
    finally:
        for fd in fds:
            os.close(fd)
        if own:
            st.close()
    return {n: as_tensor(bufs[i], plan.output(i)) for i, n in enumerate(names)}
