"""Test-only safetensors writer (seeded input generators, part 3).

Serializes the container the paper describes in Section II-A / Fig. 1: 8 bytes holding the header
size, a JSON layout definition (per tensor: dtype, shape, data_offsets), then the tensor bytes back
to back.  Used to build inputs and for serialize -> deserialize round trips; it never reads a file.
"""
from __future__ import annotations

import json
import struct
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

from .specs import DTYPE_SIZE


def build_header(entries: Sequence[Tuple[str, str, Sequence[int], int]],
                 metadata: Optional[Dict[str, str]] = None,
                 body_residue: Optional[int] = None,
                 order: Optional[Sequence[int]] = None) -> Tuple[bytes, List[Tuple[int, int]]]:
    """entries: (name, dtype, shape, nbytes) in on-disk order.  Returns (first 8+N bytes of the
    file, [(begin, end)] per entry, relative to the body).  `body_residue`: pad the JSON with
    spaces until (8 + N) % 16 equals it.  `order`: order of the keys inside the JSON text
    (default = on-disk order); key order carries no meaning in the format."""
    offs, at = [], 0
    for _, dt, shape, nbytes in entries:
        n = 1
        for s in shape:
            n *= s
        assert nbytes == n * DTYPE_SIZE[dt], (dt, shape, nbytes)
        offs.append((at, at + nbytes))
        at += nbytes
    d: Dict[str, object] = {}
    if metadata is not None:
        d["__metadata__"] = metadata
    idx = list(order) if order is not None else list(range(len(entries)))
    for i in idx:
        name, dt, shape, _ = entries[i]
        d[name] = {"dtype": dt, "shape": list(shape), "data_offsets": [offs[i][0], offs[i][1]]}
    text = json.dumps(d, separators=(",", ":"), ensure_ascii=False).encode("utf-8")
    if body_residue is not None:
        while (8 + len(text)) % 16 != body_residue % 16:
            text += b" "
    return struct.pack("<Q", len(text)) + text, offs


def write_file(path: str, tensors: Sequence[Tuple[str, str, Sequence[int], bytes]],
               metadata: Optional[Dict[str, str]] = None, body_residue: Optional[int] = None,
               order: Optional[Sequence[int]] = None) -> bytes:
    """tensors: (name, dtype, shape, raw little-endian bytes) in on-disk order.  Writes the file and
    returns its bytes."""
    entries = [(n, dt, sh, len(b)) for n, dt, sh, b in tensors]
    head, _ = build_header(entries, metadata, body_residue, order)
    blob = head + b"".join(bytes(b) for _, _, _, b in tensors)
    if path is not None:
        with open(path, "wb") as f:
            f.write(blob)
    return blob
