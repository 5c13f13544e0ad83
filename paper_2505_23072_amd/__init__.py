"""Device-side deserialization of safetensors files on AMD MI355X (method of arXiv 2505.23072).

`binding` mirrors the C ABI of include/fst.h; `device` holds the PyTorch plumbing (device memory,
streams) around it.  All arithmetic and data movement happen inside libfst.so.
"""
from . import binding  # noqa: F401
from .binding import (FST_ALL_GROUPS, FST_STAGE_NO_KERNELS, FST_STAGE_NO_READ, FstError, Header, Plan, Stager,
                      fst_header_len, fst_materialize, fst_materialize_slot)

__all__ = ["binding", "FST_ALL_GROUPS", "FST_STAGE_NO_KERNELS", "FST_STAGE_NO_READ", "FstError", "Header", "Plan",
           "Stager", "fst_header_len", "fst_materialize", "fst_materialize_slot"]
