"""Seeded random test cases shared by the CPU planner tests and the GPU parity tests: small files with
every kind of tensor and request.  Input generation only."""
import numpy as np

from synth import writer

NP = {"U8": np.uint8, "I8": np.int8, "I16": np.int16, "U16": np.uint16, "F16": np.uint16, "BF16": np.uint16,
      "F32": np.uint32, "I32": np.int32, "F64": np.float64, "I64": np.int64, "BOOL": np.uint8,
      "F8_E5M2": np.uint8, "F8_E4M3": np.uint8, "U32": np.uint32, "U64": np.uint64}
ES = {k: np.dtype(v).itemsize for k, v in NP.items()}
FLOATS = ("F32", "F16", "BF16")
ALL_FLOATS = ("F64", "F32", "F16", "BF16")
F8S = ("F8_E5M2", "F8_E4M3")
F8_TARGETS = ("F16", "BF16", "F32")


def cast_targets(dtype):
    """The element types a stored dtype can be converted to (other than itself)."""
    if dtype in F8S:
        return list(F8_TARGETS)
    return [d for d in ALL_FLOATS if d != dtype] if dtype in ALL_FLOATS else []


def random_bits(rng, dtype, shape):
    """Random bit patterns (for floats: all exponents incl. NaN/inf/subnormal appear)."""
    n = int(np.prod(shape)) if len(shape) else 1
    raw = rng.integers(0, 256, n * ES[dtype], dtype=np.uint8)
    if dtype == "BOOL":
        raw &= 1
    return raw


def make_file(rng, n_tensors=8, residue=None, max_dim=40, dtypes=None, big=False, prefix=""):
    """Returns (blob, [(name, dtype, shape)]) with tensors of mixed rank, incl. empty and scalar."""
    dtypes = dtypes or list(NP)
    ts = []
    for i in range(n_tensors):
        dt = dtypes[int(rng.integers(len(dtypes)))]
        nd = int(rng.integers(0, 4))
        shape = tuple(int(x) for x in rng.integers(0 if rng.random() < 0.1 else 1, max_dim, nd))
        if big and i % 3 == 0:
            shape = (int(rng.integers(200, 700)), int(rng.integers(8, 33)) * 8)
        ts.append((f"{prefix}layer.{i}.w", dt, shape, random_bits(rng, dt, shape).tobytes()))
    blob = writer.write_file(None, ts, None, residue if residue is not None else int(rng.integers(16)))
    return blob, [(n, d, s) for n, d, s, _ in ts]


def random_request(rng, dtype, shape, world):
    """A valid (dst_dtype, shard_dim, blocks, world) for the tensor, or whole-tensor when nothing divides."""
    dst = None
    if dtype in FLOATS and rng.random() < 0.6:
        dst = FLOATS[int(rng.integers(3))]
    elif dtype in ("F32", "F64") and rng.random() < 0.5:
        dst = "F64" if dtype == "F32" else "F32"
    if dtype in ALL_FLOATS and rng.random() < 0.15:          # drawn last: the older cases keep their requests
        dst = ALL_FLOATS[int(rng.integers(4))]
    if dtype in F8S and rng.random() < 0.5:
        dst = F8_TARGETS[int(rng.integers(3))]
    dims = [d for d in range(len(shape)) if shape[d] % world == 0]
    if not dims or rng.random() < 0.25:
        return dst, -1, 1
    d = dims[int(rng.integers(len(dims)))]
    blocks = 1
    if d == 0:
        for b in (3, 2):
            if shape[0] % (b * world) == 0 and rng.random() < 0.5:
                blocks = b
                break
    return dst, d, blocks
