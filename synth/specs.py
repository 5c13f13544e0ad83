"""Shapes of the synthetic checkpoints (seeded input generators, part 1: structure only).

These stand in for the checkpoints of the paper's evaluation (Table I: Llama-7B in 2 files,
Llama-13B in 3, Llama-70B in 15, Bloom-176B in 72; tensors serialized in layer order, Section
IV "Data").  Only tensor names, dtypes, shapes and the split over files are reproduced; the
values are synthetic (see source.py / writer.py).  Nothing in this module parses, slices or
casts anything: it holds none of the method's arithmetic and is the only code shared by the
CPU oracle's tests and the GPU path's tests.

A model is a list of files; a file is a list of TensorSpec in on-disk (offset) order.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

DTYPE_SIZE = {
    "BOOL": 1, "U8": 1, "I8": 1, "F8_E5M2": 1, "F8_E4M3": 1,
    "I16": 2, "U16": 2, "F16": 2, "BF16": 2,
    "I32": 4, "U32": 4, "F32": 4,
    "I64": 8, "U64": 8, "F64": 8,
}


@dataclass
class TensorSpec:
    name: str
    dtype: str
    shape: Tuple[int, ...]
    # how the values are produced: "normal" (N(0, 0.02) pool), "ones", "bytes" (uniform bytes),
    # "bool" ({0,1} bytes)
    fill: str = "normal"
    # the load request the configuration makes for this tensor (consumed by tests / bench):
    # shard_dim -1 = whole tensor; blocks > 1 = stacked sub-matrices split one by one
    shard_dim: int = -1
    blocks: int = 1
    dst_dtype: Optional[str] = None  # None = keep the stored dtype

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= s
        return n

    @property
    def nbytes(self) -> int:
        return self.numel * DTYPE_SIZE[self.dtype]


@dataclass
class FileSpec:
    filename: str
    tensors: List[TensorSpec]
    # residue of (8 + header length) modulo 16 that the writer pads the header to; the format
    # fixes no alignment and real checkpoints have odd-sized headers (Section III-B)
    body_residue: Optional[int] = None

    @property
    def body_bytes(self) -> int:
        return sum(t.nbytes for t in self.tensors)


@dataclass
class ModelSpec:
    name: str
    seed: int
    files: List[FileSpec]
    world: int = 1
    rank: int = 0
    notes: str = ""

    @property
    def n_tensors(self) -> int:
        return sum(len(f.tensors) for f in self.files)

    @property
    def body_bytes(self) -> int:
        return sum(f.body_bytes for f in self.files)


def _llama_layer(i: int, h: int, inter: int, kv: int, dt: str, tp: bool) -> List[TensorSpec]:
    p = f"model.layers.{i}."
    col = 0 if tp else -1   # input projections: split along the output dim (dim 0 as stored)
    row = 1 if tp else -1   # output projections: split along the input dim (dim 1 as stored)
    return [
        TensorSpec(p + "self_attn.q_proj.weight", dt, (h, h), shard_dim=col),
        TensorSpec(p + "self_attn.k_proj.weight", dt, (kv, h), shard_dim=col),
        TensorSpec(p + "self_attn.v_proj.weight", dt, (kv, h), shard_dim=col),
        TensorSpec(p + "self_attn.o_proj.weight", dt, (h, h), shard_dim=row),
        TensorSpec(p + "mlp.gate_proj.weight", dt, (inter, h), shard_dim=col),
        TensorSpec(p + "mlp.up_proj.weight", dt, (inter, h), shard_dim=col),
        TensorSpec(p + "mlp.down_proj.weight", dt, (h, inter), shard_dim=row),
        TensorSpec(p + "input_layernorm.weight", dt, (h,), fill="ones"),
        TensorSpec(p + "post_attention_layernorm.weight", dt, (h,), fill="ones"),
    ]


def _llama(name: str, seed: int, layers: int, h: int, inter: int, vocab: int, kv: int, dt: str,
           cuts: List[int], tp_world: int = 1, dst: Optional[str] = None,
           residues: Optional[List[int]] = None) -> ModelSpec:
    """`cuts` = index of the first layer of every file after the first."""
    tp = tp_world > 1
    bounds = [0] + list(cuts) + [layers]
    nfiles = len(bounds) - 1
    files = []
    for f in range(nfiles):
        ts: List[TensorSpec] = []
        if f == 0:
            ts.append(TensorSpec("model.embed_tokens.weight", dt, (vocab, h)))
        for i in range(bounds[f], bounds[f + 1]):
            ts += _llama_layer(i, h, inter, kv, dt, tp)
        if f == nfiles - 1:
            ts.append(TensorSpec("model.norm.weight", dt, (h,), fill="ones"))
            ts.append(TensorSpec("lm_head.weight", dt, (vocab, h)))
        for t in ts:
            t.dst_dtype = dst
        res = residues[f % len(residues)] if residues else None
        files.append(FileSpec(f"model-{f + 1:05d}-of-{nfiles:05d}.safetensors", ts, res))
    return ModelSpec(name, seed, files, world=tp_world, rank=0)


# residues of the body start modulo 16 handed out to the files of the large models, so that
# aligned, 4-byte-aligned, 2-byte-aligned and odd starts all occur
_RESIDUES = [3, 8, 0, 14, 5, 4, 10, 9, 12, 1, 6, 15, 2, 7, 11, 13]


def config1_tiny() -> ModelSpec:
    """2-layer Llama-like model (hidden 256, 4 heads, intermediate 688, vocab 1000), bf16, plus an
    int8[37] and a bool[13] tensor stored before the weights so that every later tensor starts at
    an odd byte offset (37) and then at an even, non-4-aligned one (50)."""
    m = _llama("tiny-llama", 1, 2, 256, 688, 1000, 256, "BF16", cuts=[])
    f = m.files[0]
    f.filename = "tiny.safetensors"
    extra = [TensorSpec("aux.int8", "I8", (37,), fill="bytes"),
             TensorSpec("aux.flags", "BOOL", (13,), fill="bool")]
    # order on disk: int8[37], embed, bool[13], rest -> the embedding sits at odd offset 37, the
    # remaining weights at offset = 37 + 512000 + 13 (even, == 2 mod 4)
    f.tensors = [extra[0], f.tensors[0], extra[1]] + f.tensors[1:]
    f.body_residue = None  # header left exactly as serialized (not padded)
    return m


def config2_llama7b() -> ModelSpec:
    return _llama("llama-7b", 2, 32, 4096, 11008, 32000, 4096, "BF16", cuts=[24],
                  residues=[3, 8])


def config3_llama13b() -> ModelSpec:
    return _llama("llama-13b", 3, 40, 5120, 13824, 32000, 5120, "F16", cuts=[13, 27],
                  dst="BF16", residues=[14, 5, 0])


def config4_llama70b(layers: int = 80, nfiles: int = 15) -> ModelSpec:
    per, extra = divmod(layers, nfiles)
    cuts, at = [], 0
    for f in range(nfiles - 1):
        at += per + (1 if f < extra else 0)
        cuts.append(at)
    return _llama("llama-70b", 4, layers, 8192, 28672, 32000, 1024, "BF16", cuts=cuts,
                  tp_world=8, residues=_RESIDUES)


def _bloom_layer(i: int, h: int, dt: str) -> List[TensorSpec]:
    p = f"h.{i}."
    ln = dict(dst_dtype="F32")
    return [
        TensorSpec(p + "input_layernorm.weight", dt, (h,), fill="ones", **ln),
        TensorSpec(p + "input_layernorm.bias", dt, (h,), **ln),
        # stacked [Q; K; V]: each of the three sub-matrices is split by rank
        TensorSpec(p + "self_attention.query_key_value.weight", dt, (3 * h, h), shard_dim=0, blocks=3),
        TensorSpec(p + "self_attention.query_key_value.bias", dt, (3 * h,), shard_dim=0, blocks=3),
        TensorSpec(p + "self_attention.dense.weight", dt, (h, h), shard_dim=1),
        TensorSpec(p + "self_attention.dense.bias", dt, (h,)),
        TensorSpec(p + "post_attention_layernorm.weight", dt, (h,), fill="ones", **ln),
        TensorSpec(p + "post_attention_layernorm.bias", dt, (h,), **ln),
        TensorSpec(p + "mlp.dense_h_to_4h.weight", dt, (4 * h, h), shard_dim=0),
        TensorSpec(p + "mlp.dense_h_to_4h.bias", dt, (4 * h,), shard_dim=0),
        TensorSpec(p + "mlp.dense_4h_to_h.weight", dt, (h, 4 * h), shard_dim=1),
        TensorSpec(p + "mlp.dense_4h_to_h.bias", dt, (h,)),
    ]


def config5_bloom176b(layers: int = 70, h: int = 14336, vocab: int = 250880) -> ModelSpec:
    dt = "BF16"
    nfiles = layers + 2
    files = [FileSpec(f"model_{1:05d}-of-{nfiles:05d}.safetensors",
                      [TensorSpec("word_embeddings.weight", dt, (vocab, h))], _RESIDUES[0])]
    for i in range(layers):
        files.append(FileSpec(f"model_{i + 2:05d}-of-{nfiles:05d}.safetensors",
                              _bloom_layer(i, h, dt), _RESIDUES[(i + 1) % 16]))
    ln = dict(dst_dtype="F32")
    files.append(FileSpec(f"model_{nfiles:05d}-of-{nfiles:05d}.safetensors", [
        TensorSpec("word_embeddings_layernorm.weight", dt, (h,), fill="ones", **ln),
        TensorSpec("word_embeddings_layernorm.bias", dt, (h,), **ln),
        TensorSpec("ln_f.weight", dt, (h,), fill="ones", **ln),
        TensorSpec("ln_f.bias", dt, (h,), **ln),
    ], _RESIDUES[(layers + 1) % 16]))
    return ModelSpec("bloom-176b", 5, files, world=8, rank=0)


def _falcon_layer(i: int, h: int, qkv_rows: int, dt: str, tp: bool) -> List[TensorSpec]:
    p = f"transformer.h.{i}."
    col = 0 if tp else -1
    row = 1 if tp else -1
    return [
        TensorSpec(p + "ln_attn.weight", dt, (h,), fill="ones"),
        TensorSpec(p + "ln_attn.bias", dt, (h,)),
        TensorSpec(p + "ln_mlp.weight", dt, (h,), fill="ones"),
        TensorSpec(p + "ln_mlp.bias", dt, (h,)),
        # fused QKV stored group by group (per KV group: its query heads, one key head, one value
        # head): a plain split of dim 0 hands each rank whole groups
        TensorSpec(p + "self_attention.query_key_value.weight", dt, (qkv_rows, h), shard_dim=col),
        TensorSpec(p + "self_attention.dense.weight", dt, (h, h), shard_dim=row),
        TensorSpec(p + "mlp.dense_h_to_4h.weight", dt, (4 * h, h), shard_dim=col),
        TensorSpec(p + "mlp.dense_4h_to_h.weight", dt, (h, 4 * h), shard_dim=row),
    ]


def config_falcon40b(layers: int = 60, nfiles: int = 9, world: int = 2) -> ModelSpec:
    """Falcon-40B-shaped checkpoint (Table I: 9 files, 78 GiB): 60 layers, hidden 8192, 128 query heads
    and 8 key/value heads of 64, vocabulary 65024, bf16; rank 0 of a 2-way split (the paper loads it
    on two GPUs)."""
    h, dt, vocab = 8192, "BF16", 65024
    qkv_rows = (128 + 2 * 8) * 64
    per, extra = divmod(layers, nfiles)
    files, at = [], 0
    for f in range(nfiles):
        n = per + (1 if f < extra else 0)
        ts: List[TensorSpec] = []
        if f == 0:
            ts.append(TensorSpec("transformer.word_embeddings.weight", dt, (vocab, h)))
        for i in range(at, at + n):
            ts += _falcon_layer(i, h, qkv_rows, dt, world > 1)
        at += n
        if f == nfiles - 1:
            ts.append(TensorSpec("transformer.ln_f.weight", dt, (h,), fill="ones"))
            ts.append(TensorSpec("transformer.ln_f.bias", dt, (h,)))
            ts.append(TensorSpec("lm_head.weight", dt, (vocab, h)))
        files.append(FileSpec(f"model-{f + 1:05d}-of-{nfiles:05d}.safetensors", ts, _RESIDUES[(f + 5) % 16]))
    return ModelSpec("falcon-40b", 6, files, world=world, rank=0)


def micro_ragged(seg_bytes_x4: int = 8200, rows: int = 262144, dst: Optional[str] = None) -> ModelSpec:
    """One bf16 matrix whose dim-1 share (rank 1 of 4) has row segments of seg_bytes_x4 / 4 bytes: 2050 by
    default, not a multiple of 16 (a kernel-only case: spliced chunks)."""
    cols = seg_bytes_x4 // 2
    t = TensorSpec("w", "BF16", (rows, cols), shard_dim=1, dst_dtype=dst)
    return ModelSpec(f"ragged-rows-{seg_bytes_x4 // 4}B" + (f"-to-{dst}" if dst else ""), 71,
                     [FileSpec("a.safetensors", [t], 5)], world=4, rank=1)


def micro_short_rows(dtype: str, cols: int, world: int, rows: int = 1 << 24) -> ModelSpec:
    """One matrix with very short rows split along dim 1: the share's row segments are
    cols / world elements, shorter than one 16-byte chunk (gathered chunks)."""
    t = TensorSpec("w", dtype, (rows, cols), fill="normal" if dtype != "U8" else "bytes", shard_dim=1)
    seg = cols // world * DTYPE_SIZE[dtype]
    return ModelSpec(f"short-rows-{seg}B-of-{cols * DTYPE_SIZE[dtype]}B", 72, [FileSpec("a.safetensors", [t], 6)],
                     world=world, rank=world - 1)


def micro_small_tensors(n: int = 4096, elems: int = 4096, dst: Optional[str] = None) -> ModelSpec:
    """n bf16 vectors of `elems` elements (8 KiB each by default) in one file."""
    ts = [TensorSpec(f"t{i}", "BF16", (elems,), dst_dtype=dst) for i in range(n)]
    return ModelSpec(f"{n}-tensors-of-{elems * 2}B" + (f"-to-{dst}" if dst else ""), 73, [FileSpec("a.safetensors", ts, 5)])


def micro_one_tensor(dtype: str, elems: int, dst: Optional[str] = None, residue: int = 3) -> ModelSpec:
    """One vector of `elems` elements of `dtype`, converted to `dst`; the file body starts at `residue` mod 16."""
    t = TensorSpec("w", dtype, (elems,), dst_dtype=dst)
    return ModelSpec(f"one-{dtype}-tensor-of-{elems}" + (f"-to-{dst}" if dst else ""), 74,
                     [FileSpec("a.safetensors", [t], residue)])


CONFIGS = {
    "tiny": config1_tiny,
    "llama-7b": config2_llama7b,
    "llama-13b": config3_llama13b,
    "llama-70b": config4_llama70b,
    "bloom-176b": config5_bloom176b,
    "falcon-40b": config_falcon40b,
}
