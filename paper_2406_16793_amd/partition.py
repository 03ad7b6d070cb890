"""Parameter partition of Adam-mini expressed as per-tensor block descriptors.

The paper's listing "Partition for Transformers" (Appendix B) cuts each
named weight along its outermost dimension: embedding / output layers by token,
query / key by attention head, value / attention projection / MLP weights by
output neuron, and leaves every other tensor whole.  Its "Partition for
non-Transformers" (same appendix) leaves every tensor whole.  For a row-major
tensor whose partition dimension is outermost all of these are equal contiguous
runs, so one integer per tensor -- ``block_numel`` -- states the partition; this
module computes that integer from a tensor's name and shape.  Host-side integer
logic only.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterable, List, Optional, Sequence, Tuple

# substrings that select a rule (the paper's keywords first, then common spellings)
EMBED_KEYS = ("embed", "output", "wte", "lm_head", "tok_embeddings")
QUERY_KEYS = ("query", "q_proj", "wq", "attn.q")
KEY_KEYS = ("key", "k_proj", "wk", "attn.k")
NEURON_KEYS = ("value", "v_proj", "wv", "attn.v", "attn.proj", "o_proj", "wo", "mlp",
               "feed_forward", "w1", "w2", "w3")


@dataclass(frozen=True)
class TensorSpec:
    """One tensor of the multi-tensor list handed to the library."""
    name: str
    shape: Tuple[int, ...]
    block_numel: int
    wd_scale: float = 1.0
    strided: bool = False   # blocks are the COLUMNS of the stored [block_numel, n_blocks] matrix (weight kept transposed)
    reducer: str = "mean"   # block statistic of g*g that feeds v: "mean" (the method), or the appendix
                            # ablation's "norm1", "norm2", "max", "min"

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= int(s)
        return n

    @property
    def n_blocks(self) -> int:
        return self.numel // self.block_numel


def _numel(shape: Sequence[int]) -> int:
    n = 1
    for s in shape:
        n *= int(s)
    return n


def _has(name: str, keys: Iterable[str]) -> bool:
    return any(k in name for k in keys)


def block_numel_for(name: str, shape: Sequence[int], n_heads: int,
                    n_kv_heads: Optional[int] = None, value_whole: bool = False) -> int:
    """block_numel of one named tensor under "Partition for Transformers" (Appendix B).

    n_heads / n_kv_heads: number of query heads / key heads (grouped-query
    attention keeps one block per KEY head).  value_whole=True is the appendix's
    "strategy II" that treats each value matrix as a single block.
    Tensors that match no rule -- and all 1-D tensors -- are one block.
    """
    numel = _numel(shape)
    if len(shape) < 2:
        return numel
    rows = int(shape[0])
    # the attention-output projection contains "proj"/"wo": test the neuron rule for
    # it before the embedding rule sees the substring "output" of e.g. "attn.output"
    is_attn_out = _has(name, ("attn.proj", "o_proj", "wo", "attention.output"))
    if not is_attn_out and _has(name, EMBED_KEYS):
        return numel // rows
    if _has(name, QUERY_KEYS):
        if rows % n_heads:
            raise ValueError("%s: %d rows not divisible by %d heads" % (name, rows, n_heads))
        return numel // n_heads
    if _has(name, KEY_KEYS):
        kv = n_kv_heads or n_heads
        if rows % kv:
            raise ValueError("%s: %d rows not divisible by %d key heads" % (name, rows, kv))
        return numel // kv
    if is_attn_out or _has(name, NEURON_KEYS):
        if value_whole and _has(name, ("value", "v_proj", "wv", "attn.v")):
            return numel
        return numel // rows
    return numel


def partition_transformer(named_shapes: Sequence[Tuple[str, Sequence[int]]], n_heads: int,
                          n_kv_heads: Optional[int] = None, value_whole: bool = False,
                          decay_1d: bool = False) -> List[TensorSpec]:
    """"Partition for Transformers" (Appendix B) over a list of (name, shape).  1-D tensors (norm gains, biases)
    get wd_scale 0 unless decay_1d (Algorithm 1 itself decays every block; exempting
    1-D gains is the usual practice and is what the benchmark configurations use)."""
    out = []
    for name, shape in named_shapes:
        shape = tuple(int(s) for s in shape)
        bn = block_numel_for(name, shape, n_heads, n_kv_heads, value_whole)
        wd = 1.0 if (len(shape) >= 2 or decay_1d) else 0.0
        out.append(TensorSpec(name, shape, bn, wd))
    return out


def partition_whole(named_shapes: Sequence[Tuple[str, Sequence[int]]], decay_1d: bool = False) -> List[TensorSpec]:
    """"Partition for non-Transformers": every tensor is a single block."""
    out = []
    for name, shape in named_shapes:
        shape = tuple(int(s) for s in shape)
        wd = 1.0 if (len(shape) >= 2 or decay_1d) else 0.0
        out.append(TensorSpec(name, shape, _numel(shape), wd))
    return out


def as_adamw(specs: Sequence[TensorSpec]) -> List[TensorSpec]:
    """The AdamW-equivalent mode: same tensors, every block of size 1."""
    return [TensorSpec(s.name, s.shape, 1, s.wd_scale) for s in specs]


def with_reducer(specs: Sequence[TensorSpec], reducer: str) -> List[TensorSpec]:
    """The same partition with another block statistic in the v update (the candidates of the
    paper's "Ablation Studies on the Design of Adam-mini": 1-norm, 2-norm, max, min of g*g)."""
    if reducer not in ("mean", "norm1", "norm2", "max", "min"):
        raise ValueError("unknown reducer %r" % (reducer,))
    return [TensorSpec(s.name, s.shape, s.block_numel, s.wd_scale, s.strided, reducer) for s in specs]


def transposed(spec: TensorSpec) -> TensorSpec:
    """The same 2-D weight and the same blocks, stored as the transpose: a [rows, cols] tensor cut
    by rows becomes a [cols, rows] tensor whose blocks are its columns (the re-ordering case of the
    paper's Appendix D).  Only for tensors partitioned by their outermost dimension's rows."""
    if len(spec.shape) != 2 or spec.strided or spec.block_numel != spec.shape[1]:
        raise ValueError("transposed() needs a 2-D tensor partitioned by rows")
    return TensorSpec(spec.name + ".T", (spec.shape[1], spec.shape[0]), spec.block_numel, spec.wd_scale, True,
                      spec.reducer)
