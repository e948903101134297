"""Seeded synthetic inputs for a GPT-style pipeline stage.

This module holds no arithmetic of the method itself: it only draws random
numbers, rounds them to the storage type and names the tensors.  Both the CPU
oracle's tests and the HIP path's tests/bench read their inputs from here, so
the two sides always see the same arrays.

Recipe (one ``numpy`` Philox generator per tensor, keyed by ``seed`` and a
stable tensor id, so any tensor can be regenerated on its own):

* weight matrices, biases, token/position embeddings: N(0, 0.02)
* LayerNorm gain: 1 + N(0, 0.02); LayerNorm shift: N(0, 0.02)
* stage input activations and upstream gradients: N(0, 1)
* token ids (first-stage configuration only): uniform integers in [0, vocab)

In bf16 mode every array is rounded once to bf16 (round-to-nearest-even) and
widened back to fp32, so that both sides start from identical values and a
comparison measures compute error, not input quantisation.
"""
from __future__ import annotations

import dataclasses
import zlib

import numpy as np


@dataclasses.dataclass(frozen=True)
class StageShape:
    """Shape of one pipeline stage's share of a GPT model (b = 1)."""

    n_layers: int      # L
    n_chunks: int      # v  (virtual chunks on this rank; L % v == 0)
    hidden: int        # h
    n_heads: int       # a
    ffn: int           # f
    seq: int           # s
    vocab: int = 0     # > 0: chunk 0 starts with a token + position embedding
    dtype: str = "bf16"  # "f32" or "bf16"
    pipeline_degree: int = 1  # d
    rank: int = 0
    n_microbatches: int = 1   # m
    n_kv_heads: int = 0       # key/value heads of grouped-query attention; 0 = n_heads (plain multi-head)

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads or self.n_heads

    @property
    def kv_width(self) -> int:
        """Columns of the key (and of the value) block of the QKV projection."""
        return self.kv_heads * (self.hidden // self.n_heads)

    @property
    def layers_per_chunk(self) -> int:
        return self.n_layers // self.n_chunks

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads


# The five workloads named by the baseline description.
CONFIGS = {
    "C1": StageShape(2, 1, 256, 4, 1024, 128, vocab=1024, dtype="f32", pipeline_degree=2, n_microbatches=4),
    "C2": StageShape(4, 1, 2048, 16, 8192, 2048, dtype="bf16", pipeline_degree=4, n_microbatches=8),
    "C3": StageShape(4, 1, 4096, 32, 16384, 4096, dtype="bf16", pipeline_degree=8, n_microbatches=16),
    "C4": StageShape(4, 2, 4096, 32, 16384, 4096, dtype="bf16", pipeline_degree=8, n_microbatches=32),
    "C5": StageShape(2, 1, 5120, 40, 20480, 16384, dtype="bf16", pipeline_degree=16, n_microbatches=16),
}

# Per-layer parameter tensors, in flat-buffer order: (name, rows, cols) as
# functions of (h, f, q) with q = h + 2 * kv_width, the width of the QKV projection
# (3h for plain multi-head attention).  Vectors have rows == 1.
LAYER_PARAMS = (
    ("ln1_g", lambda h, f, q: (1, h)),
    ("ln1_b", lambda h, f, q: (1, h)),
    ("w_qkv", lambda h, f, q: (h, q)),
    ("b_qkv", lambda h, f, q: (1, q)),
    ("w_o", lambda h, f, q: (h, h)),
    ("b_o", lambda h, f, q: (1, h)),
    ("ln2_g", lambda h, f, q: (1, h)),
    ("ln2_b", lambda h, f, q: (1, h)),
    ("w_fc1", lambda h, f, q: (h, f)),
    ("b_fc1", lambda h, f, q: (1, f)),
    ("w_fc2", lambda h, f, q: (f, h)),
    ("b_fc2", lambda h, f, q: (1, h)),
)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    rounded = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The upper 16 bits of already bf16-representable fp32 values, as uint16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def _rng(seed: int, tag: str) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), zlib.crc32(tag.encode())]))


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    a = a.astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


def layer_params(shape: StageShape, layer: int, seed: int = 1234) -> dict:
    """Named fp32 arrays for one decoder layer (bf16-representable in bf16 mode)."""
    h, f = shape.hidden, shape.ffn
    out = {}
    for name, dims in LAYER_PARAMS:
        r, c = dims(h, f, h + 2 * shape.kv_width)
        g = _rng(seed, f"L{layer}.{name}")
        a = g.standard_normal((r, c), dtype=np.float32) * np.float32(0.02)
        if name in ("ln1_g", "ln2_g"):
            a = a + np.float32(1.0)
        if r == 1:
            a = a.reshape(c)
        out[name] = _store(a, shape.dtype)
    return out


def stage_params(shape: StageShape, seed: int = 1234) -> dict:
    """{'layers': [dict per layer], 'wte': ..., 'wpe': ...} (embeddings iff vocab > 0)."""
    p = {"layers": [layer_params(shape, l, seed) for l in range(shape.n_layers)]}
    if shape.vocab > 0:
        p["wte"] = _store(_rng(seed, "wte").standard_normal((shape.vocab, shape.hidden), dtype=np.float32) * np.float32(0.02), shape.dtype)
        p["wpe"] = _store(_rng(seed, "wpe").standard_normal((shape.seq, shape.hidden), dtype=np.float32) * np.float32(0.02), shape.dtype)
    return p


def unit_input(shape: StageShape, mb: int, chunk: int, seed: int = 1234) -> np.ndarray:
    """Stage input of one (microbatch, chunk) unit: int32 tokens [s] if it feeds
    the embedding (vocab > 0 and chunk 0), else activations [s, h]."""
    if shape.vocab > 0 and chunk == 0:
        return _rng(seed, f"tok.{mb}").integers(0, shape.vocab, size=shape.seq, dtype=np.int32)
    a = _rng(seed, f"x.{mb}.{chunk}").standard_normal((shape.seq, shape.hidden), dtype=np.float32)
    return _store(a, shape.dtype)


def unit_upstream_grad(shape: StageShape, mb: int, chunk: int, seed: int = 1234) -> np.ndarray:
    """Upstream gradient dy [s, h] of one unit."""
    a = _rng(seed, f"dy.{mb}.{chunk}").standard_normal((shape.seq, shape.hidden), dtype=np.float32)
    return _store(a, shape.dtype)
