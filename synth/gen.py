"""Counter-based seeded generators for weights, token ids, hidden states, lengths.

Every tensor gets its own Philox stream keyed by (seed, layer, tensor id), so a
tensor's values do not depend on which other tensors were drawn before it, and
any layer of a large model can be regenerated alone.

Recipe (the synthetic stand-in for trained Llama-2 weights and request traces):
  * matrices and embeddings  ~ N(0, 0.02)
  * RMSNorm gains            ~ 1 + N(0, 0.02)
  * token ids                ~ uniform integers on [0, vocab)
  * hidden-state inputs      ~ N(0, 1)
  * ragged prompt lengths    ~ uniform integers on [lo, hi] inclusive
Values are drawn in fp32; for a bf16 shape they are rounded once, to nearest
even, and handed out as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class StageShape:
    """Hyper-parameters of the decoder a stage belongs to (data only)."""

    dtype: str  # "f32" or "bf16": storage type of weights and hidden states
    n_layers_total: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int  # 0: the model has no embedding / LM head blocks
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    def with_(self, **kw) -> "StageShape":
        return replace(self, **kw)

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2


# The workloads named by the benchmark definition (shapes only).
CONFIGS: Dict[str, StageShape] = {
    # tiny fp32 decoder, the whole model is one stage
    "tiny_f32": StageShape("f32", 2, 256, 4, 4, 64, 688, 512),
    # Llama-7B-shaped, bf16 (stage = layers 8..15 when used as a middle stage)
    "llama7b": StageShape("bf16", 32, 4096, 32, 32, 128, 11008, 32000),
    # Llama-13B-shaped, bf16
    "llama13b": StageShape("bf16", 40, 5120, 40, 40, 128, 13824, 32000),
    # Llama-70B-shaped with grouped-query attention, bf16
    "llama70b": StageShape("bf16", 80, 8192, 64, 8, 128, 28672, 32000),
}

# Tensor ids are part of the stream key; never renumber.
_TID = {
    "attn_norm": 1,
    "wqkv": 2,
    "wo": 3,
    "ffn_norm": 4,
    "wgu": 5,
    "wd": 6,
    "embed": 7,
    "final_norm": 8,
    "lm_head": 9,
    "tokens": 10,
    "hidden": 11,
    "lengths": 12,
}

# Order in which a layer's tensors are laid into its packed block.
TENSOR_ORDER_LAYER = ("attn_norm", "wqkv", "wo", "ffn_norm", "wgu", "wd")
TENSOR_ORDER_HEAD = ("final_norm", "lm_head")


def _rng(seed: int, layer: int, name: str, extra: int = 0) -> np.random.Generator:
    sub = ((layer + 2) << 40) | (_TID[name] << 32) | (extra & 0xFFFFFFFF)
    key = np.array([np.uint64(seed), np.uint64(sub)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def bf16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); return the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def _store(shape: StageShape, a: np.ndarray) -> np.ndarray:
    return a if shape.dtype == "f32" else bf16_bits_from_f32(a)


def _normal(rng, shp, mean, std) -> np.ndarray:
    out = rng.standard_normal(size=shp, dtype=np.float32)
    out *= np.float32(std)
    if mean:
        out += np.float32(mean)
    return out


def layer_shapes(s: StageShape) -> Dict[str, Tuple[int, ...]]:
    return {
        "attn_norm": (s.hidden,),
        "wqkv": (s.qkv_rows, s.hidden),
        "wo": (s.hidden, s.n_q_heads * s.head_dim),
        "ffn_norm": (s.hidden,),
        "wgu": (2 * s.ffn, s.hidden),
        "wd": (s.hidden, s.ffn),
    }


def layer_tensors(s: StageShape, seed: int, layer: int) -> Dict[str, np.ndarray]:
    """Tensors of decoder layer `layer` (global index), row-major [out, in].

    wqkv stacks the query, key and value projections by rows; wgu stacks the
    gate and up projections by rows.
    """
    out = {}
    for name, shp in layer_shapes(s).items():
        rng = _rng(seed, layer, name)
        if name.endswith("_norm"):
            out[name] = _store(s, _normal(rng, shp, 1.0, 0.02))
        else:
            out[name] = _store(s, _normal(rng, shp, 0.0, 0.02))
    return out


def embed_tensors(s: StageShape, seed: int) -> Dict[str, np.ndarray]:
    rng = _rng(seed, -1, "embed")
    return {"embed": _store(s, _normal(rng, (s.vocab, s.hidden), 0.0, 0.02))}


def head_tensors(s: StageShape, seed: int) -> Dict[str, np.ndarray]:
    return {
        "final_norm": _store(
            s, _normal(_rng(seed, s.n_layers_total, "final_norm"), (s.hidden,), 1.0, 0.02)
        ),
        "lm_head": _store(
            s, _normal(_rng(seed, s.n_layers_total, "lm_head"), (s.vocab, s.hidden), 0.0, 0.02)
        ),
    }


def token_ids(seed: int, n: int, vocab: int, stream: int = 0) -> np.ndarray:
    return _rng(seed, 0, "tokens", stream).integers(0, vocab, size=n, dtype=np.int32)


def hidden_states(s: StageShape, seed: int, rows: int, stream: int = 0) -> np.ndarray:
    """N(0,1) hidden states [rows, hidden] in the shape's storage type."""
    return _store(s, _normal(_rng(seed, 0, "hidden", stream), (rows, s.hidden), 0.0, 1.0))


def ragged_lengths(seed: int, batch: int, lo: int, hi: int) -> np.ndarray:
    return _rng(seed, 0, "lengths").integers(lo, hi + 1, size=batch, dtype=np.int32)
