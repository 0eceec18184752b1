"""CPU oracle for one pipeline stage of a Llama-2-style decoder.  TEST INFRASTRUCTURE.

This file is the slow, plain definition that the HIP path is checked against.
It is imported only by the tests, by the smoke check and by the benchmark's CPU
baseline leg; the product never calls it.  It shares no code with the HIP path.

What it follows.  The paper (Section 2.1) describes inference as autoregressive
generation with a KV cache; Section 4.1 describes an execution pipeline whose
stages each hold a contiguous span of model blocks, receive the previous
stage's intermediate result, hand theirs on, and keep their own KV cache;
Section 5 says each block is one contiguous packed memory region and that
packing does not change what is computed; Section 6 says the per-layer math is
that of Meta's Llama inference code (evaluated on Llama-2 7B/13B/70B).  The
paper itself defines no layer arithmetic, so the operators below are the public
Llama-2 pre-norm decoder block, with the hyper-parameters of the benchmark
configurations.  Because execute-while-load, packing and stage splitting change
only when and where things run, the oracle is simply the plain forward pass.

All arithmetic is float64 with no intermediate rounding.  numpy's matmul is
used as a library step for the projections and for score/value products.

Pins (tests/test_oracle_pins.py): RMSNorm closed forms, RoPE invariants,
attention against a literal triple loop and special cases, matmul orientation
against explicit loops, SwiGLU special values, layer identity cases,
prefill/decode KV consistency, ragged-vs-alone, split invariance, argmax ties,
the final norm + LM head against scalar loops and a closed form, the embedding
and head block layouts against hand-computed offsets.
End-to-end values are "parity unpinned" against any published number: the paper
prints none for this path.

Diagnostic mode (not the parity bar).  OracleStage(..., bf16_handoffs=True) rounds
to bfloat16 (nearest even) at the places where a 16-bit pipeline of this layer
must store an activation in its 16-bit type: the normalised rows that feed a
projection, the q/k/v projections, the rotated q and k, the softmax weights
that multiply the values, the attention output, the SwiGLU output, and the
stage's hidden-state output.  Everything else stays float64.  Random-weight
decoders of this recipe amplify a relative perturbation from layer to layer, so
at depths of tens of layers ANY 16-bit pipeline drifts from the float64 result
by more than its per-layer error; this mode tells that arithmetic drift (it
shows the same drift) from a defect in a kernel (it would not).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np

ALIGN = 256  # every tensor inside a packed block starts on a 256-byte boundary


# ----------------------------------------------------------------------------
# byte formats
# ----------------------------------------------------------------------------
def decode_values(a: np.ndarray) -> np.ndarray:
    """Storage format -> float64.  uint16 holds bf16 bit patterns."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """float64 -> nearest bfloat16 (ties to even) -> float64; used by the diagnostic mode only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    u = (u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64)


def _round_up(n: int, m: int) -> int:
    return (n + m - 1) // m * m


def layer_block_layout(s) -> Dict[str, tuple]:
    """name -> (byte offset, shape) of a decoder layer's packed block.

    Order: attention-norm gain, stacked q/k/v projection [(Hq+2Hkv)*hd, d],
    output projection [d, Hq*hd], FFN-norm gain, stacked gate/up projection
    [2F, d], down projection [d, F]; all row-major [out, in].
    """
    isz = 4 if s.dtype == "f32" else 2
    d, hd = s.hidden, s.head_dim
    entries = [
        ("attn_norm", (d,)),
        ("wqkv", ((s.n_q_heads + 2 * s.n_kv_heads) * hd, d)),
        ("wo", (d, s.n_q_heads * hd)),
        ("ffn_norm", (d,)),
        ("wgu", (2 * s.ffn, d)),
        ("wd", (d, s.ffn)),
    ]
    return _lay(entries, isz)


def embed_block_layout(s) -> Dict[str, tuple]:
    return _lay([("embed", (s.vocab, s.hidden))], 4 if s.dtype == "f32" else 2)


def head_block_layout(s) -> Dict[str, tuple]:
    return _lay(
        [("final_norm", (s.hidden,)), ("lm_head", (s.vocab, s.hidden))],
        4 if s.dtype == "f32" else 2,
    )


def _lay(entries, isz):
    out, off = {}, 0
    for name, shp in entries:
        out[name] = (off, shp)
        off = _round_up(off + int(np.prod(shp)) * isz, ALIGN)
    out["__bytes__"] = (off, ())
    return out


def unpack_block(s, layout: Dict[str, tuple], buf: np.ndarray) -> Dict[str, np.ndarray]:
    """Read the tensors of a packed block (uint8 buffer) as float64 arrays."""
    buf = np.asarray(buf).view(np.uint8).reshape(-1)
    assert buf.size == layout["__bytes__"][0], "packed block has the wrong size"
    st = np.float32 if s.dtype == "f32" else np.uint16
    out = {}
    for name, (off, shp) in layout.items():
        if name == "__bytes__":
            continue
        n = int(np.prod(shp))
        raw = buf[off : off + n * np.dtype(st).itemsize].view(st).reshape(shp)
        out[name] = decode_values(raw)
    return out


# ----------------------------------------------------------------------------
# operators
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gamma: np.ndarray, eps: float) -> np.ndarray:
    """y_i = x_i / sqrt(mean_j x_j^2 + eps) * gamma_i, row by row."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gamma


def rope(u: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding on [rows, heads, head_dim]; row r sits at position pos[r].

    Adjacent elements (2i, 2i+1) of a head form a pair that is rotated by the
    angle pos * base^(-2i/head_dim).
    """
    hd = u.shape[-1]
    i = np.arange(hd // 2, dtype=np.float64)
    theta = np.power(float(base), -2.0 * i / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]  # [rows, hd/2]
    c, sn = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    u0, u1 = u[..., 0::2], u[..., 1::2]
    out = np.empty_like(u)
    out[..., 0::2] = u0 * c - u1 * sn
    out[..., 1::2] = u0 * sn + u1 * c
    return out


def attention_rows(q: np.ndarray, k: np.ndarray, v: np.ndarray, pos: np.ndarray, round_weights=None) -> np.ndarray:
    """Causal softmax attention of one sequence.

    q   [n, Hq, hd]   the n query rows, row r at absolute position pos[r]
    k,v [Hkv, ctx, hd] cached keys / values at positions 0..ctx-1
    Query head h reads kv head h // (Hq/Hkv).  Key j is visible to row r iff
    j <= pos[r].  Scores are scaled by 1/sqrt(hd).  round_weights (diagnostic mode
    only) is applied to the un-normalised softmax weights that multiply v.
    """
    n, hq, hd = q.shape
    hkv, ctx, _ = k.shape
    g = hq // hkv
    out = np.empty((n, hq, hd), dtype=np.float64)
    visible = np.arange(ctx)[None, :] <= np.asarray(pos)[:, None]  # [n, ctx]
    for h in range(hq):
        s = q[:, h, :] @ k[h // g].T / math.sqrt(hd)
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        if round_weights is None:
            p = p / p.sum(axis=-1, keepdims=True)
            out[:, h, :] = p @ v[h // g]
        else:
            out[:, h, :] = (round_weights(p) @ v[h // g]) / p.sum(axis=-1, keepdims=True)
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def head_logits(x: np.ndarray, gamma: np.ndarray, w_head: np.ndarray, eps: float) -> np.ndarray:
    """Final norm and LM head: logits[r, v] = sum_i RMSNorm(x[r]; gamma)_i * w_head[v, i].

    x [rows, d] is the residual stream after the last layer at the rows that
    produce a token; w_head is [vocab, d] (row-major [out, in] like every matrix).
    """
    return rmsnorm(x, gamma, eps) @ w_head.T


def greedy(logits: np.ndarray) -> np.ndarray:
    """argmax per row; the lowest index wins a tie."""
    return np.argmax(logits, axis=-1).astype(np.int32)


# ----------------------------------------------------------------------------
# the stage
# ----------------------------------------------------------------------------
class OracleStage:
    """Layers [layer_lo, layer_hi) of a decoder with shape `s`.

    A stage whose span starts at layer 0 of a model with a vocabulary takes
    token ids and gathers embeddings; otherwise it takes hidden states.  A
    stage whose span ends at the last layer of a model with a vocabulary
    applies the final norm and the LM head to the last row of every sequence
    and returns (next token ids, logits); otherwise it returns the residual
    stream after its last layer, un-normalised.
    """

    def __init__(self, s, layer_lo: int, layer_hi: int, max_batch: int, max_seq: int, bf16_handoffs: bool = False):
        assert 0 <= layer_lo < layer_hi <= s.n_layers_total
        # diagnostic mode (see the file header): identity unless switched on
        self._r = round_bf16 if bf16_handoffs else (lambda a: a)
        self._rw = round_bf16 if bf16_handoffs else None
        self.round_output = bf16_handoffs  # a middle stage's hidden-state output is stored in 16 bits too
        self.s, self.lo, self.hi = s, layer_lo, layer_hi
        self.first = s.vocab > 0 and layer_lo == 0
        self.last = s.vocab > 0 and layer_hi == s.n_layers_total
        self.w: Dict[int, Dict[str, np.ndarray]] = {}
        self.max_batch, self.max_seq = max_batch, max_seq
        nl = layer_hi - layer_lo
        self.k = np.zeros((nl, max_batch, s.n_kv_heads, max_seq, s.head_dim))
        self.v = np.zeros_like(self.k)
        self.seq_lens = np.zeros(max_batch, dtype=np.int64)

    # -- weights ------------------------------------------------------------
    def load_block(self, layer: int, buf: np.ndarray) -> None:
        """Take one packed block: layer index, -1 (embedding) or L (head)."""
        s = self.s
        if layer == -1:
            lay = embed_block_layout(s)
        elif layer == s.n_layers_total:
            lay = head_block_layout(s)
        else:
            lay = layer_block_layout(s)
        self.w[layer] = unpack_block(s, lay, buf)

    def load_tensors(self, layer: int, tensors: Dict[str, np.ndarray]) -> None:
        """Take the same tensors unpacked (storage format or float)."""
        self.w[layer] = {k: decode_values(v) for k, v in tensors.items()}

    # -- one decoder layer ----------------------------------------------------
    def _layer(self, li: int, x: np.ndarray, seq_of_row, pos, rows_of_seq) -> np.ndarray:
        s, w = self.s, self.w[self.lo + li]
        hq, hkv, hd = s.n_q_heads, s.n_kv_heads, s.head_dim
        r = self._r
        y = r(rmsnorm(x, w["attn_norm"], s.rms_eps))
        qkv = r(y @ w["wqkv"].T)
        q = qkv[:, : hq * hd].reshape(-1, hq, hd)
        k = qkv[:, hq * hd : (hq + hkv) * hd].reshape(-1, hkv, hd)
        v = qkv[:, (hq + hkv) * hd :].reshape(-1, hkv, hd)
        q = r(rope(q, pos, s.rope_base))
        k = r(rope(k, pos, s.rope_base))
        # append to the cache, then attend over everything cached so far
        sq = np.asarray(seq_of_row)
        self.k[li, sq, :, pos, :] = k  # row r goes to [li, seq r, every kv head, pos r, :]
        self.v[li, sq, :, pos, :] = v
        o = np.empty_like(q)
        for b, rows in rows_of_seq.items():
            ctx = int(pos[rows[-1]]) + 1
            o[rows] = attention_rows(q[rows], self.k[li, b, :, :ctx], self.v[li, b, :, :ctx], pos[rows], self._rw)
        x = x + r(o).reshape(-1, hq * hd) @ w["wo"].T
        y = r(rmsnorm(x, w["ffn_norm"], s.rms_eps))
        gu = y @ w["wgu"].T
        h = r(silu(gu[:, : s.ffn]) * gu[:, s.ffn :])
        return x + h @ w["wd"].T

    def _run(self, inp, seq_of_row, pos, rows_of_seq, last_rows):
        s = self.s
        if self.first:
            x = self.w[-1]["embed"][np.asarray(inp, dtype=np.int64)]
        else:
            x = decode_values(inp).reshape(-1, s.hidden)
        for li in range(self.hi - self.lo):
            x = self._layer(li, x, seq_of_row, pos, rows_of_seq)
        if not self.last:
            return round_bf16(x) if self.round_output else x
        wl = self.w[s.n_layers_total]
        if self._rw is not None:  # diagnostic mode: the normalised rows are stored in 16 bits
            logits = self._r(rmsnorm(x[last_rows], wl["final_norm"], s.rms_eps)) @ wl["lm_head"].T
            return greedy(logits), logits
        logits = head_logits(x[last_rows], wl["final_norm"], wl["lm_head"], s.rms_eps)
        return greedy(logits), logits

    # -- entry points ---------------------------------------------------------
    def prefill(self, inp, lengths: Sequence[int]):
        """Prompt pass.  Rows are packed sequence after sequence (no padding);
        sequence b has lengths[b] rows at positions 0..lengths[b]-1."""
        lengths = [int(n) for n in lengths]
        assert len(lengths) <= self.max_batch and max(lengths) <= self.max_seq
        seq_of_row, pos, rows_of_seq, last_rows, r = [], [], {}, [], 0
        for b, n in enumerate(lengths):
            seq_of_row += [b] * n
            pos += list(range(n))
            rows_of_seq[b] = list(range(r, r + n))
            r += n
            last_rows.append(r - 1)
        out = self._run(inp, seq_of_row, np.array(pos), rows_of_seq, last_rows)
        self.seq_lens[:] = 0
        self.seq_lens[: len(lengths)] = lengths
        self.batch = len(lengths)
        return out

    def decode(self, inp):
        """One generation step: one new row per sequence, at position seq_lens[b]."""
        bsz = self.batch
        pos = self.seq_lens[:bsz].copy()
        assert pos.max() < self.max_seq
        rows_of_seq = {b: [b] for b in range(bsz)}
        out = self._run(inp, list(range(bsz)), pos, rows_of_seq, list(range(bsz)))
        self.seq_lens[:bsz] += 1
        return out
