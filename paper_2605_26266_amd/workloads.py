"""Seeded synthetic inputs shaped like the benchmark configurations.

This module only produces numbers: it contains none of the method's arithmetic
(no rotation, no quantizer, no attention).  Both the CPU oracle's tests and the
GPU path's tests/bench feed from it, so the two sides see identical inputs.

Recipe (every config):
  * values are i.i.d. N(0,1) drawn with numpy's counter-based Philox bit
    generator, keyed by (seed, tensor id, chunk index, head) so that any
    (chunk, head) block can be produced on its own, in any order;
  * keys get channel-wise outliers: a fixed set of channels per head (chosen
    once from the seed, identical for every token and chunk) is multiplied by
    ``outlier_scale`` -- the "few channels much larger than the rest" structure
    that motivates the Hadamard rotation (paper, Preliminaries, "Hadamard
    rotation");
  * everything is then rounded to the nearest BF16 value (ties to even) and
    magnitudes below 2**-20 are flushed to zero, which keeps every rotated sum
    exactly representable in double precision;
  * layout is [token][head][channel], batch 1.

The shapes stand in for the video-diffusion workloads of the paper (several
thousand tokens per chunk, head dimension 128, a window of cached chunks); the
paper's real activations are not available.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Iterable, Optional, Sequence

import numpy as np

_TENSOR_Q, _TENSOR_K, _TENSOR_V, _TENSOR_OUTLIER = 0, 1, 2, 3
_FLUSH_BELOW = 2.0 ** -20


@dataclass(frozen=True)
class Workload:
    name: str
    num_heads: int
    head_dim: int
    chunk_tokens: int          # tokens per chunk (= queries M = current keys N_R)
    cached_chunks: int         # chunks already in the cache when attention runs
    bits: int
    io_dtype: str              # "bf16" or "fp32" (fp32 arrays still hold BF16-representable values)
    seed: int
    outlier_channels: int      # number of key channels scaled up, per head
    outlier_scale: float
    repeat_chunk: bool = False  # stream config: the same chunk is appended every time

    @property
    def cached_tokens(self) -> int:
        return self.chunk_tokens * self.cached_chunks

    @property
    def attention_flop(self) -> float:
        """4*H*M*(N_S+N_R)*d: QK^T and PV, multiply and add each counted."""
        m = self.chunk_tokens
        return 4.0 * self.num_heads * m * (self.cached_tokens + m) * self.head_dim

    def quantize_bytes(self, n_tokens: Optional[int] = None, meta_bytes: int = 8) -> float:
        """Bytes one append moves: K and V read once, codes + (scale, zero) written once.
        meta_bytes per token and tensor: 8 (fp32 pair) or 3 per group (FP8 scale + BF16 zero-point)."""
        n = self.chunk_tokens if n_tokens is None else n_tokens
        elt = 2 if self.io_dtype == "bf16" else 4
        per_row = self.head_dim * elt + self.head_dim * self.bits // 8 + meta_bytes
        return 2.0 * n * self.num_heads * per_row

    def with_bits(self, bits: int) -> "Workload":
        return replace(self, bits=bits)


WORKLOADS = {
    "tiny": Workload("tiny", 1, 64, 64, 4, 2, "fp32", 0, 4, 8.0),
    "small": Workload("small", 8, 128, 1024, 4, 2, "bf16", 1, 3, 10.0),
    "mid": Workload("mid", 24, 128, 4680, 6, 2, "bf16", 2, 3, 10.0),
    "large": Workload("large", 48, 128, 4096, 16, 2, "bf16", 3, 3, 10.0),
    "stream": Workload("stream", 48, 128, 4096, 32, 2, "bf16", 4, 3, 10.0, repeat_chunk=True),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest BF16 value (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    out = r.view(np.float32).copy()
    out[np.abs(out) < _FLUSH_BELOW] = 0.0
    return out


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array of BF16-representable values -> uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_float(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(seed: int, tensor: int, chunk: int, head: int, shape) -> np.ndarray:
    gen = np.random.Generator(np.random.Philox(key=[(seed << 8) | tensor, (chunk << 16) | head]))
    return gen.standard_normal(shape, dtype=np.float32)


def outlier_channels(w: Workload, head: int) -> np.ndarray:
    """The key channels of `head` that carry outliers (sorted, fixed by the seed)."""
    gen = np.random.Generator(np.random.Philox(key=[(w.seed << 8) | _TENSOR_OUTLIER, head]))
    return np.sort(gen.permutation(w.head_dim)[: w.outlier_channels])


def _heads(w: Workload, heads: Optional[Iterable[int]]) -> Sequence[int]:
    return list(range(w.num_heads)) if heads is None else list(heads)


def chunk_kv(w: Workload, chunk: int, heads: Optional[Iterable[int]] = None, n_tokens: Optional[int] = None):
    """K and V of chunk number `chunk` as float32 [n][len(heads)][d] (BF16-representable).

    Chunks 0..cached_chunks-1 are the cached ones, chunk `cached_chunks` is the
    current chunk.  With repeat_chunk the same block is returned for every index.
    `n_tokens` < chunk_tokens returns the leading tokens of the same block.
    """
    hs = _heads(w, heads)
    n = w.chunk_tokens
    c = 0 if w.repeat_chunk else chunk
    k = np.empty((n, len(hs), w.head_dim), dtype=np.float32)
    v = np.empty_like(k)
    for j, h in enumerate(hs):
        kh = _normal(w.seed, _TENSOR_K, c, h, (n, w.head_dim))
        kh[:, outlier_channels(w, h)] *= np.float32(w.outlier_scale)
        k[:, j, :] = kh
        v[:, j, :] = _normal(w.seed, _TENSOR_V, c, h, (n, w.head_dim))
    k, v = round_to_bf16(k), round_to_bf16(v)
    if n_tokens is not None:
        k, v = k[:n_tokens], v[:n_tokens]
    return k, v


def chunk_q(w: Workload, heads: Optional[Iterable[int]] = None, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Queries of the current chunk, float32 [M][len(heads)][d] (optionally a row subset)."""
    hs = _heads(w, heads)
    q = np.empty((w.chunk_tokens, len(hs), w.head_dim), dtype=np.float32)
    for j, h in enumerate(hs):
        q[:, j, :] = _normal(w.seed, _TENSOR_Q, w.cached_chunks, h, (w.chunk_tokens, w.head_dim))
    q = round_to_bf16(q)
    return q if rows is None else q[rows]


def sample_rows(w: Workload, count: int, salt: int = 0) -> np.ndarray:
    """A sorted, seeded subset of query rows that always includes the first and last row."""
    m = w.chunk_tokens
    if count >= m:
        return np.arange(m)
    gen = np.random.Generator(np.random.Philox(key=[(w.seed << 8) | 0x7F, salt]))
    rows = set(gen.choice(m, size=count, replace=False).tolist())
    rows.update((0, m - 1))
    return np.array(sorted(rows))[:max(count, 2)]
