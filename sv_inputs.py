"""Seeded synthetic inputs shared by the CPU oracle tests and the GPU parity tests.

This module holds no arithmetic of the streaming method itself: it only lays
out token streams (how many vision / text tokens arrive when, and with which
vision grid) and draws Q/K/V values.  Values come from a counter-based
generator, so the value of element (tensor, layer, token id, head, dim) depends
on nothing but the seed and those five coordinates: any chunk of a very long
stream can be produced without replaying the chunks before it.

Stream shapes follow the paper's interleaved vision/text layout at one-second
steps (Sec. 2.2) and the inference budgets of Fig. 3; head shapes are those of
Qwen-2.5-VL-7B attention.  Values are i.i.d. N(0,1); for bf16 workloads each
sample is rounded once to the nearest bf16 (ties to even) and handed out as
float32, so both sides start from identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

TEXT = 0
VISION = 1

TENSOR_Q = 0
TENSOR_K = 1
TENSOR_V = 2

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on uint64 arrays (wrap-around arithmetic)."""
    x = x.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        x ^= x >> np.uint64(30)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


def _key(seed: int, tensor: int, layer: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix64(np.array([seed], dtype=np.uint64) + np.uint64(0x9E3779B97F4A7C15))
        k = _mix64(k ^ np.uint64(tensor * 0x100000001B3 + 0x51ED27))
        k = _mix64(k ^ np.uint64(layer * 0xD6E8FEB86659FD93 & 0xFFFFFFFFFFFFFFFF))
    return k[0]


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result is float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def normal(seed: int, tensor: int, layer: int, gids: np.ndarray, n_heads: int,
           head_dim: int, bf16: bool = False) -> np.ndarray:
    """N(0,1) samples of shape [len(gids), n_heads, head_dim], float32.

    Element (g, h, i) is a pure function of (seed, tensor, layer, gids[g], h, i).
    """
    gids = np.asarray(gids, dtype=np.uint64).reshape(-1, 1, 1)
    h = np.arange(n_heads, dtype=np.uint64).reshape(1, -1, 1)
    i = np.arange(head_dim, dtype=np.uint64).reshape(1, 1, -1)
    key = _key(seed, tensor, layer)
    with np.errstate(over="ignore"):
        ctr = (gids * np.uint64(n_heads) + h) * np.uint64(head_dim) + i
        a = _mix64(ctr * np.uint64(2) + key)
        b = _mix64(ctr * np.uint64(2) + np.uint64(1) + key)
    # Box-Muller from two uniforms in (0,1) built from the top 53 bits.
    u1 = ((a >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    u2 = ((b >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    z = z.astype(np.float32)
    if bf16:
        z = round_to_bf16(z)
    return z


# ----------------------------------------------------------------------------
# Stream layouts
# ----------------------------------------------------------------------------

@dataclass
class Span:
    """One append call: `n` tokens of one type; vision spans may carry a grid."""
    type: int
    n: int
    grid_thw: Optional[Tuple[int, int, int]] = None
    gid0: int = 0  # global arrival id of the span's first token


@dataclass
class Chunk:
    """One second of stream: a vision span, then `n_decode` single text tokens."""
    vision: Span
    n_text: int
    text_gid0: int


@dataclass
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                    # "f32" or "bf16"
    rope_mode: int                # 0 = 1-D, 1 = 3-section M-RoPE
    rope_theta: float
    mrope_sections: Tuple[int, int, int]
    n_sink: int
    vision_window: int            # tokens
    text_window: int              # tokens
    preamble_text: int            # text tokens appended before the first chunk
    vision_per_chunk: int
    text_per_chunk: int
    grid_thw: Optional[Tuple[int, int, int]]
    n_chunks: int
    seed: int

    @property
    def bf16(self) -> bool:
        return self.dtype == "bf16"

    @property
    def tokens_per_chunk(self) -> int:
        return self.vision_per_chunk + self.text_per_chunk

    def chunk(self, c: int) -> Chunk:
        g0 = self.preamble_text + c * self.tokens_per_chunk
        return Chunk(Span(VISION, self.vision_per_chunk, self.grid_thw, g0),
                     self.text_per_chunk, g0 + self.vision_per_chunk)

    def retained_steady(self) -> int:
        return self.n_sink + self.text_window + self.vision_window

    def capacity(self) -> int:
        """Slots needed for the largest cache this workload ever holds."""
        total = self.preamble_text + self.n_chunks * self.tokens_per_chunk
        steady = self.retained_steady() + self.tokens_per_chunk
        # before steady state nothing beyond the budgets is held either
        if self.vision_window < 0 or self.text_window < 0:   # an infinite window: nothing of that class is dropped
            return total
        return min(total, steady + self.preamble_text)

    def qkv(self, layer: int, gids: np.ndarray):
        q = normal(self.seed, TENSOR_Q, layer, gids, self.n_q_heads, self.head_dim, self.bf16)
        k = normal(self.seed, TENSOR_K, layer, gids, self.n_kv_heads, self.head_dim, self.bf16)
        v = normal(self.seed, TENSOR_V, layer, gids, self.n_kv_heads, self.head_dim, self.bf16)
        return q, k, v


def workload_tiny(n_chunks: int = 10) -> Workload:
    """fp32 single layer, 1-D RoPE: 16 vision + 4 text tokens per chunk, budgets 8/32/16."""
    return Workload("tiny_f32", 1, 2, 1, 64, "f32", 0, 10000.0, (0, 0, 0),
                    8, 32, 16, 0, 16, 4, None, n_chunks, 1001)


def workload_qwen_layer(n_chunks: int = 40, n_layers: int = 1, seed: int = 1002) -> Workload:
    """Qwen-2.5-VL-7B-shaped, bf16, M-RoPE: 256 vision (1x16x16) + 16 text per chunk, 512/4096/512."""
    return Workload("qwen7b_256v", n_layers, 28, 4, 128, "bf16", 1, 1.0e6, (16, 24, 24),
                    512, 4096, 512, 512, 256, 16, (1, 16, 16), n_chunks, seed)


def workload_qwen_stream(n_chunks: int = 3600) -> Workload:
    """Full 28-layer, one-hour stream with the shapes and budgets of workload_qwen_layer."""
    w = workload_qwen_layer(n_chunks, 28, 1003)
    w.name = "qwen7b_256v_28L"
    return w


def workload_high_fps(n_chunks: int = 20, n_layers: int = 1) -> Workload:
    """1024 vision tokens per chunk (8 frames x 128 tokens, grid 8x8x16), window 16 chunks."""
    return Workload("qwen7b_1024v", n_layers, 28, 4, 128, "bf16", 1, 1.0e6, (16, 24, 24),
                    512, 16384, 512, 512, 1024, 16, (8, 8, 16), n_chunks, 1004)


@dataclass
class RaggedBatch:
    """16 independent streams with per-stream budgets (decode-only workload)."""
    base: Workload
    n_streams: int
    vision_windows: List[int] = field(default_factory=list)
    text_windows: List[int] = field(default_factory=list)

    def lengths(self) -> List[int]:
        b = self.base
        return [b.n_sink + tw + vw for vw, tw in zip(self.vision_windows, self.text_windows)]


def workload_ragged_batch(n_streams: int = 16, n_layers: int = 1, seed: int = 1005) -> RaggedBatch:
    """Per-stream vision_window = 256*U{4..32}, text_window = U{128..1024}, n_sink = 512."""
    rng = np.random.Generator(np.random.Philox(seed))
    base = workload_qwen_layer(0, n_layers, seed)
    vw = [int(256 * rng.integers(4, 33)) for _ in range(n_streams)]
    tw = [int(rng.integers(128, 1025)) for _ in range(n_streams)]
    return RaggedBatch(base, n_streams, vw, tw)
