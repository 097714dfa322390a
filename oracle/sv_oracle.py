"""CPU oracle for the streaming KV-cache hot path of StreamingVLM (arXiv 2510.09608).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 statement of what one
per-chunk inference step computes; it exists so that the HIP library can be
checked against it.  Nothing in the product path may import it: only tests,
the smoke check and the CPU-baseline leg of the benchmark do.  It shares no
code, tables or helpers with the HIP path.

The method is exact once the retained set is fixed (there is no approximation
inside the path), so every function below is the definition written out:

  * which tokens stay          -- Sec. 2.1 "Streaming-aware KV Cache", Fig. 3
  * which positions they get   -- Sec. 2.1 "Contiguous RoPE" (1-D and 3-D)
  * what the attention returns -- causal softmax attention over the retained
                                  tokens with Q/K rotated at those positions

Raw (un-rotated) K is kept for every retained token and rotated once at its
final position whenever attention is evaluated, so no rounding accumulates.

Readings of the paper where it is silent (kept identical in the C ABI):
  - "sink" = the first n_sink tokens counted over TEXT tokens only;
  - sink, text window and vision window are three independent budgets, a token
    in both sink and window is kept once;
  - budgets count tokens present when evict() is called (the past), the new
    chunk is appended afterwards;
  - 1-D contiguous position = index in the compacted cache;
  - 3-D rule = the public Qwen2-VL M-RoPE convention: a text token has
    t = h = w = next, next += 1; a vision block with grid (T, H, W) starts at
    base = next, token (lt, lh, lw) sits at (base+lt, base+lh, base+lw), and
    after the block next = base + max(T, H, W).  A block that lost its oldest
    tokens to eviction keeps local coordinates and extent;
  - rotate-half pairing (i, i + d/2), frequency i uses theta^(-2i/d); in 3-D
    mode the first s_t frequencies read the t index, the next s_h the h index,
    the last s_w the w index;
  - query head h reads kv head h // (H_q / H_kv); scale 1/sqrt(d).

Parity pins (tests/test_oracle_pins.py): hand-enumerated retained sets and
positions (tests/golden), brute-force causal attention in pure Python loops,
closed forms (constant V, equal keys, one key), RoPE group laws and relative-
position invariance, GQA == MHA with repeated KV, incremental == one-shot
eviction.  The 3-D rule, the pairing and the causal reading are not printed by
the paper: for those, parity is unpinned by the paper and rests on the
readings above plus internal consistency.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

TEXT = 0
VISION = 1
ROPE_1D = 0
ROPE_3D = 1
ROPE_NONE = 2
INF = -1  # a window of -1 keeps every token of that class


class OracleStream:
    """One stream's cache as a list of retained tokens in arrival order."""

    def __init__(self, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                 rope_mode: int = ROPE_1D, rope_theta: float = 10000.0,
                 mrope_sections: Sequence[int] = (0, 0, 0)):
        assert n_q_heads % n_kv_heads == 0 and head_dim % 2 == 0
        if rope_mode == ROPE_3D:
            assert sum(mrope_sections) == head_dim // 2
        self.L, self.Hq, self.Hkv, self.d = n_layers, n_q_heads, n_kv_heads, head_dim
        self.rope_mode, self.theta, self.sections = rope_mode, float(rope_theta), tuple(mrope_sections)
        # per retained token (parallel lists)
        self.gid: List[int] = []
        self.type: List[int] = []
        self.rank: List[int] = []      # index among tokens of the same type ever appended
        self.blk: List[int] = []       # vision block id, -1 for text / 1-D vision
        self.local: List[Tuple[int, int, int]] = []
        self.extent: List[int] = []
        # raw K, V per layer, one [Hkv, d] fp64 array per retained token
        self.k: List[List[np.ndarray]] = [[] for _ in range(n_layers)]
        self.v: List[List[np.ndarray]] = [[] for _ in range(n_layers)]
        self.n_text = 0
        self.n_vis = 0
        self.next_gid = 0
        self.next_blk = 0

    def __len__(self) -> int:
        return len(self.gid)

    # -- Sec. 2.1: new tokens join the cache in arrival order -----------------
    def append_meta(self, types: Sequence[int], grid_thw: Optional[Tuple[int, int, int]] = None) -> int:
        """Register len(types) new tokens; returns the slot of the first one."""
        slot0 = len(self.gid)
        n = len(types)
        if grid_thw is not None:
            T, H, W = grid_thw
            assert all(t == VISION for t in types) and n == T * H * W
            blk = self.next_blk
            self.next_blk += 1
            ext = max(T, H, W)
        for j, ty in enumerate(types):
            self.gid.append(self.next_gid)
            self.next_gid += 1
            self.type.append(ty)
            if ty == TEXT:
                self.rank.append(self.n_text)
                self.n_text += 1
            else:
                self.rank.append(self.n_vis)
                self.n_vis += 1
            if grid_thw is not None:
                self.blk.append(blk)
                self.local.append((j // (H * W), (j // W) % H, j % W))
                self.extent.append(ext)
            else:
                assert not (self.rope_mode == ROPE_3D and ty == VISION), "3-D RoPE needs a vision grid"
                self.blk.append(-1)
                self.local.append((0, 0, 0))
                self.extent.append(1)
        return slot0

    def append_kv(self, layer: int, k: np.ndarray, v: np.ndarray) -> None:
        """Store raw K, V rows ([n, Hkv, d]) of the tokens registered last, for one layer."""
        k = np.asarray(k, dtype=np.float64)
        v = np.asarray(v, dtype=np.float64)
        assert k.shape == v.shape and k.shape[1:] == (self.Hkv, self.d)
        for j in range(k.shape[0]):
            self.k[layer].append(k[j].copy())
            self.v[layer].append(v[j].copy())
        assert len(self.k[layer]) <= len(self.gid)

    # -- Sec. 2.1 "Streaming-aware KV Cache": sink text + text window + vision window
    def keep_flags(self, n_sink: int, vision_window: int, text_window: int) -> List[bool]:
        flags = []
        for ty, r in zip(self.type, self.rank):
            if ty == TEXT:
                in_sink = r < n_sink
                in_window = text_window == INF or r >= self.n_text - text_window
                flags.append(in_sink or in_window)
            else:
                flags.append(vision_window == INF or r >= self.n_vis - vision_window)
        return flags

    def evict(self, n_sink: int, vision_window: int, text_window: int) -> int:
        """Drop every token outside the three budgets; survivors keep their order."""
        keep = self.keep_flags(n_sink, vision_window, text_window)
        idx = [i for i, f in enumerate(keep) if f]
        for name in ("gid", "type", "rank", "blk", "local", "extent"):
            old = getattr(self, name)
            setattr(self, name, [old[i] for i in idx])
        for l in range(self.L):
            assert len(self.k[l]) == len(keep), "evict with a half-appended layer"
            self.k[l] = [self.k[l][i] for i in idx]
            self.v[l] = [self.v[l][i] for i in idx]
        return len(idx)

    # -- Sec. 2.1 "Contiguous RoPE": positions are re-assigned from the retained list
    def positions(self) -> np.ndarray:
        """[N, 3] int64 positions (t, h, w) of the retained tokens; 1-D mode repeats the index."""
        n = len(self.gid)
        pos = np.zeros((n, 3), dtype=np.int64)
        if self.rope_mode != ROPE_3D:
            for i in range(n):
                pos[i, :] = i
            return pos
        nxt = 0
        base = 0
        for i in range(n):
            if self.type[i] == TEXT:
                pos[i, :] = nxt
                nxt += 1
                continue
            first = i == 0 or self.blk[i - 1] != self.blk[i]
            last = i == n - 1 or self.blk[i + 1] != self.blk[i]
            if first:
                base = nxt
            lt, lh, lw = self.local[i]
            pos[i] = (base + lt, base + lh, base + lw)
            if last:
                nxt = base + self.extent[i]
        return pos

    def next_position(self) -> int:
        """Scalar position the next appended token would start from."""
        n = len(self.gid)
        if self.rope_mode != ROPE_3D:
            return n
        nxt = 0
        base = 0
        for i in range(n):
            if self.type[i] == TEXT:
                nxt += 1
                continue
            if i == 0 or self.blk[i - 1] != self.blk[i]:
                base = nxt
            if i == n - 1 or self.blk[i + 1] != self.blk[i]:
                nxt = base + self.extent[i]
        return nxt

    # -- attention of queries sitting at given slots ---------------------------
    def attend(self, layer: int, q: np.ndarray, slots: Sequence[int], causal: bool = True) -> np.ndarray:
        """q: raw [n, Hq, d]; query j sits at cache slot slots[j].  Returns [n, Hq, d] fp64."""
        pos = self.positions()
        n = len(self.gid)
        assert len(self.k[layer]) == n
        K = np.stack(self.k[layer]) if n else np.zeros((0, self.Hkv, self.d))
        V = np.stack(self.v[layer]) if n else np.zeros((0, self.Hkv, self.d))
        Kr = rope(K, pos, self.rope_mode, self.theta, self.sections)
        q = np.asarray(q, dtype=np.float64)
        Qr = rope(q, pos[np.asarray(slots, dtype=np.int64)], self.rope_mode, self.theta, self.sections)
        return gqa_attention(Qr, Kr, V, np.asarray(slots, dtype=np.int64), causal)


def inv_freq(head_dim: int, theta: float) -> np.ndarray:
    """theta^(-2i/d) for i = 0 .. d/2-1 (rotary frequencies)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.float64(theta) ** (-2.0 * i / head_dim)


def rope_angles(pos: np.ndarray, head_dim: int, rope_mode: int, theta: float,
                sections: Sequence[int]) -> np.ndarray:
    """[N, d/2] rotation angles.  pos is [N, 3]; 1-D mode reads column 0."""
    pos = np.asarray(pos, dtype=np.float64).reshape(-1, 3)
    f = inv_freq(head_dim, theta)
    half = head_dim // 2
    if rope_mode == ROPE_NONE:
        return np.zeros((pos.shape[0], half))
    if rope_mode == ROPE_1D:
        return pos[:, 0:1] * f[None, :]
    # 3-D: frequency i reads t for i < s_t, h for the next s_h, w for the last s_w
    sec = np.repeat(np.arange(3), np.asarray(sections, dtype=np.int64))
    assert sec.shape[0] == half
    return pos[:, sec] * f[None, :]


def rope(x: np.ndarray, pos: np.ndarray, rope_mode: int, theta: float,
         sections: Sequence[int]) -> np.ndarray:
    """Rotate x [N, H, d] at positions pos [N, 3]: pairs (i, i + d/2) turn by angle_i."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    a = rope_angles(pos, d, rope_mode, theta, sections)[:, None, :]
    c, s = np.cos(a), np.sin(a)
    lo, hi = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    return out


def gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_slots: np.ndarray,
                  causal: bool = True) -> np.ndarray:
    """softmax(q k^T / sqrt(d)) v with grouped heads; query j sees keys at slots <= q_slots[j].

    q [n, Hq, d], k and v [N, Hkv, d], already rotated.  fp64, max subtracted.
    """
    n, Hq, d = q.shape
    N, Hkv, _ = k.shape
    g = Hq // Hkv
    out = np.zeros((n, Hq, d), dtype=np.float64)
    key_slot = np.arange(N)
    for h in range(Hq):
        kv = h // g
        s = (q[:, h, :] @ k[:, kv, :].T) / np.sqrt(np.float64(d))      # [n, N]
        if causal:
            s = np.where(key_slot[None, :] <= q_slots[:, None], s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, kv, :]
    return out
