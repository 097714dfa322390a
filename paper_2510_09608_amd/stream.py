"""Per-second stream loop over the C calls (call sequencing only, no arithmetic).

Order per chunk, as the method states it (Sec. 2.1): cut the past to the three
budgets (evict + compaction + contiguous re-index), then layer by layer store
the new vision chunk's K/V, rotate its Q and run chunk-prefill attention, then
for each decoded text token do the same with one query (decode attention).
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from .binding import Cache, SV_TEXT, SV_VISION


class StreamRunner:
    def __init__(self, cache: Cache, n_sink: int, vision_window: int, text_window: int, stream_id: int = 0,
                 fused_decode: bool = True):
        self.cache = cache
        self.fused_decode = fused_decode
        self.budgets = (n_sink, vision_window, text_window)
        self.sid = stream_id
        self.L = cache.cfg.n_layers
        self._ids = np.array([stream_id], dtype=np.int32)

    def preamble(self, k_layers: Sequence, v_layers: Sequence) -> None:
        """Text that precedes the video: stored only (K/V per layer, [n, Hkv, d])."""
        n = int(k_layers[0].shape[0])
        types = np.zeros(n, dtype=np.uint8)
        for l in range(self.L):
            self.cache.append(self.sid, l, types if l == 0 else None, None, k_layers[l], v_layers[l])

    def evict(self) -> int:
        return self.cache.evict(self.sid, *self.budgets)

    def prefill(self, q_layers: Sequence, k_layers: Sequence, v_layers: Sequence, o_layers: Sequence,
                grid_thw: Optional[Sequence[int]]) -> int:
        """Vision chunk: q is rotated in place; o_layers[l] receives the attention output."""
        n = int(k_layers[0].shape[0])
        types = np.full(n, SV_VISION, dtype=np.uint8)
        slot0 = -1
        for l in range(self.L):
            slot0 = self.cache.append(self.sid, l, types if l == 0 else None, grid_thw if l == 0 else None,
                                      k_layers[l], v_layers[l])
            self.cache.rope_apply(self.sid, slot0, n, q_layers[l], None)
            self.cache.attn_chunk(self.sid, l, q_layers[l], o_layers[l], True)
        return slot0

    def decode(self, q_layers: Sequence, k_layers: Sequence, v_layers: Sequence, o_layers: Sequence) -> int:
        """One text token: q/k/v per layer are [1, H, d].  Fused: one launch per layer, q is left un-rotated."""
        if self.fused_decode:
            for l in range(self.L):
                self.cache.decode_step(l, self._ids, q_layers[l], k_layers[l], v_layers[l], o_layers[l])
            return self.cache.len(self.sid) - 1
        types = np.zeros(1, dtype=np.uint8)
        slot = -1
        for l in range(self.L):
            slot = self.cache.append(self.sid, l, types if l == 0 else None, None, k_layers[l], v_layers[l])
            self.cache.rope_apply(self.sid, slot, 1, q_layers[l], None)
            self.cache.attn_decode(l, self._ids, q_layers[l], o_layers[l])
        return slot
