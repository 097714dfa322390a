"""Oracle driver for the per-second stream loop (TEST INFRASTRUCTURE ONLY).

One step per second of video, in the order the method states it (Sec. 2.1):
cut the past to the three budgets, re-assign contiguous positions, take in the
new vision chunk and attend from it (chunk prefill), then decode the second's
text tokens one at a time, each attending to everything retained so far.
Inputs come from the seeded generators in sv_inputs; all arithmetic is the
oracle's (oracle.sv_oracle), in fp64.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

import sv_inputs as si
from oracle.sv_oracle import OracleStream, TEXT, VISION


def new_stream(w: si.Workload, layers: Sequence[int]) -> OracleStream:
    """Oracle cache holding only the listed model layers (index j holds layers[j])."""
    return OracleStream(len(layers), w.n_q_heads, w.n_kv_heads, w.head_dim,
                        w.rope_mode, w.rope_theta, w.mrope_sections)


def append_preamble(st: OracleStream, w: si.Workload, layers: Sequence[int]) -> None:
    """Text that precedes the video (system prompt and previous text): K/V only."""
    if w.preamble_text == 0:
        return
    gids = np.arange(w.preamble_text)
    st.append_meta([TEXT] * w.preamble_text)
    for j, l in enumerate(layers):
        _, k, v = w.qkv(l, gids)
        st.append_kv(j, k, v)


def step_chunk(st: OracleStream, w: si.Workload, c: int, layers: Sequence[int],
               want_outputs: bool = True) -> Dict[str, object]:
    """Run chunk c.  Returns retained ids / positions after the evict and the attention outputs."""
    n_ret = st.evict(w.n_sink, w.vision_window, w.text_window)
    res: Dict[str, object] = {
        "n_retained": n_ret,
        "gids_after_evict": list(st.gid),
        "pos_after_evict": st.positions().copy(),
    }
    ch = w.chunk(c)
    nv = ch.vision.n
    gids = np.arange(ch.vision.gid0, ch.vision.gid0 + nv)
    slot0 = st.append_meta([VISION] * nv, ch.vision.grid_thw)
    prefill: List[np.ndarray] = []
    qs = []
    for j, l in enumerate(layers):
        q, k, v = w.qkv(l, gids)
        st.append_kv(j, k, v)
        qs.append(q)
    if want_outputs:
        for j, l in enumerate(layers):
            prefill.append(st.attend(j, qs[j], list(range(slot0, slot0 + nv)), causal=True))
    decode: List[List[np.ndarray]] = []
    for t in range(ch.n_text):
        gid = np.array([ch.text_gid0 + t])
        slot = st.append_meta([TEXT])
        outs = []
        for j, l in enumerate(layers):
            q, k, v = w.qkv(l, gid)
            st.append_kv(j, k, v)
            if want_outputs:
                outs.append(st.attend(j, q, [slot], causal=True))
        decode.append(outs)
    res["prefill"] = prefill          # per layer [nv, Hq, d]
    res["decode"] = decode            # per decode step, per layer [1, Hq, d]
    res["gids_end"] = list(st.gid)
    res["pos_end"] = st.positions().copy()
    return res
