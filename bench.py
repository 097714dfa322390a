#!/usr/bin/env python3
"""Benchmark of the streaming KV-cache hot path on one MI355X.

One "step" is one second of stream through the whole path for all 28 layers of
a Qwen-2.5-VL-7B-shaped decoder at steady state (retained cache = 512 sink text
+ 512 recent text + 4096 recent vision tokens): evict + compaction + contiguous
re-index, then per layer append + RoPE + chunk-prefill attention for the 256
new vision tokens, then 16 decode steps of append + RoPE + decode attention.
Inputs are synthetic N(0,1) bf16 tensors already resident in HBM.

Prints ONE JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=40, help="untimed chunks; >= 33 reaches steady state")
    ap.add_argument("--workload", default="qwen7b_256v_28L", choices=["qwen7b_256v_28L", "qwen7b_1024v_28L"])
    ap.add_argument("--layers", type=int, default=28)
    ap.add_argument("--pool", type=int, default=6, help="distinct pre-generated chunks cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--roofline-kernel", default="attn_chunk", choices=["attn_chunk", "attn_decode", "compact"])
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2510_09608_amd as sv
    import sv_inputs as si
    from paper_2510_09608_amd.stream import StreamRunner

    if not os.path.exists(sv.lib_path()):
        from paper_2510_09608_amd import build
        build.build(verbose=False)
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    w = si.workload_qwen_stream() if args.workload == "qwen7b_256v_28L" else si.workload_high_fps(n_layers=28)
    L = args.layers
    Hq, Hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    nv, nt = w.vision_per_chunk, w.text_per_chunk
    R = w.retained_steady()
    cap = R + w.tokens_per_chunk + 64
    cache = sv.Cache(L, Hq, Hkv, d, sv.SV_DTYPE_BF16, w.rope_mode, w.rope_theta, w.mrope_sections, 1, cap, nv)
    run = StreamRunner(cache, w.n_sink, w.vision_window, w.text_window)

    g = torch.Generator(device=dev).manual_seed(w.seed)
    rnd = lambda *shape: torch.randn(*shape, device=dev, generator=g).to(torch.bfloat16)
    # pool[p] = inputs of one chunk for all layers: vision q/k/v and the 16 text tokens' q/k/v
    pool = []
    for _ in range(args.pool):
        pool.append(dict(qv=rnd(L, nv, Hq, d), kv=rnd(L, nv, Hkv, d), vv=rnd(L, nv, Hkv, d),
                         qt=rnd(nt, L, 1, Hq, d), kt=rnd(nt, L, 1, Hkv, d), vt=rnd(nt, L, 1, Hkv, d)))
    ov = torch.empty(L, nv, Hq, d, device=dev, dtype=torch.bfloat16)
    ot = torch.empty(L, 1, Hq, d, device=dev, dtype=torch.bfloat16)
    run.preamble(list(rnd(L, w.preamble_text, Hkv, d)), list(rnd(L, w.preamble_text, Hkv, d)))

    ev = lambda: torch.cuda.Event(enable_timing=True)
    roof_events = []            # (start, stop) around every launch of the roofline kernel in the timed region
    roof_units = []             # algorithmic units (flops or bytes) of each of those launches

    def step(c: int, timed: bool):
        p = pool[c % len(pool)]
        n_before = cache.len(0)
        if timed and args.roofline_kernel == "compact":
            e0, e1 = ev(), ev()
            e0.record()
            n_ret = run.evict()
            e1.record()
            if n_ret != n_before:
                roof_events.append((e0, e1))
                roof_units.append(2.0 * n_ret * 2 * Hkv * d * 2 * L)       # read + write of every retained K and V row
        else:
            run.evict()
        qv, kv, vv = p["qv"], p["kv"], p["vv"]
        types_v = np.ones(nv, dtype=np.uint8)
        for l in range(L):
            slot0 = cache.append(0, l, types_v if l == 0 else None, w.grid_thw if l == 0 else None, kv[l], vv[l])
            cache.rope_apply(0, slot0, nv, qv[l], None)
            if timed and args.roofline_kernel == "attn_chunk":
                e0, e1 = ev(), ev()
                e0.record()
                cache.attn_chunk(0, l, qv[l], ov[l], True)
                e1.record()
                roof_events.append((e0, e1))
                roof_units.append(4.0 * d * nv * (slot0 + (nv + 1) / 2.0) * Hq)   # visible (query, key) pairs only
            else:
                cache.attn_chunk(0, l, qv[l], ov[l], True)
        types_t = np.zeros(1, dtype=np.uint8)
        ids = np.zeros(1, dtype=np.int32)
        for t in range(nt):
            qt, kt, vt = p["qt"][t], p["kt"][t], p["vt"][t]
            for l in range(L):
                slot = cache.append(0, l, types_t if l == 0 else None, None, kt[l], vt[l])
                cache.rope_apply(0, slot, 1, qt[l], None)
                if timed and args.roofline_kernel == "attn_decode":
                    e0, e1 = ev(), ev()
                    e0.record()
                    cache.attn_decode(l, ids, qt[l], ot[l])
                    e1.record()
                    roof_events.append((e0, e1))
                    roof_units.append((slot + 1) * 2.0 * Hkv * d * 2)              # K and V rows of every cached token
                else:
                    cache.attn_decode(l, ids, qt[l], ot[l])

    for c in range(args.warmup):
        step(c, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for c in range(args.warmup, args.warmup + args.steps):
        step(c, True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    steady = cache.len(0) == R + w.tokens_per_chunk

    # roofline of the chosen kernel from the events recorded in the timed region
    durs_ms = [a.elapsed_time(b) for a, b in roof_events]
    avg_ms = sum(durs_ms) / max(len(durs_ms), 1)
    units = sum(roof_units) / max(len(roof_units), 1)
    if args.roofline_kernel == "attn_chunk":
        achieved, peak, unit, bound = units / (avg_ms * 1e-3) / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s", "mfma"
    else:
        achieved, peak, unit, bound = units / (avg_ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s", "hbm"
    roofline = {"kernel": args.roofline_kernel, "bound": bound, "achieved": round(achieved, 2), "peak": peak,
                "unit": unit, "frac": round(achieved / peak, 4), "traffic": None,
                "avg_launch_us": round(avg_ms * 1e3, 2), "launches": len(durs_ms),
                "algorithmic_units_per_launch": units}

    # untimed breakdown pass: mean microseconds per call of each class (events around every call)
    breakdown = breakdown_pass(cache, run, pool, w, L, args.warmup + args.steps, ov, ot)

    out = {
        "metric": "ms per 1-s video chunk", "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {L} layers, {Hq}q/{Hkv}kv heads x {d}, M-RoPE (16,24,24); per chunk "
                               f"{nv} vision + {nt} text tokens; budgets sink {w.n_sink} / vision {w.vision_window} / "
                               f"text {w.text_window}; retained {R}", "steady_state": bool(steady)},
        "prefill_attn_tflops": breakdown.get("prefill_attn_tflops"),
        "decode_kv_gbs": breakdown.get("decode_kv_gbs"),
        "compaction_gbs": breakdown.get("compaction_gbs"),
        "breakdown_us_per_call": breakdown.get("us"),
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L)
    print(json.dumps(out))


def breakdown_pass(cache, run, pool, w, L, c0, ov, ot, n_chunks: int = 3):
    import numpy as np
    import torch
    Hq, Hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    nv, nt = w.vision_per_chunk, w.text_per_chunk
    ev = lambda: torch.cuda.Event(enable_timing=True)
    rec = {k: [] for k in ("evict", "append_chunk", "rope_chunk", "attn_chunk", "append_decode", "rope_decode",
                           "attn_decode")}

    def timed(key, fn):
        a, b = ev(), ev()
        a.record()
        r = fn()
        b.record()
        rec[key].append((a, b))
        return r

    slot0_seen, slots_decode, n_ret_seen = [], [], []
    for c in range(c0, c0 + n_chunks):
        p = pool[c % len(pool)]
        n_ret_seen.append(timed("evict", run.evict))
        tv, tt, ids = np.ones(nv, dtype=np.uint8), np.zeros(1, dtype=np.uint8), np.zeros(1, dtype=np.int32)
        for l in range(L):
            slot0 = timed("append_chunk", lambda: cache.append(0, l, tv if l == 0 else None,
                                                               w.grid_thw if l == 0 else None, p["kv"][l], p["vv"][l]))
            timed("rope_chunk", lambda: cache.rope_apply(0, slot0, nv, p["qv"][l], None))
            timed("attn_chunk", lambda: cache.attn_chunk(0, l, p["qv"][l], ov[l], True))
            slot0_seen.append(slot0)
        for t in range(nt):
            for l in range(L):
                slot = timed("append_decode", lambda: cache.append(0, l, tt if l == 0 else None, None,
                                                                   p["kt"][t][l], p["vt"][t][l]))
                timed("rope_decode", lambda: cache.rope_apply(0, slot, 1, p["qt"][t][l], None))
                timed("attn_decode", lambda: cache.attn_decode(l, ids, p["qt"][t][l], ot[l]))
                slots_decode.append(slot)
    torch.cuda.synchronize()
    us = {k: round(1e3 * sum(a.elapsed_time(b) for a, b in v) / max(len(v), 1), 2) for k, v in rec.items()}
    flops = [4.0 * d * nv * (s + (nv + 1) / 2.0) * Hq for s in slot0_seen]
    bytes_dec = [(s + 1) * 2.0 * Hkv * d * 2 for s in slots_decode]
    bytes_cmp = [2.0 * n * 2 * Hkv * d * 2 * L for n in n_ret_seen]
    return {
        "us": us,
        "prefill_attn_tflops": round(sum(flops) / len(flops) / (us["attn_chunk"] * 1e-6) / 1e12, 2),
        "decode_kv_gbs": round(sum(bytes_dec) / len(bytes_dec) / (us["attn_decode"] * 1e-6) / 1e9, 2),
        "compaction_gbs": round(sum(bytes_cmp) / len(bytes_cmp) / (us["evict"] * 1e-6) / 1e9, 2),
    }


def cpu_baseline(L: int):
    """The fp64 oracle, as it stands, on the host cores: one steady-state chunk of ONE layer, scaled by L."""
    import sv_inputs as si
    from oracle import sv_step
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    w = si.workload_qwen_layer(n_chunks=34)
    st = sv_step.new_stream(w, [0])
    sv_step.append_preamble(st, w, [0])
    for c in range(33):
        sv_step.step_chunk(st, w, c, [0], want_outputs=False)
    t0 = time.perf_counter()
    sv_step.step_chunk(st, w, 33, [0], want_outputs=True)
    dt = time.perf_counter() - t0
    return {"value": round(dt * 1e3 * L, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
            "sample": f"one steady-state chunk (evict, 256-token prefill, 16 decode steps) of ONE layer took "
                      f"{dt * 1e3:.0f} ms in the fp64 numpy oracle; value = that x {L} layers (extrapolated)"}


if __name__ == "__main__":
    main()
