"""GPU parity at the exact shapes and launch configurations that bench.py times.

Each case builds the cache the benchmark builds (layer count, capacity, budgets, chunk size), drives it through the
same C entry points (sv_stream_step for the per-second workloads, sv_attn_decode for the decode batches, the
evict-all / re-append / one causal prefill sequence of the sliding-window-with-overlap baseline), and compares with
the fp64 oracle: retained ids and positions bit for bit, attention within 2e-2 (bf16, unit-variance inputs).
Layers that are not compared carry random filler so that the arena, the launch grids and the kernels' strides are
those of the full-size run.
"""
import numpy as np
import pytest
import torch

import paper_2510_09608_amd as sv
import sv_inputs as si
from oracle import sv_oracle as orc
from oracle import sv_step
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
HQ, HKV, D = 28, 4, 128


def _say(msg):
    print(msg, flush=True)


def _bf(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV).to(torch.bfloat16)


def _filler(gen, *shape):
    return torch.randn(*shape, device=DEV, generator=gen).to(torch.bfloat16)


def _stream_step_case(w: si.Workload, checked, n_chunks, compare_chunks, decode_steps_checked):
    """Run `n_chunks` seconds of workload w through sv_stream_step on a 28-layer cache sized as bench.py sizes it;
    layers `checked` carry the seeded data and are compared with the oracle at `compare_chunks`."""
    L, nv, nt = 28, w.vision_per_chunk, w.text_per_chunk
    cap = w.retained_steady() + w.tokens_per_chunk + 64                       # bench.py's capacity
    cache = sv.Cache(L, HQ, HKV, D, sv.SV_DTYPE_BF16, w.rope_mode, w.rope_theta, w.mrope_sections, 1, cap, nv)
    gen = torch.Generator(device=DEV).manual_seed(11)
    o = sv_step.new_stream(w, checked)
    sv_step.append_preamble(o, w, checked)
    # preamble: K/V only
    kp, vp = _filler(gen, L, w.preamble_text, HKV, D), _filler(gen, L, w.preamble_text, HKV, D)
    for l in checked:
        _, k, v = w.qkv(l, np.arange(w.preamble_text))
        kp[l], vp[l] = _bf(k), _bf(v)
    run = gu.StreamRunner(cache, w.n_sink, w.vision_window, w.text_window)
    run.preamble(list(kp), list(vp))
    # filler of the unchecked layers is the same every chunk (its values do not matter), checked layers are overwritten
    qv, kv, vv = _filler(gen, L, nv, HQ, D), _filler(gen, L, nv, HKV, D), _filler(gen, L, nv, HKV, D)
    qt, kt, vt = _filler(gen, nt, L, HQ, D), _filler(gen, nt, L, HKV, D), _filler(gen, nt, L, HKV, D)
    ov, ot = torch.empty_like(qv), torch.empty_like(qt)
    worst = 0.0
    for c in range(n_chunks):
        ch = w.chunk(c)
        gv = np.arange(ch.vision.gid0, ch.vision.gid0 + nv)
        gt = np.arange(ch.text_gid0, ch.text_gid0 + nt)
        for l in checked:
            q, k, v = w.qkv(l, gv)
            qv[l], kv[l], vv[l] = _bf(q), _bf(k), _bf(v)
            q, k, v = w.qkv(l, gt)
            qt[:, l], kt[:, l], vt[:, l] = _bf(q), _bf(k), _bf(v)
        n_ret = cache.stream_step(0, w.n_sink, w.vision_window, w.text_window, q_vision=qv, k_vision=kv, v_vision=vv,
                                  o_vision=ov, grid_thw=w.grid_thw, q_text=qt, k_text=kt, v_text=vt, o_text=ot)
        ro = sv_step.step_chunk(o, w, c, checked, want_outputs=c in compare_chunks)
        assert n_ret == ro["n_retained"], c
        ids, pos = cache.retained(0)
        assert np.array_equal(ids, np.asarray(ro["gids_end"], dtype=np.int64)), c
        assert np.array_equal(pos.astype(np.int64), ro["pos_end"]), c
        if c in compare_chunks:
            gvh, gth = gu.host(ov), gu.host(ot)
            for j, l in enumerate(checked):
                e = gu.max_err(gvh[l], ro["prefill"][j])
                assert e <= gu.TOL["bf16"], (c, l, e)
                worst = max(worst, e)
                for t in decode_steps_checked:
                    e = gu.max_err(gth[t, l], ro["decode"][t][j][0])
                    assert e <= gu.TOL["bf16"], (c, l, t, e)
                    worst = max(worst, e)
            _say(f"  chunk {c}: cache {cache.len(0)} tokens, retained {n_ret}, worst max-abs err so far {worst:.3e}")
    return cache, n_ret


def test_default_workload_28_layers_full_budgets_steady_state():
    """bench.py's default workload: 28 layers, capacity 5456, budgets 512/4096/512, 256 + 16 tokens per second,
    through sv_stream_step into steady state; layers 0, 13, 27 against the oracle at chunks 33 and 34 (every
    prefill row, every decode step), ids and positions at every chunk."""
    w = gu.pooled(si.workload_qwen_stream(n_chunks=35), 8)
    _say("default workload, 28 layers, full budgets")
    cache, n_ret = _stream_step_case(w, [0, 13, 27], 35, {33, 34}, range(16))
    assert n_ret == 5120 and cache.len(0) == 5120 + 272


def test_high_frame_rate_28_layers_all_rows_of_a_steady_chunk():
    """bench.py's 1024-token workload: 28-layer cache (arena above 2 GiB), fused token store (K rows, V^T blocks; Q
    rotated by the attention kernel while loading) with n = 1024, all 1024 query rows of a steady-state chunk (both windows full: chunk 33) on layers 0 and 27, plus the first and
    last decode step."""
    w = gu.pooled(si.workload_high_fps(n_chunks=34, n_layers=28), 4)
    _say("high-frame-rate workload, 28 layers")
    cache, n_ret = _stream_step_case(w, [0, 27], 34, {33}, (0, 15))
    assert cache.arena.numel() > (2 << 30)
    assert n_ret == 512 + 512 + 16384 and cache.len(0) == n_ret + 1040


def _text_stream_kv(n, pool, shift):
    """K/V of an n-token text-only stream: a pool of seeded rows, cycled, rotated by `shift` rows."""
    idx = (np.arange(n) + shift) % pool[0].shape[0]
    return pool[0][idx], pool[1][idx]


def test_decode_batch_16_streams_of_32768_tokens():
    """The no-eviction baseline of the decode batch: sv_attn_decode on 16 caches of 32768 tokens each (1.07 GB of K
    and V per launch: non-temporal loads, 16 tiles per wavefront, 16 key ranges per row)."""
    n, S, theta, sec = 32768, 16, 1.0e6, (16, 24, 24)
    _say(f"decode batch {S} x {n}")
    gids = np.arange(n)
    pool = (si.normal(1005, si.TENSOR_K, 0, gids, HKV, D, True), si.normal(1005, si.TENSOR_V, 0, gids, HKV, D, True))
    cache = sv.Cache(1, HQ, HKV, D, sv.SV_DTYPE_BF16, sv.SV_ROPE_3D, theta, sec, S, n + 8, 16)
    ty = np.zeros(n, dtype=np.uint8)
    q = si.normal(1005, si.TENSOR_Q, 0, np.arange(S), HQ, D, True)
    for s_ in range(S):
        k, v = _text_stream_kv(n, pool, 2048 * s_ + 7 * s_)
        cache.append(s_, 0, ty, None, _bf(k), _bf(v))
    qd = _bf(q)
    for s_ in range(S):
        cache.rope_apply(s_, n - 1, 1, qd[s_:s_ + 1], None)
    od = torch.empty_like(qd)
    cache.attn_decode(0, list(range(S)), qd, od)
    got = gu.host(od)
    pos = np.arange(n)[:, None].repeat(3, 1)
    worst = 0.0
    for s_ in range(S):
        k, v = _text_stream_kv(n, pool, 2048 * s_ + 7 * s_)
        kr = orc.rope(k, pos, orc.ROPE_3D, theta, sec)
        qr = orc.rope(q[s_:s_ + 1], pos[n - 1:], orc.ROPE_3D, theta, sec)
        ref = orc.gqa_attention(qr, kr, v.astype(np.float64), np.array([n - 1]), True)
        e = gu.max_err(got[s_:s_ + 1], ref)
        assert e <= gu.TOL["bf16"], (s_, e)
        worst = max(worst, e)
    _say(f"  worst max-abs err {worst:.3e}")


def test_decode_single_stream_131072_tokens():
    """One stream grown to 131072 tokens without eviction (the end point of bench.py's no-eviction growth curve):
    plain decode of the last token and one fused decode step."""
    n, theta, sec = 131072, 1.0e6, (16, 24, 24)
    _say(f"single stream decode at {n} tokens")
    gids = np.arange(32768)
    pool = (si.normal(1006, si.TENSOR_K, 0, gids, HKV, D, True), si.normal(1006, si.TENSOR_V, 0, gids, HKV, D, True))
    k, v = _text_stream_kv(n, pool, 0)
    cache = sv.Cache(1, HQ, HKV, D, sv.SV_DTYPE_BF16, sv.SV_ROPE_3D, theta, sec, 1, n + 8, 16)
    for g0 in range(0, n, 32768):
        cache.append(0, 0, np.zeros(32768, dtype=np.uint8), None, _bf(k[g0:g0 + 32768]), _bf(v[g0:g0 + 32768]))
    q = si.normal(1006, si.TENSOR_Q, 0, np.array([n - 1, n]), HQ, D, True)
    qd = _bf(q[:1])
    cache.rope_apply(0, n - 1, 1, qd, None)
    od = torch.empty_like(qd)
    cache.attn_decode(0, [0], qd, od)
    pos = np.arange(n + 1)[:, None].repeat(3, 1)
    kr = orc.rope(k, pos[:n], orc.ROPE_3D, theta, sec)
    ref = orc.gqa_attention(orc.rope(q[:1], pos[n - 1:n], orc.ROPE_3D, theta, sec), kr, v.astype(np.float64),
                            np.array([n - 1]), True)
    e = gu.max_err(gu.host(od), ref)
    assert e <= gu.TOL["bf16"], e
    # one more token through the fused step
    k2 = si.normal(1006, si.TENSOR_K, 0, np.array([n]), HKV, D, True)
    v2 = si.normal(1006, si.TENSOR_V, 0, np.array([n]), HKV, D, True)
    od2 = torch.empty_like(qd)
    cache.decode_step(0, [0], _bf(q[1:]), _bf(k2), _bf(v2), od2)
    kr2 = np.concatenate([kr, orc.rope(k2, pos[n:], orc.ROPE_3D, theta, sec)])
    ref2 = orc.gqa_attention(orc.rope(q[1:], pos[n:], orc.ROPE_3D, theta, sec), kr2,
                             np.concatenate([v, v2]).astype(np.float64), np.array([n]), True)
    e2 = gu.max_err(gu.host(od2), ref2)
    assert e2 <= gu.TOL["bf16"], e2
    _say(f"  max-abs err {e:.3e} (decode), {e2:.3e} (fused step)")


def test_overlap_recompute_pattern_whole_window_prefill():
    """The sliding-window-with-overlap baseline as bench.py runs it: drop everything (evict with all budgets 0),
    re-append the whole window (1024 text tokens, then 17 s of vision as one block), rotate Q and run ONE causal
    prefill with n_q = n_kv = 5376; query rows sampled from every 256-row tile of the launch, then a decode step."""
    w = si.workload_qwen_layer(n_chunks=0)
    W = w.retained_steady() + w.vision_per_chunk          # 5376
    n_text0, n_vis0 = w.n_sink + w.text_window, W - (w.n_sink + w.text_window)
    grid = (n_vis0 // w.vision_per_chunk, w.grid_thw[1], w.grid_thw[2])
    _say(f"overlap recompute: window {W}")
    cache = sv.Cache(1, HQ, HKV, D, sv.SV_DTYPE_BF16, w.rope_mode, w.rope_theta, w.mrope_sections, 1, W + 16 + 64, W)
    o = orc.OracleStream(1, HQ, HKV, D, orc.ROPE_3D, w.rope_theta, w.mrope_sections)
    ids = np.zeros(1, dtype=np.int32)
    for second in range(2):                               # the second pass evicts a full cache first
        assert cache.evict(0, 0, 0, 0) == 0 and o.evict(0, 0, 0) == 0
        g0 = 100_000 * second
        gt, gv = np.arange(g0, g0 + n_text0), np.arange(g0 + n_text0, g0 + W)
        qt_, kt_, vt_ = w.qkv(0, gt)
        qv_, kv_, vv_ = w.qkv(0, gv)
        cache.append(0, 0, np.zeros(n_text0, np.uint8), None, _bf(kt_), _bf(vt_))
        cache.append(0, 0, np.ones(n_vis0, np.uint8), grid, _bf(kv_), _bf(vv_))
        o.append_meta([orc.TEXT] * n_text0)
        o.append_kv(0, kt_, vt_)
        o.append_meta([orc.VISION] * n_vis0, grid)
        o.append_kv(0, kv_, vv_)
        q = np.concatenate([qt_, qv_])
        qd = _bf(q)
        cache.rope_apply(0, 0, W, qd, None)
        od = torch.empty_like(qd)
        cache.attn_chunk(0, 0, qd, od, True)
        ids_g, pos_g = cache.retained(0)
        assert np.array_equal(ids_g, np.asarray(o.gid, dtype=np.int64))
        assert np.array_equal(pos_g.astype(np.int64), o.positions())
        # a 256-row tile of the launch holds rows query * 7 + head of 36.6 queries: every 17th query, both ends
        rows = np.unique(np.concatenate([np.arange(0, W, 17), [1, 36, 37, W - 2, W - 1]]))
        ref = o.attend(0, q[rows], list(rows))
        e = gu.max_err(gu.host(od)[rows], ref)
        assert e <= gu.TOL["bf16"], (second, e)
        gd = np.array([g0 + W])
        qd1, kd1, vd1 = w.qkv(0, gd)
        od1 = torch.empty(1, HQ, D, device=DEV, dtype=torch.bfloat16)
        cache.decode_step(0, ids, _bf(qd1), _bf(kd1), _bf(vd1), od1)
        o.append_meta([orc.TEXT])
        o.append_kv(0, kd1, vd1)
        e1 = gu.max_err(gu.host(od1), o.attend(0, qd1, [W]))
        assert e1 <= gu.TOL["bf16"], (second, e1)
        _say(f"  pass {second}: {len(rows)} sampled rows, max-abs err {e:.3e}; decode step {e1:.3e}")


def test_device_count_is_cross_checked():
    """sv_cache_retained compares the device's own token count with the host's bookkeeping: they agree through
    appends, decode steps and evictions, and a corrupted device count is reported as SV_ERR_STATE."""
    w = si.workload_tiny()
    cache = gu.make_cache(w, capacity=128)
    z = lambda n: torch.zeros(n, 1, 64, device=DEV)
    cache.append(0, 0, np.zeros(20, dtype=np.uint8), None, z(20), z(20))
    assert cache.retained(0)[0].size == 20
    cache.decode_step(0, [0], torch.zeros(1, 2, 64, device=DEV), z(1), z(1), torch.zeros(1, 2, 64, device=DEV))
    assert cache.retained(0)[0].size == 21
    assert cache.evict(0, 2, 0, 3) == 5 and cache.retained(0)[0].size == 5
    # everything behind the K/V store is metadata and scratch: overwrite it, as a stray write would
    kv_bytes = 2 * 1 * 2 * 1 * 128 * 64 * 4
    torch.cuda.synchronize()
    cache.arena[kv_bytes:].fill_(0xFF)
    torch.cuda.synchronize()
    with pytest.raises(sv.SvError) as e:
        cache.retained(0)
    assert e.value.status == -3
