"""GPU parity: the HIP library against the fp64 oracle on the same seeded inputs.

Integer state (retained arrival ids, positions) must match bit for bit; attention
outputs within max-abs 1e-5 (fp32 workload) and 2e-2 (bf16 workloads, unit-variance
inputs, oracle fed the bf16-rounded values).  Everything goes through the C ABI.
"""
import copy

import numpy as np
import pytest
import torch

import paper_2510_09608_amd as sv
import sv_inputs as si
from oracle import sv_oracle as orc
from oracle import sv_step
from tests import golden_io as gio
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


# ----------------------------------------------------------------------------
# whole per-chunk step
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("fused", [True, False])
def test_tiny_stream_f32_every_chunk(fused):
    w = si.workload_tiny()
    g, o = gu.GpuStream(w, [0], fused_decode=fused), sv_step.new_stream(w, [0])
    worst = 0.0
    for c in range(w.n_chunks):
        _say(f"tiny_f32 chunk {c}")
        rg, ro = g.step_chunk(c), sv_step.step_chunk(o, w, c, [0])
        gu.assert_int_parity(rg, ro, f"chunk {c}")
        worst = max(worst, gu.assert_attn_parity(rg, ro, gu.TOL["f32"], f"chunk {c}"))
    _say(f"tiny_f32 worst max-abs err {worst:.3e}")


@pytest.mark.parametrize("fused", [True, False])
def test_qwen_layer_bf16_stream(fused):
    """One Qwen-7B-shaped layer through warm-up into steady state (retained = 5120)."""
    w = si.workload_qwen_layer(n_chunks=35)
    g, o = gu.GpuStream(w, [0], fused_decode=fused), sv_step.new_stream(w, [0])
    g.preamble()
    sv_step.append_preamble(o, w, [0])
    check = {0, 1, 31, 32, 33, 34}
    worst = 0.0
    for c in range(w.n_chunks):
        _say(f"qwen_layer chunk {c}")
        rg = g.step_chunk(c)
        ro = sv_step.step_chunk(o, w, c, [0], want_outputs=c in check)
        gu.assert_int_parity(rg, ro, f"chunk {c}")
        if c in check:
            worst = max(worst, gu.assert_attn_parity(rg, ro, gu.TOL["bf16"], f"chunk {c}"))
    assert rg["n_retained"] == 5120 and int(np.max(rg["pos_end"])) == 1311
    _say(f"qwen_layer worst max-abs err {worst:.3e}")


def test_multi_layer_step_sampled_layers():
    """28-layer step: layers 0, 13, 27 carry seeded data and are checked, the rest carry filler."""
    w = si.workload_qwen_layer(n_chunks=4, n_layers=28, seed=1003)
    w.preamble_text, w.vision_window, w.text_window, w.n_sink = 64, 512, 40, 32
    checked = [0, 13, 27]
    cache = gu.make_cache(w, n_layers=28, capacity=2048)
    run = gu.StreamRunner(cache, w.n_sink, w.vision_window, w.text_window)
    o = sv_step.new_stream(w, checked)
    sv_step.append_preamble(o, w, checked)
    gen = torch.Generator(device="cuda:0").manual_seed(5)

    def tensors(gids, heads, which):
        out = []
        for l in range(28):
            if l in checked:
                out.append(gu.dev(si.normal(w.seed, which, l, gids, heads, w.head_dim, True), w))
            else:
                out.append(torch.randn(len(gids), heads, w.head_dim, device="cuda:0", generator=gen).to(torch.bfloat16))
        return out

    gids = np.arange(w.preamble_text)
    run.preamble(tensors(gids, 4, si.TENSOR_K), tensors(gids, 4, si.TENSOR_V))
    for c in range(w.n_chunks):
        _say(f"multi_layer chunk {c}")
        ro = sv_step.step_chunk(o, w, c, checked)
        n_ret = run.evict()
        assert n_ret == ro["n_retained"]
        ids, pos = cache.retained(0)
        assert np.array_equal(ids, np.asarray(ro["gids_after_evict"])) and np.array_equal(pos, ro["pos_after_evict"])
        ch = w.chunk(c)
        gids = np.arange(ch.vision.gid0, ch.vision.gid0 + ch.vision.n)
        qs, ks, vs = tensors(gids, 28, si.TENSOR_Q), tensors(gids, 4, si.TENSOR_K), tensors(gids, 4, si.TENSOR_V)
        os_ = [torch.empty_like(q) for q in qs]
        run.prefill(qs, ks, vs, os_, ch.vision.grid_thw)
        for j, l in enumerate(checked):
            e = gu.max_err(gu.host(os_[l]), ro["prefill"][j])
            assert e <= gu.TOL["bf16"], (c, l, e)
        for t in range(ch.n_text):
            gid = np.array([ch.text_gid0 + t])
            qs, ks, vs = tensors(gid, 28, si.TENSOR_Q), tensors(gid, 4, si.TENSOR_K), tensors(gid, 4, si.TENSOR_V)
            os_ = [torch.empty_like(q) for q in qs]
            run.decode(qs, ks, vs, os_)
            for j, l in enumerate(checked):
                e = gu.max_err(gu.host(os_[l]), ro["decode"][t][j])
                assert e <= gu.TOL["bf16"], (c, t, l, e)
        ids, pos = cache.retained(0)
        assert np.array_equal(ids, np.asarray(ro["gids_end"])) and np.array_equal(pos, ro["pos_end"])


@pytest.mark.parametrize("layers_batched", [False, True])
def test_native_stream_step_matches_oracle(layers_batched):
    """sv_stream_step (the whole second sequenced in C, all layers) on a 3-layer cache, every output checked;
    decode steps as one launch per layer, or as one launch for all layers (sv_decode_step_layers)."""
    w = si.workload_qwen_layer(n_chunks=5, n_layers=3, seed=1003)
    w.preamble_text, w.vision_window, w.text_window, w.n_sink = 48, 512, 40, 32
    layers = [0, 1, 2]
    cache = gu.make_cache(w, n_layers=3, capacity=2048)
    o = sv_step.new_stream(w, layers)
    sv_step.append_preamble(o, w, layers)
    gids = np.arange(w.preamble_text)
    run = gu.StreamRunner(cache, w.n_sink, w.vision_window, w.text_window)
    run.preamble([gu.dev(si.normal(w.seed, si.TENSOR_K, l, gids, 4, 128, True), w) for l in layers],
                 [gu.dev(si.normal(w.seed, si.TENSOR_V, l, gids, 4, 128, True), w) for l in layers])
    stack = lambda which, g, heads: torch.stack([gu.dev(si.normal(w.seed, which, l, g, heads, 128, True), w)
                                                 for l in layers])
    for c in range(w.n_chunks):
        _say(f"native_step chunk {c}")
        ro = sv_step.step_chunk(o, w, c, layers)
        ch = w.chunk(c)
        gv = np.arange(ch.vision.gid0, ch.vision.gid0 + ch.vision.n)
        gt = np.arange(ch.text_gid0, ch.text_gid0 + ch.n_text)
        qv, kv, vv = stack(si.TENSOR_Q, gv, 28), stack(si.TENSOR_K, gv, 4), stack(si.TENSOR_V, gv, 4)
        # text tensors are [n_text][L][H][d]
        qt = stack(si.TENSOR_Q, gt, 28).transpose(0, 1).contiguous()
        kt = stack(si.TENSOR_K, gt, 4).transpose(0, 1).contiguous()
        vt = stack(si.TENSOR_V, gt, 4).transpose(0, 1).contiguous()
        ov, ot = torch.empty_like(qv), torch.empty_like(qt)
        n_ret = cache.stream_step(0, w.n_sink, w.vision_window, w.text_window, q_vision=qv, k_vision=kv, v_vision=vv,
                                  o_vision=ov, grid_thw=ch.vision.grid_thw, q_text=qt, k_text=kt, v_text=vt, o_text=ot,
                                  decode_layers_batched=layers_batched)
        assert n_ret == ro["n_retained"]
        for j in range(3):
            assert gu.max_err(gu.host(ov[j]), ro["prefill"][j]) <= gu.TOL["bf16"]
            for t in range(ch.n_text):
                assert gu.max_err(gu.host(ot[t, j]), ro["decode"][t][j][0]) <= gu.TOL["bf16"]
        ids, pos = cache.retained(0)
        assert np.array_equal(ids, np.asarray(ro["gids_end"])) and np.array_equal(pos, ro["pos_end"])


@pytest.mark.parametrize("preamble,grid,n_text,splits,budgets,store,sid", [
    (48, (1, 16, 16), 4, 0, (32, 600, 40), 2, 0),     # whole blocks and tiles
    (51, (1, 7, 5), 3, 0, (9, 100, 11), 2, 0),        # 35-token chunks, the first new key in the middle of a V^T block
    (13, (1, 1, 1), 1, 0, (2, 5, 3), 2, 0),           # one-token chunks
    (77, (1, 17, 16), 5, 3, (50, 1000, 21), 2, 0),    # 272 tokens, three forced key ranges: the new keys straddle two
    (77, (1, 17, 16), 5, 1, (50, 1000, 21), 2, 0),    # ... and no split at all
    (100, (2, 16, 16), 2, 0, (64, 1100, 30), 2, 0),   # 512 tokens: the longest chunk the attention launch can store
    (100, (1, 19, 27), 2, 0, (64, 1100, 30), 2, 0),   # 513: stored by the launch of their own whatever the option says
    (77, (1, 17, 16), 5, 0, (50, 1000, 21), 1, 0),    # the store launch forced
    (77, (1, 17, 16), 5, 0, (50, 1000, 21), 0, 0),    # the library's own choice, which changes as the cache grows
    (51, (1, 7, 5), 3, 0, (9, 100, 11), 2, 1),     # the second stream of a cache (its own cos/sin table and K/V planes)
])
def test_stream_step_chunk_stored_by_attention_launch(preamble, grid, n_text, splits, budgets, store, sid):
    """sv_stream_step on a blocked-V^T cache: a short chunk's K/V can reach the cache inside the attention launch
    (SV_OPT_CHUNK_STORE: forced here, chosen by the balance of the key ranges otherwise).  After every second the
    stored V rows are the appended ones bit for bit, the stored K rows the rotated ones to a bf16 rounding per
    compaction, and every prefill and decode output matches the oracle; chunk sizes, preambles and budgets chosen so
    that the first new key falls inside a block and a tile, the last one too, and key ranges cut the chunk."""
    n_sink, vw, tw = budgets
    nv = grid[0] * grid[1] * grid[2]
    w = si.Workload("t", 2, 28, 4, 128, "bf16", 1, 1.0e6, (16, 24, 24), n_sink, vw, tw, preamble, nv, n_text, grid, 6,
                    4242 + preamble + nv)
    layers = [0, 1]
    cache = gu.make_cache(w, n_layers=2, capacity=w.capacity() + 64, n_streams=sid + 1)
    if splits:
        cache.set_option(sv.SV_OPT_CHUNK_SPLITS, splits)
    cache.set_option(sv.SV_OPT_CHUNK_STORE, store)
    o = sv_step.new_stream(w, layers)
    sv_step.append_preamble(o, w, layers)
    gids = np.arange(w.preamble_text)
    run = gu.StreamRunner(cache, w.n_sink, w.vision_window, w.text_window, stream_id=sid)
    run.preamble([gu.dev(si.normal(w.seed, si.TENSOR_K, l, gids, 4, 128, True), w) for l in layers],
                 [gu.dev(si.normal(w.seed, si.TENSOR_V, l, gids, 4, 128, True), w) for l in layers])
    stack = lambda which, g, heads: torch.stack([gu.dev(si.normal(w.seed, which, l, g, heads, 128, True), w)
                                                 for l in layers])
    for c in range(w.n_chunks):
        _say(f"chunk stored by attention launch: preamble {preamble} grid {grid} splits {splits} store {store} chunk {c}")
        ro = sv_step.step_chunk(o, w, c, layers)
        ch = w.chunk(c)
        gv = np.arange(ch.vision.gid0, ch.vision.gid0 + ch.vision.n)
        gt = np.arange(ch.text_gid0, ch.text_gid0 + ch.n_text)
        qv, kv, vv = stack(si.TENSOR_Q, gv, 28), stack(si.TENSOR_K, gv, 4), stack(si.TENSOR_V, gv, 4)
        qt = stack(si.TENSOR_Q, gt, 28).transpose(0, 1).contiguous()
        kt = stack(si.TENSOR_K, gt, 4).transpose(0, 1).contiguous()
        vt = stack(si.TENSOR_V, gt, 4).transpose(0, 1).contiguous()
        ov, ot = torch.empty_like(qv), torch.empty_like(qt)
        n_ret = cache.stream_step(sid, w.n_sink, w.vision_window, w.text_window, q_vision=qv, k_vision=kv, v_vision=vv,
                                  o_vision=ov, grid_thw=ch.vision.grid_thw, q_text=qt, k_text=kt, v_text=vt, o_text=ot)
        assert n_ret == ro["n_retained"]
        n = len(o)
        pos = o.positions()
        for j in range(2):
            assert gu.max_err(gu.host(ov[j]), ro["prefill"][j]) <= gu.TOL["bf16"], (c, j)
            for t in range(ch.n_text):
                assert gu.max_err(gu.host(ot[t, j]), ro["decode"][t][j][0]) <= gu.TOL["bf16"], (c, j, t)
            K, V = np.stack(o.k[j]), np.stack(o.v[j])
            assert np.array_equal(cache.read_kv(sid, j, 1, 0, n).astype(np.float64), V), (c, j)
            e = gu.max_err(cache.read_kv(sid, j, 0, 0, n), orc.rope(K, pos, w.rope_mode, w.rope_theta, w.mrope_sections))
            assert e <= 4e-2 * (1 + c), (c, j, e)
        ids, p2 = cache.retained(sid)
        assert np.array_equal(ids, np.asarray(ro["gids_end"])) and np.array_equal(p2, ro["pos_end"])


# ----------------------------------------------------------------------------
# integer state
# ----------------------------------------------------------------------------

def test_mrope_golden_positions_on_gpu():
    g = gio.read_keyed("mrope_positions.txt")
    cache = sv.Cache(1, 1, 1, 64, sv.SV_DTYPE_F32, sv.SV_ROPE_3D, 1e4, (8, 12, 12), 1, 64, 16)
    for op in g["append"]:
        n = int(op[1])
        ty = np.full(n, sv.SV_TEXT if op[0] == "text" else sv.SV_VISION, dtype=np.uint8)
        grid = [int(x) for x in op[2:5]] if len(op) >= 5 else None
        z = torch.zeros(n, 1, 64, device="cuda:0")
        cache.append(0, 0, ty, grid, z, z)
    ids, pos = cache.retained(0)
    assert [tuple(r) for r in pos.tolist()] == gio.triples(g["pos_before"][0])
    ns, vw, tw = (int(x) for x in g["evict"][0])
    assert cache.evict(0, ns, vw, tw) == len(g["retained_gids"][0])
    ids, pos = cache.retained(0)
    assert ids.tolist() == [int(x) for x in g["retained_gids"][0]]
    assert [tuple(r) for r in pos.tolist()] == gio.triples(g["pos_after"][0])
    # the next token continues from the re-walked scalar position
    z = torch.zeros(1, 1, 64, device="cuda:0")
    cache.append(0, 0, np.zeros(1, dtype=np.uint8), None, z, z)
    _, pos = cache.retained(0)
    assert pos[-1].tolist() == [int(g["next_after"][0][0])] * 3


def test_fig3_budgets_golden_on_gpu():
    g = gio.read_keyed("evict_fig3_budgets.txt")
    ns, vw, tw = (int(x) for x in g["budgets"][0])
    cache = sv.Cache(1, 1, 1, 64, sv.SV_DTYPE_F32, sv.SV_ROPE_1D, 1e4, (0, 0, 0), 1, 64, 16)
    z = torch.zeros(2, 1, 64, device="cuda:0")
    for _ in range(int(g["pairs"][0][0])):
        cache.append(0, 0, np.array([sv.SV_VISION, sv.SV_TEXT], dtype=np.uint8), None, z, z)   # mixed-type append
    cache.evict(0, ns, vw, tw)
    ids, pos = cache.retained(0)
    assert ids.tolist() == [int(x) for x in g["retained"][0]]
    assert pos[:, 0].tolist() == [int(x) for x in g["positions"][0]]


def test_long_stream_integer_state():
    """One-hour stream (3600 chunks): integer state at sampled chunks equals a one-shot oracle eviction."""
    w = si.workload_qwen_stream()
    cache = sv.Cache(1, 1, 1, 64, sv.SV_DTYPE_F32, sv.SV_ROPE_3D, 1e6, (8, 12, 12), 1, w.capacity() + 64, 256)
    zv = torch.zeros(256, 1, 64, device="cuda:0")
    zt = torch.zeros(512, 1, 64, device="cuda:0")
    tv, tt, t1 = np.ones(256, dtype=np.uint8), np.zeros(512, dtype=np.uint8), np.zeros(1, dtype=np.uint8)
    one = orc.OracleStream(1, 1, 1, 2, orc.ROPE_3D, 1e6, (1, 0, 0))   # never evicted until asked
    z = lambda n: np.zeros((n, 1, 2))
    cache.append(0, 0, tt, None, zt, zt)
    one.append_meta([orc.TEXT] * 512)
    one.append_kv(0, z(512), z(512))
    samples = {0, 1, 31, 32, 33, 64, 1800, 3599}
    for c in range(w.n_chunks):
        n_ret = cache.evict(0, w.n_sink, w.vision_window, w.text_window)
        if c in samples:
            _say(f"long_stream chunk {c}")
            shot = copy.deepcopy(one)
            assert shot.evict(w.n_sink, w.vision_window, w.text_window) == n_ret
            ids, pos = cache.retained(0)
            assert np.array_equal(ids, np.asarray(shot.gid, dtype=np.int64))
            assert np.array_equal(pos.astype(np.int64), shot.positions())
        if c % 40 == 0:
            # keep the never-evicted oracle list short: drop only what no later evict could keep
            one.evict(w.n_sink, 2 * w.vision_window, 2 * w.text_window)
        cache.append(0, 0, tv, (1, 16, 16), zv, zv)
        for _ in range(16):
            cache.append(0, 0, t1, None, zt[:1], zt[:1])
        one.append_meta([orc.VISION] * 256, (1, 16, 16))
        one.append_kv(0, z(256), z(256))
        one.append_meta([orc.TEXT] * 16)
        one.append_kv(0, z(16), z(16))
        if c >= 32 and c % 400 == 0:
            _, pos = cache.retained(0)
            assert int(pos.max()) == 1311 and cache.len(0) == 5120 + 272     # positions stay bounded
    assert cache.len(0) == 5392


def test_long_cache_eviction_many_scan_workgroups():
    """Eviction of caches long enough for the scan's workgroup limit (128 workgroups of 256 tokens, then several
    passes per workgroup): 40000 and 70000 tokens of mixed vision blocks and text, windows that cut a block, four
    evictions in a row each (the scan's launch tag moves on in device memory, the workgroup count shrinks).  Retained
    ids and positions bit-exact against the oracle."""
    zt = torch.zeros(4096, 1, 64, device="cuda:0")
    z = lambda n: np.zeros((n, 1, 2))
    for total in [40000, 70000]:
        _say(f"long-cache eviction: {total} tokens")
        cache = sv.Cache(1, 1, 1, 64, sv.SV_DTYPE_F32, sv.SV_ROPE_3D, 1e4, (8, 12, 12), 1, total + 4096, 4096)
        o = orc.OracleStream(1, 1, 1, 2, orc.ROPE_3D, 1e4, (1, 0, 0))
        n = 0
        while n < total:
            for ty, cnt, grid in ((orc.VISION, 2 * 12 * 16, (2, 12, 16)), (orc.TEXT, 37, None)):
                cache.append(0, 0, np.full(cnt, 1 if ty == orc.VISION else 0, dtype=np.uint8), grid, zt[:cnt], zt[:cnt])
                o.append_meta([ty] * cnt, grid)
                o.append_kv(0, z(cnt), z(cnt))
                n += cnt
        for budgets in [(100, total // 3 + 77, total // 20), (64, 5000, 333), (64, 5000, 333), (0, 100, 0)]:
            assert cache.evict(0, *budgets) == o.evict(*budgets)
            ids, pos = cache.retained(0)
            assert np.array_equal(ids, np.asarray(o.gid, dtype=np.int64))
            assert np.array_equal(pos.astype(np.int64), o.positions())
        cache.close()


def test_randomized_streams_integer_state():
    """Seeded sweep: streams of random vision grids (1..3 x 1..12 x 1..16) and text runs, random budgets (0, infinite,
    windows that cut blocks in the middle), evictions skipped now and then, 1-D and 3-D positions: retained ids and
    positions after every eviction equal the oracle's, bit for bit."""
    rng = np.random.default_rng(2510_09608)
    z = lambda n: np.zeros((n, 1, 2))
    zt = torch.zeros(640, 1, 64, device="cuda:0")
    for case in range(100):
        mode3d = bool(rng.integers(0, 2))
        n_sink = int(rng.choice([0, 1, 5, 64]))
        vw = int(rng.choice([-1, 0, 7, 100, 300, 1000]))
        tw = int(rng.choice([-1, 0, 3, 40, 200]))
        n_chunks = int(rng.integers(3, 25))
        ncmp = 3 if mode3d else 1
        _say(f"randomized stream {case}: 3d={mode3d} budgets=({n_sink},{vw},{tw}) chunks={n_chunks}")
        cache = sv.Cache(1, 1, 1, 64, sv.SV_DTYPE_F32, sv.SV_ROPE_3D if mode3d else sv.SV_ROPE_1D, 1e4,
                         (8, 12, 12) if mode3d else (0, 0, 0), 1, 64 + n_chunks * 700, 640)
        o = orc.OracleStream(1, 1, 1, 2, orc.ROPE_3D if mode3d else orc.ROPE_1D, 1e4, (1, 0, 0))

        def check():
            assert cache.evict(0, n_sink, vw, tw) == o.evict(n_sink, vw, tw)
            ids, pos = cache.retained(0)
            assert np.array_equal(ids, np.asarray(o.gid, dtype=np.int64))
            assert np.array_equal(pos.astype(np.int64)[:, :ncmp], o.positions()[:, :ncmp])

        pre = int(rng.choice([0, 3, 50]))
        if pre:
            cache.append(0, 0, np.zeros(pre, dtype=np.uint8), None, zt[:pre], zt[:pre])
            o.append_meta([orc.TEXT] * pre)
            o.append_kv(0, z(pre), z(pre))
        for _ in range(n_chunks):
            if rng.integers(0, 4) != 0:
                check()
            T, H, W = int(rng.integers(1, 4)), int(rng.integers(1, 13)), int(rng.integers(1, 17))
            nv = T * H * W
            if rng.integers(0, 5) != 0:
                cache.append(0, 0, np.ones(nv, dtype=np.uint8), (T, H, W), zt[:nv], zt[:nv])
                o.append_meta([orc.VISION] * nv, (T, H, W))
                o.append_kv(0, z(nv), z(nv))
            nt = int(rng.integers(0, 20))
            if nt:
                cache.append(0, 0, np.zeros(nt, dtype=np.uint8), None, zt[:nt], zt[:nt])
                o.append_meta([orc.TEXT] * nt)
                o.append_kv(0, z(nt), z(nt))
        check()


def test_randomized_streams_stored_kv():
    """Seeded sweep, two layers, fp32 (d 64) and bf16 (d 128), 1-D and 3-D positions, random grids / text runs /
    budgets: after every step V as stored is the appended V bit for bit and K as stored is the raw K rotated at the
    token's CURRENT position (appended rotated, re-rotated by every compaction that moved it: one rounding each)."""
    rng = np.random.default_rng(96082510)
    worst = {"f32": 0.0, "bf16": 0.0}
    for case in range(40):
        dtype = "f32" if rng.integers(0, 2) else "bf16"
        mode = int(rng.integers(0, 2))
        d, Hq, Hkv = (64, 2, 1) if dtype == "f32" else (128, 28, 4)
        sec = (0, 0, 0) if mode == 0 else ((8, 12, 12) if d == 64 else (16, 24, 24))
        theta = 1e4 if dtype == "f32" else 1e6
        n_sink, vw, tw = int(rng.choice([0, 2, 9])), int(rng.choice([0, 17, 90, 200])), int(rng.choice([0, 4, 30]))
        w = si.Workload("t", 2, Hq, Hkv, d, dtype, mode, theta, sec, n_sink, vw, tw, 0, 0, 0, None, 0, 100 + case)
        cache = gu.make_cache(w, capacity=4096)
        o = orc.OracleStream(2, Hq, Hkv, d, mode, theta, sec)
        _say(f"randomized stored K/V {case}: {dtype} mode={mode} budgets=({n_sink},{vw},{tw})")
        g0 = 0
        for c in range(int(rng.integers(3, 9))):
            spans = []
            if rng.integers(0, 4):
                T, H, W = int(rng.integers(1, 3)), int(rng.integers(1, 7)), int(rng.integers(1, 9))
                spans.append((orc.VISION, T * H * W, (T, H, W)))
            nt = int(rng.integers(0, 12))
            if nt:
                spans.append((orc.TEXT, nt, None))
            for ty, n, grid in spans:
                gids = np.arange(g0, g0 + n)
                g0 += n
                o.append_meta([ty] * n, grid)
                for l in range(2):
                    _, k, v = w.qkv(l, gids)
                    cache.append(0, l, np.full(n, ty, dtype=np.uint8) if l == 0 else None, grid if l == 0 else None,
                                 gu.dev(k, w), gu.dev(v, w))
                    o.append_kv(l, k, v)
            if rng.integers(0, 3):
                assert cache.evict(0, n_sink, vw, tw) == o.evict(n_sink, vw, tw)
            n = len(o)
            if n == 0:
                continue
            pos = o.positions()
            tol = (1e-5 if dtype == "f32" else 4e-2) * (1 + c)      # one rounding per compaction so far
            for l in range(2):
                K, V = np.stack(o.k[l]), np.stack(o.v[l])
                assert np.array_equal(cache.read_kv(0, l, 1, 0, n).astype(np.float64), V), (case, c, l)
                e = gu.max_err(cache.read_kv(0, l, 0, 0, n), orc.rope(K, pos, mode, theta, sec))
                worst[dtype] = max(worst[dtype], e)
                assert e <= tol, (case, c, l, e)
    _say(f"stored K worst error {worst}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_opening_text_run_left_in_place(dtype):
    """Streams that open with a run of text (the system prompt): the sink tokens at the front keep slot, position and
    contents through every eviction, and the compaction does not move what two evictions in a row left in place.
    Budgets change between evictions (a sink count that shrinks, grows, drops to zero), the opening run is appended
    in two calls, and after every step V as stored is the appended V bit for bit and K the raw K rotated at the
    token's current position, on both layers; retained ids and positions bit-exact (Sec. 3.1: sink text, windows)."""
    rng = np.random.default_rng(25100960)
    d, Hq, Hkv = (64, 2, 1) if dtype == "f32" else (128, 28, 4)
    for case, (mode, sinks) in enumerate([(1, [96, 96, 96, 40, 40, 96, 64, 64, 0, 0, 33]),
                                          (0, [200, 200, 130, 130, 130, 500, 70, 70, 70, 70, 70])]):
        sec = (0, 0, 0) if mode == 0 else ((8, 12, 12) if d == 64 else (16, 24, 24))
        theta = 1e4 if dtype == "f32" else 1e6
        w = si.Workload("t", 2, Hq, Hkv, d, dtype, mode, theta, sec, 0, 0, 0, 0, 0, 0, None, 0, 300 + case)
        cache = gu.make_cache(w, capacity=2048)
        o = orc.OracleStream(2, Hq, Hkv, d, mode, theta, sec)
        _say(f"opening text run {dtype} mode={mode}")
        g0 = 0

        def append(ty, n, grid):
            nonlocal g0
            gids = np.arange(g0, g0 + n)
            g0 += n
            o.append_meta([ty] * n, grid)
            for l in range(2):
                _, k, v = w.qkv(l, gids)
                cache.append(0, l, np.full(n, ty, dtype=np.uint8) if l == 0 else None, grid if l == 0 else None,
                             gu.dev(k, w), gu.dev(v, w))
                o.append_kv(l, k, v)

        append(orc.TEXT, 150, None)
        append(orc.TEXT, 75, None)          # the run grows while the cache holds nothing else
        for c, n_sink in enumerate(sinks):
            T, H, W = int(rng.integers(1, 3)), int(rng.integers(2, 7)), int(rng.integers(2, 9))
            append(orc.VISION, T * H * W, (T, H, W))
            append(orc.TEXT, int(rng.integers(1, 12)), None)
            vw, tw = int(rng.choice([60, 150])), int(rng.choice([8, 40]))
            assert cache.evict(0, n_sink, vw, tw) == o.evict(n_sink, vw, tw)
            n = len(o)
            gids, pos3 = cache.retained(0) if n else (np.zeros(0), np.zeros((0, 3)))
            assert np.array_equal(gids, np.asarray(o.gid)) and np.array_equal(pos3, o.positions()), (case, c)
            pos = o.positions()
            tol = (1e-5 if dtype == "f32" else 4e-2) * (1 + c)      # one rounding per compaction so far
            for l in range(2):
                K, V = np.stack(o.k[l]), np.stack(o.v[l])
                assert np.array_equal(cache.read_kv(0, l, 1, 0, n).astype(np.float64), V), (case, c, l)
                e = gu.max_err(cache.read_kv(0, l, 0, 0, n), orc.rope(K, pos, mode, theta, sec))
                assert e <= tol, (case, c, l, e)


def test_opening_text_runs_of_two_streams_are_tracked_apart():
    """Two streams of one cache with opening runs of different lengths, evicted in turn with different sink counts
    (one of them twice in a row): what an eviction leaves in place is per stream, and every stored K/V row of both
    streams is what the oracle holds after each step (bf16, 3-D positions; Sec. 3.1)."""
    rng = np.random.default_rng(96082511)
    d, Hq, Hkv, mode, sec, theta = 128, 28, 4, 1, (16, 24, 24), 1e6
    w = si.Workload("t", 1, Hq, Hkv, d, "bf16", mode, theta, sec, 0, 0, 0, 0, 0, 0, None, 0, 400)
    cache = gu.make_cache(w, capacity=1024, n_streams=2)
    orcs = [orc.OracleStream(1, Hq, Hkv, d, mode, theta, sec) for _ in range(2)]
    g0 = [0, 0]
    n_ev = [0, 0]

    def append(sid, ty, n, grid):
        gids = np.arange(g0[sid], g0[sid] + n) + 100000 * sid     # different data per stream
        g0[sid] += n
        orcs[sid].append_meta([ty] * n, grid)
        _, k, v = w.qkv(0, gids)
        cache.append(sid, 0, np.full(n, ty, dtype=np.uint8), grid, gu.dev(k, w), gu.dev(v, w))
        orcs[sid].append_kv(0, k, v)

    def check(sid, tag):
        o = orcs[sid]
        n = len(o)
        K, V = np.stack(o.k[0]), np.stack(o.v[0])
        assert np.array_equal(cache.read_kv(sid, 0, 1, 0, n).astype(np.float64), V), (tag, sid)
        e = gu.max_err(cache.read_kv(sid, 0, 0, 0, n), orc.rope(K, o.positions(), mode, theta, sec))
        assert e <= 4e-2 * (1 + n_ev[sid]), (tag, sid, e)

    append(0, orc.TEXT, 96, None)
    append(1, orc.TEXT, 200, None)
    schedule = [(0, 64), (1, 160), (1, 160), (0, 64), (0, 32), (1, 40), (0, 64), (1, 160), (0, 0), (1, 96)]
    for step, (sid, n_sink) in enumerate(schedule):
        for s2 in (0, 1):
            append(s2, orc.VISION, 2 * 4 * 6, (2, 4, 6))
            append(s2, orc.TEXT, int(rng.integers(1, 9)), None)
        _say(f"two streams: step {step}, stream {sid} evicts with {n_sink} sinks")
        assert cache.evict(sid, n_sink, 100, 12) == orcs[sid].evict(n_sink, 100, 12)
        n_ev[sid] += 1
        for s2 in (0, 1):
            check(s2, step)


# ----------------------------------------------------------------------------
# single operations
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("dtype,mode", [("f32", 0), ("bf16", 1), ("bf16", 0), ("f32", 1)])
def test_rope_apply_and_stored_kv(dtype, mode):
    """sv_rope_apply on Q and K, K as stored by append, and K/V rows after a compaction."""
    d, Hq, Hkv = (64, 2, 1) if dtype == "f32" else (128, 28, 4)
    sec = (0, 0, 0) if mode == 0 else ((8, 12, 12) if d == 64 else (16, 24, 24))
    theta = 1e4 if dtype == "f32" else 1e6
    w = si.Workload("t", 1, Hq, Hkv, d, dtype, mode, theta, sec, 3, 70, 5, 0, 0, 0, None, 0, 77)
    cache = gu.make_cache(w, capacity=512)
    o = orc.OracleStream(1, Hq, Hkv, d, mode, theta, sec)
    spans = [(orc.TEXT, 7, None), (orc.VISION, 60, (3, 4, 5)), (orc.TEXT, 9, None), (orc.VISION, 48, (1, 6, 8)),
             (orc.TEXT, 3, None)]
    g0 = 0
    for ty, n, grid in spans:
        gids = np.arange(g0, g0 + n)
        g0 += n
        q, k, v = w.qkv(0, gids)
        grid_use = grid if (mode == 1 or ty == orc.VISION) else None
        cache.append(0, 0, np.full(n, ty, dtype=np.uint8), grid_use, gu.dev(k, w), gu.dev(v, w))
        o.append_meta([ty] * n, grid_use if mode == 1 else None)
        o.append_kv(0, k, v)
    tol = 1e-5 if dtype == "f32" else 4e-2     # bf16: one rounding of values up to ~4.5 in magnitude
    n = len(o)
    # fresh Q and K rotated in place at the positions of all slots
    q, k, _ = w.qkv(0, np.arange(1000, 1000 + n))
    qd, kd = gu.dev(q, w), gu.dev(k, w)
    cache.rope_apply(0, 0, n, qd, kd)
    pos = o.positions()
    assert gu.max_err(gu.host(qd), orc.rope(q, pos, mode, theta, sec)) <= tol
    assert gu.max_err(gu.host(kd), orc.rope(k, pos, mode, theta, sec)) <= tol
    # K as stored (rotated on append), V as stored (verbatim)
    K, V = np.stack(o.k[0]), np.stack(o.v[0])
    assert gu.max_err(cache.read_kv(0, 0, 0, 0, n), orc.rope(K, pos, mode, theta, sec)) <= tol
    assert np.array_equal(cache.read_kv(0, 0, 1, 0, n).astype(np.float64), V)
    # evict: V rows move verbatim, K rows are re-rotated to the new positions
    n2 = cache.evict(0, w.n_sink, w.vision_window, w.text_window)
    assert n2 == o.evict(w.n_sink, w.vision_window, w.text_window) and 0 < n2 < n
    ids, pos_g = cache.retained(0)
    assert np.array_equal(ids, np.asarray(o.gid)) and np.array_equal(pos_g.astype(np.int64), o.positions())
    K, V = np.stack(o.k[0]), np.stack(o.v[0])
    assert np.array_equal(cache.read_kv(0, 0, 1, 0, n2).astype(np.float64), V)
    assert gu.max_err(cache.read_kv(0, 0, 0, 0, n2), orc.rope(K, o.positions(), mode, theta, sec)) <= 2 * tol


def _attn_case(dtype, Hq, Hkv, d, n_kv, n_q, causal, seed, splits=0, flags=0):
    w = si.Workload("a", 1, Hq, Hkv, d, dtype, 2, 1e4, (0, 0, 0), 0, 0, 0, 0, 0, 0, None, 0, seed)
    cache = sv.Cache(1, Hq, Hkv, d, sv.SV_DTYPE_F32 if dtype == "f32" else sv.SV_DTYPE_BF16, sv.SV_ROPE_NONE, 1e4,
                     (0, 0, 0), 1, n_kv + 8, max(n_q, 1), flags=flags)
    cache.set_option(sv.SV_OPT_CHUNK_SPLITS, splits)
    gids = np.arange(n_kv)
    bf = dtype == "bf16"
    k = si.normal(seed, si.TENSOR_K, 0, gids, Hkv, d, bf)
    v = si.normal(seed, si.TENSOR_V, 0, gids, Hkv, d, bf)
    q = si.normal(seed, si.TENSOR_Q, 0, gids[n_kv - n_q:], Hq, d, bf)
    cache.append(0, 0, np.zeros(n_kv, dtype=np.uint8), None, gu.dev(k, w), gu.dev(v, w))
    qd = gu.dev(q, w)
    od = torch.empty_like(qd)
    cache.attn_chunk(0, 0, qd, od, causal)
    ref = orc.gqa_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64),
                            np.arange(n_kv - n_q, n_kv), causal)
    return gu.max_err(gu.host(od), ref), cache, w, q, k, v


@pytest.mark.parametrize("n_kv,n_q,causal,splits", [
    (64, 64, True, 0), (200, 37, True, 0), (1000, 256, True, 0), (1333, 300, True, 3),
    (777, 100, False, 2), (5392, 256, True, 0), (130, 1, True, 0)])
def test_attn_chunk_mfma_shapes(n_kv, n_q, causal, splits):
    _say(f"attn_chunk mfma n_kv={n_kv} n_q={n_q} causal={causal} splits={splits}")
    err, *_ = _attn_case("bf16", 28, 4, 128, n_kv, n_q, causal, 300 + n_kv, splits=splits)
    assert err <= gu.TOL["bf16"], err


@pytest.mark.parametrize("n_kv,n_q,causal,splits", [(200, 37, True, 0), (777, 100, False, 3), (1400, 1, True, 5)])
def test_generic_kernels_on_bf16_head_dim_128(n_kv, n_q, causal, splits):
    """SV_FLAG_GENERIC_KERNELS: the vector-ALU row kernels (chunk prefill and decode, forced key-range counts) on the
    data type and head shape that the matrix-core kernels normally take."""
    _say(f"generic kernels bf16 d128 n_kv={n_kv} n_q={n_q} causal={causal} splits={splits}")
    err, cache, w, q, k, v = _attn_case("bf16", 28, 4, 128, n_kv, n_q, causal, 900 + n_kv,
                                        flags=sv.SV_FLAG_GENERIC_KERNELS)
    assert err <= gu.TOL["bf16"], err
    cache.set_option(sv.SV_OPT_DECODE_SPLITS, splits)
    qd1 = gu.dev(q[-1:], w)
    od1 = torch.empty_like(qd1)
    cache.attn_decode(0, [0], qd1, od1)
    ref1 = orc.gqa_attention(q[-1:].astype(np.float64), k.astype(np.float64), v.astype(np.float64),
                             np.array([n_kv - 1]), True)
    assert gu.max_err(gu.host(od1), ref1) <= gu.TOL["bf16"]


def test_attn_chunk_wide_score_range():
    """Scores whose row maxima jump by tens to hundreds of binary orders from one key tile to the next (key blocks
    scaled by exact powers of two, one late key by 128): the running-maximum logic of the chunk kernel (steps of
    the reference maximum, probabilities taken before the tile's maxima are known, redo on overflow) must still
    reproduce the plain softmax, which is then nearly one-hot."""
    Hq, Hkv, d, n_kv, n_q, seed = 28, 4, 128, 1100, 200, 4242
    w = si.Workload("a", 1, Hq, Hkv, d, "bf16", 2, 1e4, (0, 0, 0), 0, 0, 0, 0, 0, 0, None, 0, seed)
    gids = np.arange(n_kv)
    k = si.normal(seed, si.TENSOR_K, 0, gids, Hkv, d, True)
    v = si.normal(seed, si.TENSOR_V, 0, gids, Hkv, d, True)
    q = si.normal(seed, si.TENSOR_Q, 0, gids[n_kv - n_q:], Hq, d, True)
    k[0:64] *= 1.0 / 64          # a first tile far below what follows
    k[192:256] *= 16
    k[640:704] *= 32
    k[901] *= 128
    k[1000:1010] *= 8            # inside the causal part of the chunk
    _say("attn_chunk wide score range")
    for causal in (True, False):
        cache = sv.Cache(1, Hq, Hkv, d, sv.SV_DTYPE_BF16, sv.SV_ROPE_NONE, 1e4, (0, 0, 0), 1, n_kv + 8, n_q)
        cache.append(0, 0, np.zeros(n_kv, dtype=np.uint8), None, gu.dev(k, w), gu.dev(v, w))
        qd = gu.dev(q, w)
        od = torch.empty_like(qd)
        cache.attn_chunk(0, 0, qd, od, causal)
        ref = orc.gqa_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64),
                                np.arange(n_kv - n_q, n_kv), causal)
        got = gu.host(od)
        assert np.isfinite(got).all()
        assert gu.max_err(got, ref) <= gu.TOL["bf16"], (causal, gu.max_err(got, ref))


def test_attn_randomized_shapes():
    """Seeded sweep over cache lengths 1..2600, chunk lengths 1..300, both masks, forced split counts and key blocks
    scaled by powers of two (row maxima that drift or jump between tiles): chunk attention of the default kernel and
    the decode of the last token, each against the oracle."""
    rng = np.random.default_rng(20251009)
    for case in range(120):
        n_kv = int(rng.choice([rng.integers(1, 130), rng.integers(130, 700), rng.integers(700, 2600)]))
        n_q = int(min(n_kv, rng.choice([1, rng.integers(1, 40), rng.integers(40, 300)])))
        causal = bool(rng.integers(0, 2))
        splits = int(rng.choice([0, 0, 1, 2, 3, 5]))
        scale_mode = int(rng.integers(0, 3))
        seed = 7000 + case
        w = si.Workload("a", 1, 28, 4, 128, "bf16", 2, 1e4, (0, 0, 0), 0, 0, 0, 0, 0, 0, None, 0, seed)
        gids = np.arange(n_kv)
        k = si.normal(seed, si.TENSOR_K, 0, gids, 4, 128, True)
        v = si.normal(seed, si.TENSOR_V, 0, gids, 4, 128, True)
        q = si.normal(seed, si.TENSOR_Q, 0, gids[n_kv - n_q:], 28, 128, True)
        if scale_mode == 1:      # magnitudes growing along the keys (powers of two keep bf16 exact)
            for b in range(0, n_kv, 48):
                k[b:b + 48] *= 2.0 ** min(6, b // 96)
        elif scale_mode == 2:    # blocks scaled up or down at random
            for b in range(0, n_kv, 32):
                k[b:b + 32] *= 2.0 ** int(rng.integers(-5, 6))
        _say(f"randomized case {case}: n_kv={n_kv} n_q={n_q} causal={causal} splits={splits} scale_mode={scale_mode}")
        cache = sv.Cache(1, 28, 4, 128, sv.SV_DTYPE_BF16, sv.SV_ROPE_NONE, 1e4, (0, 0, 0), 1, n_kv + 8, n_q)
        cache.set_option(sv.SV_OPT_CHUNK_SPLITS, splits)
        cache.set_option(sv.SV_OPT_DECODE_TILES_PER_WAVE, int(rng.choice([0, 0, 1, 3])))
        cache.append(0, 0, np.zeros(n_kv, dtype=np.uint8), None, gu.dev(k, w), gu.dev(v, w))
        qd = gu.dev(q, w)
        od = torch.empty_like(qd)
        cache.attn_chunk(0, 0, qd, od, causal)
        k64, v64 = k.astype(np.float64), v.astype(np.float64)
        ref = orc.gqa_attention(q.astype(np.float64), k64, v64, np.arange(n_kv - n_q, n_kv), causal)
        got = gu.host(od)
        assert np.isfinite(got).all(), case
        assert gu.max_err(got, ref) <= gu.TOL["bf16"], (case, gu.max_err(got, ref))
        qd1 = gu.dev(q[-1:], w)
        od1 = torch.empty_like(qd1)
        cache.attn_decode(0, [0], qd1, od1)
        ref1 = orc.gqa_attention(q[-1:].astype(np.float64), k64, v64, np.array([n_kv - 1]), True)
        assert gu.max_err(gu.host(od1), ref1) <= gu.TOL["bf16"], (case, "decode")


@pytest.mark.parametrize("G", [1, 2, 4, 7, 8])
def test_decode_single_stream_merge_in_launch(G):
    """Single-stream decode of the matrix-core kernel, whose key ranges are merged inside the launch: group sizes
    1..8, caches that give 1, 2, 3, 5, 9, 29 and 70 key ranges of 128 keys (every thread layout of the merge, more
    than one pass over the ranges), and ranges of 3 tiles per wavefront; each output against the oracle."""
    Hkv = 2
    Hq = G * Hkv
    for n_kv, tiles in [(100, 1), (200, 1), (300, 1), (600, 1), (1100, 1), (3700, 1), (8900, 1), (2500, 3), (640, 0)]:
        seed = 9100 + 10 * G + tiles
        w = si.Workload("a", 1, Hq, Hkv, 128, "bf16", 2, 1e4, (0, 0, 0), 0, 0, 0, 0, 0, 0, None, 0, seed)
        gids = np.arange(n_kv)
        k = si.normal(seed, si.TENSOR_K, 0, gids, Hkv, 128, True)
        v = si.normal(seed, si.TENSOR_V, 0, gids, Hkv, 128, True)
        q = si.normal(seed, si.TENSOR_Q, 0, gids[-1:], Hq, 128, True)
        _say(f"decode merge in launch: G={G} n_kv={n_kv} tiles_per_wave={tiles}")
        cache = sv.Cache(1, Hq, Hkv, 128, sv.SV_DTYPE_BF16, sv.SV_ROPE_NONE, 1e4, (0, 0, 0), 1, n_kv + 8, 1)
        cache.set_option(sv.SV_OPT_DECODE_TILES_PER_WAVE, tiles)
        cache.append(0, 0, np.zeros(n_kv, dtype=np.uint8), None, gu.dev(k, w), gu.dev(v, w))
        qd = gu.dev(q, w)
        od = torch.empty_like(qd)
        cache.attn_decode(0, [0], qd, od)
        ref = orc.gqa_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64),
                                np.array([n_kv - 1]), True)
        got = gu.host(od)
        assert np.isfinite(got).all(), (G, n_kv)
        assert gu.max_err(got, ref) <= gu.TOL["bf16"], (G, n_kv, gu.max_err(got, ref))
        cache.close()


def test_decode_single_stream_repeated_launches():
    """The in-launch merge of a single stream's key ranges leaves its scratch words zero: the same decode seven
    times in a row, between them decodes of a longer and a shorter cache through the same scratch, all equal to the
    oracle's result."""
    seed = 9301
    w = si.Workload("a", 1, 28, 4, 128, "bf16", 2, 1e4, (0, 0, 0), 0, 0, 0, 0, 0, 0, None, 0, seed)
    lens = [1500, 4000, 300]
    cache = sv.Cache(1, 28, 4, 128, sv.SV_DTYPE_BF16, sv.SV_ROPE_NONE, 1e4, (0, 0, 0), len(lens), max(lens) + 8, 1)
    qs, refs = [], []
    for s_, n_kv in enumerate(lens):
        gids = np.arange(n_kv)
        k = si.normal(seed + s_, si.TENSOR_K, 0, gids, 4, 128, True)
        v = si.normal(seed + s_, si.TENSOR_V, 0, gids, 4, 128, True)
        q = si.normal(seed + s_, si.TENSOR_Q, 0, gids[-1:], 28, 128, True)
        cache.append(s_, 0, np.zeros(n_kv, dtype=np.uint8), None, gu.dev(k, w), gu.dev(v, w))
        qs.append(gu.dev(q, w))
        refs.append(orc.gqa_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64),
                                      np.array([n_kv - 1]), True))
    for i in range(7):
        for s_ in (0, 1, 0, 2):
            _say(f"repeated single-stream decode {i}, stream {s_}")
            od = torch.full_like(qs[s_], float("nan"))
            cache.attn_decode(0, [s_], qs[s_], od)
            got = gu.host(od)
            assert np.isfinite(got).all(), (i, s_)
            assert gu.max_err(got, refs[s_]) <= gu.TOL["bf16"], (i, s_, gu.max_err(got, refs[s_]))
    cache.close()


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 2, 1, 64), ("f32", 8, 2, 128), ("bf16", 4, 4, 64), ("bf16", 16, 2, 64)])
@pytest.mark.parametrize("n_kv,n_q,causal", [(72, 16, True), (300, 41, False), (1, 1, True)])
def test_attn_chunk_rows_path(dtype, Hq, Hkv, d, n_kv, n_q, causal):
    _say(f"attn_chunk rows {dtype} Hq={Hq} Hkv={Hkv} d={d} n_kv={n_kv} n_q={n_q}")
    err, *_ = _attn_case(dtype, Hq, Hkv, d, n_kv, n_q, causal, 500 + n_kv + d)
    assert err <= gu.TOL[dtype], err


def test_attn_constant_v_and_single_key():
    """Closed forms on the GPU path itself: constant V returns V; the first query of a causal chunk sees one key."""
    w = si.Workload("c", 1, 28, 4, 128, "bf16", 2, 1e4, (0, 0, 0), 0, 0, 0, 0, 0, 0, None, 0, 9)
    n = 700
    cache = sv.Cache(1, 28, 4, 128, sv.SV_DTYPE_BF16, sv.SV_ROPE_NONE, 1e4, (0, 0, 0), 1, n, n)
    q, k, _ = w.qkv(0, np.arange(n))
    v0 = si.normal(9, si.TENSOR_V, 0, np.arange(1), 4, 128, True)
    cache.append(0, 0, np.zeros(n, dtype=np.uint8), None, gu.dev(k, w), gu.dev(np.repeat(v0, n, axis=0), w))
    qd = gu.dev(q, w)
    od = torch.empty_like(qd)
    cache.attn_chunk(0, 0, qd, od, True)          # n_q == n_kv: query 0 sees only key 0
    out = gu.host(od).reshape(n, 4, 7, 128)
    assert np.abs(out - v0.astype(np.float64)[0][None, :, None, :]).max() <= 2 ** -7 * np.abs(v0).max()
    od1 = torch.empty(1, 28, 128, device="cuda:0", dtype=torch.bfloat16)
    cache.attn_decode(0, [0], qd[-1:].contiguous(), od1)
    assert np.abs(gu.host(od1).reshape(4, 7, 128) - v0.astype(np.float64)[0][:, None, :]).max() <= 2 ** -7 * np.abs(v0).max()


def test_decode_ragged_batch_full_size():
    """16 streams with per-stream budgets (ragged caches), one decode token per stream in one call."""
    rb = si.workload_ragged_batch()
    w = rb.base
    lens = rb.lengths()
    cache = sv.Cache(1, 28, 4, 128, sv.SV_DTYPE_BF16, sv.SV_ROPE_3D, w.rope_theta, w.mrope_sections, rb.n_streams,
                     max(lens) + 8, 16)
    oracles, q_all, ref = [], [], []
    for s in range(rb.n_streams):
        _say(f"ragged stream {s} len {lens[s]}")
        ws = copy.copy(w)
        ws.seed = w.seed + 10 * s
        o = orc.OracleStream(1, 28, 4, 128, orc.ROPE_3D, w.rope_theta, w.mrope_sections)
        g0 = 0
        # sink text, then the text whose vision is gone, then (vision block + 16 text) chunks
        n_chunks = rb.vision_windows[s] // 256
        text_only = 512 + rb.text_windows[s] - 16 * n_chunks
        spans = [(orc.TEXT, text_only if text_only > 0 else 512, None)]
        for _ in range(n_chunks):
            spans += [(orc.VISION, 256, (1, 16, 16)), (orc.TEXT, 16, None)]
        for ty, n, grid in spans:
            gids = np.arange(g0, g0 + n)
            g0 += n
            k = si.normal(ws.seed, si.TENSOR_K, 0, gids, 4, 128, True)
            v = si.normal(ws.seed, si.TENSOR_V, 0, gids, 4, 128, True)
            cache.append(s, 0, np.full(n, ty, dtype=np.uint8), grid, gu.dev(k, w), gu.dev(v, w))
            o.append_meta([ty] * n, grid)
            o.append_kv(0, k, v)
        assert cache.len(s) == len(o)
        oracles.append(o)
        q, _, _ = ws.qkv(0, np.array([g0 - 1]))
        q_all.append(q)
        ref.append(o.attend(0, q, [len(o) - 1]))
        ids, pos = cache.retained(s)
        assert np.array_equal(pos.astype(np.int64), o.positions())
    qd = gu.dev(np.concatenate(q_all), w)
    for s in range(rb.n_streams):
        cache.rope_apply(s, cache.len(s) - 1, 1, qd[s:s + 1], None)
    od = torch.empty_like(qd)
    cache.attn_decode(0, list(range(rb.n_streams)), qd, od)
    err = gu.max_err(gu.host(od), np.concatenate(ref))
    _say(f"ragged decode max-abs err {err:.3e}, total keys {sum(cache.len(s) for s in range(rb.n_streams))}")
    assert err <= gu.TOL["bf16"]
    # one more token per stream through the fused step (append + rotate + attend in one launch)
    q2, k2, v2, ref2 = [], [], [], []
    for s in range(rb.n_streams):
        gid = np.array([10_000_000 + s])
        q, k, v = si.normal(7, si.TENSOR_Q, 0, gid, 28, 128, True), si.normal(7, si.TENSOR_K, 0, gid, 4, 128, True), \
            si.normal(7, si.TENSOR_V, 0, gid, 4, 128, True)
        q2.append(q), k2.append(k), v2.append(v)
        oracles_s = oracles[s]
        oracles_s.append_meta([orc.TEXT])
        oracles_s.append_kv(0, k, v)
        ref2.append(oracles_s.attend(0, q, [len(oracles_s) - 1]))
    od2 = torch.empty_like(qd)
    cache.decode_step(0, list(range(rb.n_streams)), gu.dev(np.concatenate(q2), w), gu.dev(np.concatenate(k2), w),
                      gu.dev(np.concatenate(v2), w), od2)
    err2 = gu.max_err(gu.host(od2), np.concatenate(ref2))
    _say(f"ragged fused decode step max-abs err {err2:.3e}")
    assert err2 <= gu.TOL["bf16"]
    for s in range(rb.n_streams):
        _, pos = cache.retained(s)
        assert np.array_equal(pos.astype(np.int64), oracles[s].positions())


def test_decode_long_single_stream():
    """One stream long enough (50k tokens, 102 MB of K and V per layer) that its decode launch takes the
    non-temporal-load instantiation of the single-stream kernel; plain decode and the fused step against the oracle."""
    n = 50_000
    w = si.Workload("l", 1, 28, 4, 128, "bf16", 2, 1e6, (16, 24, 24), 0, 0, 0, 0, 0, 0, None, 0, 77)
    cache = sv.Cache(1, 28, 4, 128, sv.SV_DTYPE_BF16, sv.SV_ROPE_3D, w.rope_theta, w.mrope_sections, 1, n + 8, 16)
    o = orc.OracleStream(1, 28, 4, 128, orc.ROPE_3D, w.rope_theta, w.mrope_sections)
    _say(f"long single stream decode, {n} tokens")
    for g0 in range(0, n, 10_000):
        gids = np.arange(g0, g0 + 10_000)
        k = si.normal(w.seed, si.TENSOR_K, 0, gids, 4, 128, True)
        v = si.normal(w.seed, si.TENSOR_V, 0, gids, 4, 128, True)
        cache.append(0, 0, np.full(len(gids), orc.TEXT, dtype=np.uint8), None, gu.dev(k, w), gu.dev(v, w))
        o.append_meta([orc.TEXT] * len(gids))
        o.append_kv(0, k, v)
    q, _, _ = w.qkv(0, np.array([n - 1]))
    qd = gu.dev(q, w)
    cache.rope_apply(0, n - 1, 1, qd, None)
    od = torch.empty_like(qd)
    cache.attn_decode(0, [0], qd, od)
    err = gu.max_err(gu.host(od), o.attend(0, q, [n - 1]))
    assert err <= gu.TOL["bf16"], err
    gid = np.array([n])
    q2, k2, v2 = w.qkv(0, gid)
    o.append_meta([orc.TEXT])
    o.append_kv(0, k2, v2)
    od2 = torch.empty_like(qd)
    cache.decode_step(0, [0], gu.dev(q2, w), gu.dev(k2, w), gu.dev(v2, w), od2)
    err2 = gu.max_err(gu.host(od2), o.attend(0, q2, [n]))
    assert err2 <= gu.TOL["bf16"], err2


def test_high_frame_rate_chunk_sampled_rows():
    """1024 vision tokens per chunk against ~17.4k retained tokens; oracle evaluates sampled query rows."""
    w = si.workload_high_fps(n_chunks=18)
    g, o = gu.GpuStream(w, [0]), sv_step.new_stream(w, [0])
    g.preamble()
    sv_step.append_preamble(o, w, [0])
    run, cache = g.run, g.cache
    for c in range(w.n_chunks):
        _say(f"high_fps chunk {c}")
        n_ret = run.evict()
        assert n_ret == o.evict(w.n_sink, w.vision_window, w.text_window)
        ch = w.chunk(c)
        gids = np.arange(ch.vision.gid0, ch.vision.gid0 + ch.vision.n)
        q, k, v = w.qkv(0, gids)
        qd, od = gu.dev(q, w), torch.empty(ch.vision.n, 28, 128, device="cuda:0", dtype=torch.bfloat16)
        slot0 = run.prefill([qd], [gu.dev(k, w)], [gu.dev(v, w)], [od], ch.vision.grid_thw)
        assert slot0 == o.append_meta([orc.VISION] * ch.vision.n, ch.vision.grid_thw)
        o.append_kv(0, k, v)
        if c >= 16:
            rows = np.array([0, 1, 7, 130, 511, 512, 800, 1022, 1023])
            ref = o.attend(0, q[rows], list(slot0 + rows))
            e = gu.max_err(gu.host(od)[rows], ref)
            _say(f"  n_kv {len(o)}  sampled max-abs err {e:.3e}")
            assert e <= gu.TOL["bf16"]
        tg = np.arange(ch.text_gid0, ch.text_gid0 + ch.n_text)
        qt, kt, vt = w.qkv(0, tg)
        for t in range(ch.n_text):
            qd1, od1 = gu.dev(qt[t:t + 1], w), torch.empty(1, 28, 128, device="cuda:0", dtype=torch.bfloat16)
            run.decode([qd1], [gu.dev(kt[t:t + 1], w)], [gu.dev(vt[t:t + 1], w)], [od1])
            o.append_meta([orc.TEXT])
            o.append_kv(0, kt[t:t + 1], vt[t:t + 1])
            if c == 17 and t in (0, 15):
                e = gu.max_err(gu.host(od1), o.attend(0, qt[t:t + 1], [len(o) - 1]))
                assert e <= gu.TOL["bf16"], e
        ids, pos = cache.retained(0)
        assert np.array_equal(ids, np.asarray(o.gid)) and np.array_equal(pos.astype(np.int64), o.positions())
    assert n_ret == 512 + 17 * 16 + 16384      # sink + the text appended so far + the full vision window


# ----------------------------------------------------------------------------
# edge cases and the error contract
# ----------------------------------------------------------------------------

def test_edges_and_errors():
    w = si.workload_tiny()
    cache = gu.make_cache(w, capacity=64)
    z = lambda n: torch.zeros(n, 1, 64, device="cuda:0")
    ty = lambda n, t=0: np.full(n, t, dtype=np.uint8)
    assert cache.len(0) == 0 and cache.evict(0, 8, 32, 16) == 0            # empty cache
    assert cache.append(0, 0, ty(0), None, z(0), z(0)) == 0                # empty append
    ids, pos = cache.retained(0)
    assert ids.size == 0
    with pytest.raises(sv.SvError) as e:
        cache.append(0, 0, ty(65), None, z(65), z(65))
    assert e.value.status == -2 and cache.len(0) == 0                      # capacity, nothing changed
    with pytest.raises(sv.SvError) as e:
        cache.append(0, 0, ty(4, 7), None, z(4), z(4))
    assert e.value.status == -1                                            # bad type
    with pytest.raises(sv.SvError) as e:
        cache.append(0, 0, ty(6, 1), (1, 2, 2), z(6), z(6))
    assert e.value.status == -1                                            # grid does not match n
    with pytest.raises(sv.SvError) as e:
        cache.evict(0, -1, 0, 0)
    assert e.value.status == -1
    with pytest.raises(sv.SvError) as e:
        cache.attn_chunk(0, 0, z(1).expand(1, 2, 64).contiguous(), z(1).expand(1, 2, 64).contiguous())
    assert e.value.status == -1                                            # no tokens yet
    q, k, v = w.qkv(0, np.arange(20))
    cache.append(0, 0, ty(20), None, gu.dev(k, w), gu.dev(v, w))
    assert cache.evict(0, 0, sv.SV_WINDOW_INF, sv.SV_WINDOW_INF) == 20      # infinite windows keep everything
    assert cache.evict(0, 100, 0, 0) == 20                                 # sink larger than the stream
    assert cache.evict(0, 0, 0, 0) == 0                                    # evict everything
    assert cache.retained(0)[0].size == 0
    # the stream goes on after a total eviction: positions restart at 0
    cache.append(0, 0, ty(5), None, gu.dev(k[:5], w), gu.dev(v[:5], w))
    ids, pos = cache.retained(0)
    assert ids.tolist() == [20, 21, 22, 23, 24] and pos[:, 0].tolist() == [0, 1, 2, 3, 4]
    qd = gu.dev(q[:5], w)
    od = torch.empty_like(qd)
    qr = orc.rope(q[:5], np.arange(5)[:, None].repeat(3, 1), 0, 1e4, (0, 0, 0))
    cache.rope_apply(0, 0, 5, qd, None)
    cache.attn_chunk(0, 0, qd, od, True)
    ref = orc.gqa_attention(qr, orc.rope(k[:5], np.arange(5)[:, None].repeat(3, 1), 0, 1e4, (0, 0, 0)),
                            v[:5].astype(np.float64), np.arange(5), True)
    assert gu.max_err(gu.host(od), ref) <= 1e-5

    # layer bookkeeping: a 2-layer cache refuses attention / evict / a new append until every layer is stored
    c2 = sv.Cache(2, 2, 1, 64, sv.SV_DTYPE_F32, sv.SV_ROPE_1D, 1e4, (0, 0, 0), 1, 64, 16)
    c2.append(0, 0, ty(4), None, z(4), z(4))
    for call in (lambda: c2.evict(0, 1, 1, 1),
                 lambda: c2.append(0, 0, ty(1), None, z(1), z(1)),
                 lambda: c2.attn_chunk(0, 1, torch.zeros(4, 2, 64, device="cuda:0"), torch.zeros(4, 2, 64, device="cuda:0")),
                 lambda: c2.append(0, 1, None, None, z(3), z(3))):
        with pytest.raises(sv.SvError) as e:
            call()
        assert e.value.status == -3
    c2.append(0, 1, None, None, z(4), z(4))
    assert c2.evict(0, 1, 1, 1) == 2                                       # first text token + last text token
    # configuration checks
    for bad in (dict(n_q_heads=3, n_kv_heads=2), dict(head_dim=96), dict(mrope_sections=(1, 2, 3), rope_mode=1)):
        kw = dict(n_layers=1, n_q_heads=2, n_kv_heads=1, head_dim=64, dtype=0, rope_mode=0, rope_theta=1e4,
                  mrope_sections=(0, 0, 0), n_streams=1, capacity_tokens=8, max_q_tokens=8)
        kw.update(bad)
        with pytest.raises(sv.SvError):
            sv.Cache(**kw)


# ---------------------------------------------------------------------------------------------------------
# Budget sweep and the no-eviction mode (the sink / window ablations and the full-attention baseline):
# zero-length windows, infinite windows (cache grows, positions stay native), mixed.
# ---------------------------------------------------------------------------------------------------------
INF = sv.SV_WINDOW_INF


@pytest.mark.parametrize("n_sink,vision_window,text_window", [
    (0, 0, 0), (0, 128, 16), (16, 0, 16), (16, 128, 0), (16, INF, INF), (64, 256, 64), (0, INF, 0), (8, 64, INF)])
def test_budget_sweep_and_no_evict_mode(n_sink, vision_window, text_window):
    w = si.Workload("qwen7b_64v_sweep", 1, 28, 4, 128, "bf16", 1, 1.0e6, (16, 24, 24),
                    n_sink, vision_window, text_window, 24, 64, 8, (1, 8, 8), 9, 1006)
    g, o = gu.GpuStream(w, [0]), sv_step.new_stream(w, [0])
    g.preamble()
    sv_step.append_preamble(o, w, [0])
    for c in range(w.n_chunks):
        _say(f"budget sweep ({n_sink},{vision_window},{text_window}) chunk {c}")
        rg, ro = g.step_chunk(c), sv_step.step_chunk(o, w, c, [0], want_outputs=c in (0, 1, 4, 8))
        gu.assert_int_parity(rg, ro, f"chunk {c}")
        if c in (0, 1, 4, 8):
            gu.assert_attn_parity(rg, ro, gu.TOL["bf16"], f"chunk {c}")
    if vision_window == INF and text_window == INF:
        # nothing was ever dropped: every token still sits at its arrival slot
        n = w.preamble_text + w.n_chunks * w.tokens_per_chunk
        assert rg["gids_end"].tolist() == list(range(n))


def test_probe_rates_are_plausible():
    """The measurement aid returns the device's sustained rates: below the published peaks, well above zero."""
    buf = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").fill_(1.0)      # 1 GiB
    tflops, tflops_rnd, gbs = sv.sv_probe_rates(buf)
    assert 500.0 < tflops <= 2600.0, tflops
    assert 500.0 < tflops_rnd <= tflops * 1.05, (tflops_rnd, tflops)
    assert 1000.0 < gbs <= 8200.0, gbs
    with pytest.raises(sv.SvError):
        sv.sv_probe_rates(buf[:16])            # smaller than the 1 MiB the probe asks for


def test_long_stream_attention_at_late_chunks():
    """Attention parity deep into a one-hour stream (chunks 64, 1800 and 3599 of the 28q/4kv x 128 M-RoPE stream,
    three layers), driven by the native per-second call; retained counts checked at every chunk."""
    base = si.workload_qwen_layer(n_chunks=3600, n_layers=3, seed=1003)
    w = gu.pooled(base)
    layers = [0, 13, 27]
    L, nv, nt = 3, w.vision_per_chunk, w.text_per_chunk
    cache = gu.make_cache(w, n_layers=L, capacity=w.retained_steady() + w.tokens_per_chunk + 64)
    dev_tab = [[torch.from_numpy(np.ascontiguousarray(t, dtype=np.float32)).to("cuda:0").to(torch.bfloat16)
                for t in w.tables(l)] for l in layers]                 # [layer][q|k|v] -> [keys, H, d]
    Q, K, V = (torch.stack([dev_tab[j][i] for j in range(L)]) for i in range(3))   # [L, keys, H, d]
    run = gu.StreamRunner(cache, w.n_sink, w.vision_window, w.text_window)
    pre = torch.arange(w.preamble_text, device="cuda:0")
    run.preamble(list(K[:, pre]), list(V[:, pre]))
    o = sv_step.new_stream(w, layers)
    sv_step.append_preamble(o, w, layers)
    ov = torch.empty(L, nv, w.n_q_heads, w.head_dim, device="cuda:0", dtype=torch.bfloat16)
    ot = torch.empty(nt, L, w.n_q_heads, w.head_dim, device="cuda:0", dtype=torch.bfloat16)
    samples = {64, 1800, 3599}
    for c in range(w.n_chunks):
        ch = w.chunk(c)
        kv_ = torch.from_numpy(w.key(np.arange(ch.vision.gid0, ch.vision.gid0 + nv))).to("cuda:0")
        kt_ = torch.from_numpy(w.key(np.arange(ch.text_gid0, ch.text_gid0 + nt))).to("cuda:0")
        text = lambda X: X[:, kt_].permute(1, 0, 2, 3).unsqueeze(2).contiguous()      # [nt, L, 1, H, d]
        n_ret = cache.stream_step(0, w.n_sink, w.vision_window, w.text_window, q_vision=Q[:, kv_].contiguous(),
                                  k_vision=K[:, kv_].contiguous(), v_vision=V[:, kv_].contiguous(), o_vision=ov,
                                  grid_thw=w.grid_thw, q_text=text(Q), k_text=text(K), v_text=text(V), o_text=ot)
        ro = sv_step.step_chunk(o, w, c, layers, want_outputs=c in samples)
        assert n_ret == ro["n_retained"], c
        if c in samples:
            _say(f"late-chunk attention parity, chunk {c}")
            gids, pos = cache.retained(0)
            assert np.array_equal(gids, np.asarray(ro["gids_end"], dtype=np.int64))
            assert np.array_equal(pos.astype(np.int64), ro["pos_end"])
            gv, gt = gu.host(ov), gu.host(ot)
            for j in range(L):
                assert gu.max_err(gv[j], ro["prefill"][j]) <= gu.TOL["bf16"], (c, j)
                for t in range(nt):
                    assert gu.max_err(gt[t, j], ro["decode"][t][j][0]) <= gu.TOL["bf16"], (c, j, t)
