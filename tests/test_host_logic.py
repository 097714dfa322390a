"""Host logic of the C-ABI library, without a GPU: call-order rules, capacity, argument checks, lengths and the
retained counts of sv_cache_evict (computed on the host from per-type intervals) against the oracle.

The caches are created with SV_FLAG_HOST_LOGIC_ONLY, so nothing is launched and the fake arena / tensor addresses
handed in are never dereferenced."""
import ctypes as C

import numpy as np
import pytest

import sv_inputs as si
from oracle import sv_oracle as orc
from paper_2510_09608_amd import binding as B

FAKE = 0x10000          # a 256-byte aligned, non-NULL "device address" that nobody reads
OK, INVALID, CAPACITY, STATE, UNSUPPORTED = 0, -1, -2, -3, -5


def _create(n_layers=1, hq=28, hkv=4, d=128, dtype=B.SV_DTYPE_BF16, rope=B.SV_ROPE_3D, sections=(16, 24, 24),
            n_streams=1, capacity=1024, max_q=256):
    cfg = B.SvConfig(n_layers, hq, hkv, d, dtype, rope, 1.0e6, (C.c_int32 * 3)(*sections), n_streams, capacity, max_q,
                     B.SV_FLAG_HOST_LOGIC_ONLY)
    lib = B.lib()
    h = C.c_void_p()
    assert lib.sv_cache_create(C.byref(cfg), FAKE, 1 << 60, None, C.byref(h)) == OK
    return lib, h


def _append(lib, h, layer, types, grid=None, stream=0):
    n = len(types)
    t = np.ascontiguousarray(types, dtype=np.uint8)
    g = None if grid is None else np.ascontiguousarray(grid, dtype=np.int32)
    slot0 = C.c_int64(-1)
    rc = lib.sv_cache_append(h, stream, layer, n, t.ctypes.data if layer == 0 else None,
                             None if g is None or layer != 0 else g.ctypes.data, FAKE, FAKE, C.byref(slot0), None)
    return rc, slot0.value


def _evict(lib, h, budgets, stream=0):
    n = C.c_int64(-1)
    rc = lib.sv_cache_evict(h, stream, budgets[0], budgets[1], budgets[2], C.byref(n), None)
    return rc, n.value


def _len(lib, h, stream=0):
    n = C.c_int64(-1)
    assert lib.sv_cache_len(h, stream, C.byref(n)) == OK
    return n.value


@pytest.mark.parametrize("budgets", [(8, 32, 16), (0, 0, 0), (0, 32, 0), (4, -1, -1), (1000, 16, 3), (3, 0, -1)])
def test_retained_counts_follow_the_keep_rule(budgets):
    """Tiny interleaved stream, call by call: the count sv_cache_evict returns and the cache length equal the
    oracle's at every chunk, for ordinary, zero and infinite budgets."""
    lib, h = _create(n_layers=2, hq=2, hkv=1, d=64, dtype=B.SV_DTYPE_F32, rope=B.SV_ROPE_1D, sections=(0, 0, 0),
                     capacity=400)
    o = orc.OracleStream(1, 2, 1, 2, orc.ROPE_1D, 1e4, (0, 0, 0))
    z = lambda n: np.zeros((n, 1, 2))
    for c in range(12):
        rc, n_ret = _evict(lib, h, budgets)
        assert rc == OK and n_ret == o.evict(*budgets) and _len(lib, h) == n_ret
        for layer in (0, 1):
            rc, slot0 = _append(lib, h, layer, [B.SV_VISION] * 16)
            assert rc == OK and slot0 == n_ret
        o.append_meta([orc.VISION] * 16)
        o.append_kv(0, z(16), z(16))
        for _ in range(4):
            for layer in (0, 1):
                assert _append(lib, h, layer, [B.SV_TEXT])[0] == OK
            o.append_meta([orc.TEXT])
            o.append_kv(0, z(1), z(1))
        assert _len(lib, h) == len(o.gid)
    assert lib.sv_cache_destroy(h) == OK


def test_native_step_counts_on_the_qwen_stream():
    """sv_stream_step sequences the second in C: retained counts and lengths over 40 chunks, into steady state."""
    w = si.workload_qwen_layer(n_chunks=40, n_layers=3)
    lib, h = _create(n_layers=3, capacity=w.retained_steady() + w.tokens_per_chunk + 8)
    o = orc.OracleStream(1, 28, 4, 2, orc.ROPE_3D, 1e6, (1, 0, 0))
    z = lambda n: np.zeros((n, 4, 2))
    for layer in range(3):
        assert _append(lib, h, layer, [B.SV_TEXT] * w.preamble_text)[0] == OK
    o.append_meta([orc.TEXT] * w.preamble_text)
    o.append_kv(0, z(w.preamble_text), z(w.preamble_text))
    io = B.SvChunkIO()
    io.n_vision, io.grid_thw = w.vision_per_chunk, (C.c_int32 * 3)(*w.grid_thw)
    io.q_vision = io.k_vision = io.v_vision = io.o_vision = FAKE
    io.n_text = w.text_per_chunk
    io.q_text = io.k_text = io.v_text = io.o_text = FAKE
    for c in range(w.n_chunks):
        for batched in ((0,) if c % 2 else (1,)):
            io.decode_layers_batched = batched
            n = C.c_int64(-1)
            assert lib.sv_stream_step(h, 0, w.n_sink, w.vision_window, w.text_window, C.byref(io), C.byref(n), None) == OK
        assert n.value == o.evict(w.n_sink, w.vision_window, w.text_window)
        o.append_meta([orc.VISION] * w.vision_per_chunk, w.grid_thw)
        o.append_kv(0, z(w.vision_per_chunk), z(w.vision_per_chunk))
        o.append_meta([orc.TEXT] * w.text_per_chunk)
        o.append_kv(0, z(w.text_per_chunk), z(w.text_per_chunk))
        assert _len(lib, h) == len(o.gid)
    assert n.value == w.retained_steady() and _len(lib, h) == w.retained_steady() + w.tokens_per_chunk
    # the next chunk would not fit a cache that is one token too small
    lib2, h2 = _create(n_layers=1, capacity=w.preamble_text + w.tokens_per_chunk - 1)
    assert _append(lib2, h2, 0, [B.SV_TEXT] * w.preamble_text)[0] == OK
    n = C.c_int64(-1)
    assert lib2.sv_stream_step(h2, 0, w.n_sink, w.vision_window, w.text_window, C.byref(io), C.byref(n), None) == CAPACITY


def test_call_order_capacity_and_argument_errors():
    lib, h = _create(n_layers=2, capacity=64, max_q=16)
    ids = (C.c_int32 * 2)(0, 0)
    # nothing cached yet: attention has no keys
    assert lib.sv_attn_decode(h, 0, ids, 1, FAKE, FAKE, None) == INVALID
    # layer 1 cannot lead an append; layer 0 needs the token types
    assert _append(lib, h, 1, [B.SV_TEXT] * 4)[0] == STATE
    assert lib.sv_cache_append(h, 0, 0, 4, None, None, FAKE, FAKE, None, None) == INVALID
    assert _append(lib, h, 0, [B.SV_TEXT] * 4) == (OK, 0)
    # half-appended: layer 0 again, eviction, attention on the layer that lags, and a different count are refused
    assert _append(lib, h, 0, [B.SV_TEXT] * 4)[0] == STATE
    assert _evict(lib, h, (1, 1, 1))[0] == STATE
    assert lib.sv_attn_chunk(h, 0, 1, FAKE, 4, FAKE, 1, None) == STATE
    assert _append(lib, h, 1, [B.SV_TEXT] * 3)[0] == STATE
    assert _append(lib, h, 1, [B.SV_TEXT] * 4) == (OK, 0)
    assert lib.sv_attn_chunk(h, 0, 1, FAKE, 4, FAKE, 1, None) == OK
    # argument checks
    assert lib.sv_attn_chunk(h, 0, 2, FAKE, 4, FAKE, 1, None) == INVALID        # layer out of range
    assert lib.sv_attn_chunk(h, 0, 0, FAKE, 5, FAKE, 1, None) == INVALID        # more queries than cached tokens
    assert lib.sv_attn_chunk(h, 0, 0, None, 4, FAKE, 1, None) == INVALID
    assert lib.sv_attn_chunk(h, 1, 0, FAKE, 4, FAKE, 1, None) == INVALID        # stream out of range
    assert _evict(lib, h, (-1, 0, 0))[0] == INVALID and _evict(lib, h, (0, -2, 0))[0] == INVALID
    assert lib.sv_rope_apply(h, 0, 2, 3, FAKE, None, None) == INVALID           # slots [2, 5) do not exist
    assert lib.sv_decode_step(h, 0, ids, 2, FAKE, FAKE, FAKE, FAKE, None) == INVALID   # the same stream twice
    # a vision block needs its grid under 3-D positions, and the grid must match the count
    assert _append(lib, h, 0, [B.SV_VISION] * 8)[0] == INVALID
    assert _append(lib, h, 0, [B.SV_VISION] * 8, grid=(1, 2, 3))[0] == INVALID
    for layer in (0, 1):
        assert _append(lib, h, layer, [B.SV_VISION] * 8, grid=(2, 2, 2)) == (OK, 4)
    # capacity: 12 cached, 64 slots
    assert _append(lib, h, 0, [B.SV_TEXT] * 53)[0] == CAPACITY and _len(lib, h) == 12
    for layer in (0, 1):
        assert _append(lib, h, layer, [B.SV_TEXT] * 52)[0] == OK
    assert lib.sv_decode_step(h, 0, ids, 1, FAKE, FAKE, FAKE, FAKE, None) == CAPACITY
    assert lib.sv_decode_step_layers(h, 0, FAKE, FAKE, FAKE, FAKE, None) == CAPACITY
    # eviction is idempotent and total eviction is legal
    assert _evict(lib, h, (2, 4, 8)) == (OK, 2 + 8 + 4) and _evict(lib, h, (2, 4, 8)) == (OK, 14)
    assert _evict(lib, h, (0, 0, 0)) == (OK, 0) and _len(lib, h) == 0
    # decode steps: layer order, then the all-layers form
    assert lib.sv_decode_step(h, 1, ids, 1, FAKE, FAKE, FAKE, FAKE, None) == STATE
    assert lib.sv_decode_step(h, 0, ids, 1, FAKE, FAKE, FAKE, FAKE, None) == OK
    assert lib.sv_decode_step_layers(h, 0, FAKE, FAKE, FAKE, FAKE, None) == STATE   # layer 1 still owes the token
    assert lib.sv_decode_step(h, 1, ids, 1, FAKE, FAKE, FAKE, FAKE, None) == OK
    assert lib.sv_decode_step_layers(h, 0, FAKE, FAKE, FAKE, FAKE, None) == OK and _len(lib, h) == 2
    # what lives in device memory cannot be inspected in this mode
    n = C.c_int64(-1)
    assert lib.sv_cache_retained(h, 0, None, None, 0, C.byref(n), None) == UNSUPPORTED and n.value == 2
    assert lib.sv_cache_destroy(h) == OK


def test_options_and_flags():
    """sv_cache_set_option keeps per-handle launch overrides (host state only); unknown options, negative values and
    unknown flag bits are refused; the generic-kernel flag is accepted."""
    lib, h = _create()
    for opt in (B.SV_OPT_CHUNK_SPLITS, B.SV_OPT_DECODE_TILES_PER_WAVE, B.SV_OPT_DECODE_SPLITS, B.SV_OPT_CHUNK_STORE):
        assert lib.sv_cache_set_option(h, opt, 3) == OK and lib.sv_cache_set_option(h, opt, 0) == OK
    assert lib.sv_cache_set_option(h, 4, 1) == INVALID and lib.sv_cache_set_option(h, -1, 1) == INVALID
    assert lib.sv_cache_set_option(h, B.SV_OPT_CHUNK_SPLITS, -2) == INVALID
    assert lib.sv_cache_set_option(None, 0, 1) == INVALID
    cfg = B.SvConfig(1, 28, 4, 128, B.SV_DTYPE_BF16, B.SV_ROPE_3D, 1.0e6, (C.c_int32 * 3)(16, 24, 24), 1, 64, 16,
                     B.SV_FLAG_GENERIC_KERNELS)
    assert lib.sv_cache_bytes(C.byref(cfg)) > 0
    cfg.flags = 4
    assert lib.sv_cache_bytes(C.byref(cfg)) == 0
    cfg.flags, cfg.capacity_tokens = 0, (1 << 24) + 1            # slots are indexed with 32-bit arithmetic
    assert lib.sv_cache_bytes(C.byref(cfg)) == 0
