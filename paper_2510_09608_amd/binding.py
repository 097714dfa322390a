"""ctypes binding of libsv.so: same names as include/sv.h, argument marshalling only.

Device buffers are torch tensors (their data_ptr() is passed through), the HIP
stream is torch's current stream unless given.  Every step of the path runs in
the library's kernels; there is no Python or CPU fallback, and a missing
library is an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

SV_DTYPE_F32, SV_DTYPE_BF16 = 0, 1
SV_ROPE_1D, SV_ROPE_3D, SV_ROPE_NONE = 0, 1, 2
SV_TEXT, SV_VISION = 0, 1
SV_WINDOW_INF = -1
SV_FLAG_GENERIC_KERNELS, SV_FLAG_HOST_LOGIC_ONLY = 1, 2
SV_OPT_CHUNK_SPLITS, SV_OPT_DECODE_TILES_PER_WAVE, SV_OPT_DECODE_SPLITS, SV_OPT_CHUNK_STORE = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libsv.so")


class SvError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {sv_strerror(status)} ({status})")
        self.status = status


class SvConfig(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("dtype", C.c_int32), ("rope_mode", C.c_int32), ("rope_theta", C.c_double),
        ("mrope_sections", C.c_int32 * 3), ("n_streams", C.c_int32), ("capacity_tokens", C.c_int64),
        ("max_q_tokens", C.c_int32), ("flags", C.c_int32),
    ]


class SvChunkIO(C.Structure):
    _fields_ = [
        ("n_vision", C.c_int32), ("grid_thw", C.c_int32 * 3), ("q_vision", C.c_void_p), ("k_vision", C.c_void_p),
        ("v_vision", C.c_void_p), ("o_vision", C.c_void_p), ("n_text", C.c_int32), ("q_text", C.c_void_p),
        ("k_text", C.c_void_p), ("v_text", C.c_void_p), ("o_text", C.c_void_p), ("decode_layers_batched", C.c_int32),
    ]


_lib = None

_SIGNATURES = {
    "sv_strerror": (C.c_char_p, [C.c_int]),
    "sv_cache_bytes": (C.c_size_t, [C.POINTER(SvConfig)]),
    "sv_cache_create": (C.c_int, [C.POINTER(SvConfig), C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]),
    "sv_cache_destroy": (C.c_int, [C.c_void_p]),
    "sv_cache_set_option": (C.c_int, [C.c_void_p, C.c_int, C.c_int]),
    "sv_cache_append": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.POINTER(C.c_int64), C.c_void_p]),
    "sv_cache_evict": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.POINTER(C.c_int64),
                                 C.c_void_p]),
    "sv_rope_apply": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sv_attn_chunk": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]),
    "sv_attn_decode": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sv_attn_decode_static": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sv_decode_step": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_void_p]),
    "sv_decode_step_layers": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p]),
    "sv_stream_step": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.POINTER(SvChunkIO),
                                 C.POINTER(C.c_int64), C.c_void_p]),
    "sv_cache_len": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int64)]),
    "sv_cache_retained": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_int64),
                                    C.c_void_p]),
    "sv_cache_read_kv": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_void_p,
                                   C.c_void_p]),
    "sv_probe_rates": (C.c_int, [C.c_void_p, C.c_size_t, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                 C.POINTER(C.c_double), C.c_void_p]),
}


def lib() -> C.CDLL:
    """Load libsv.so (built by paper_2510_09608_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2510_09608_amd.build`")
        import torch  # noqa: F401  (loads the HIP runtime this process will use before libsv binds to it)
        _lib = C.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(_lib, name)
            fn.restype, fn.argtypes = res, args
    return _lib


def exported_names() -> Sequence[str]:
    return tuple(_SIGNATURES)


def _check(status: int, what: str) -> None:
    if status != 0:
        raise SvError(status, what)


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return int(getattr(stream, "cuda_stream", stream))


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def sv_strerror(status: int) -> str:
    return lib().sv_strerror(status).decode()


def sv_cache_bytes(cfg: SvConfig) -> int:
    return int(lib().sv_cache_bytes(C.byref(cfg)))


def sv_cache_create(cfg: SvConfig, arena, stream=None) -> int:
    """arena: 1-D uint8 device tensor of at least sv_cache_bytes(cfg) bytes.  Returns the handle."""
    h = C.c_void_p()
    _check(lib().sv_cache_create(C.byref(cfg), _ptr(arena), arena.numel() * arena.element_size(), _stream(stream),
                                 C.byref(h)), "sv_cache_create")
    return h.value


def sv_cache_destroy(handle: int) -> None:
    _check(lib().sv_cache_destroy(handle), "sv_cache_destroy")


def sv_cache_set_option(handle: int, option: int, value: int) -> None:
    _check(lib().sv_cache_set_option(handle, option, value), "sv_cache_set_option")


def sv_cache_append(handle: int, stream_id: int, layer: int, n: int, types, grid_thw, k, v, stream=None) -> int:
    """types: sequence/array of SV_TEXT/SV_VISION (read at layer 0) or None; grid_thw: (T, H, W) or None."""
    types_arr = None if types is None else np.ascontiguousarray(types, dtype=np.uint8)
    grid_arr = None if grid_thw is None else np.ascontiguousarray(grid_thw, dtype=np.int32)
    slot0 = C.c_int64(-1)
    _check(lib().sv_cache_append(handle, stream_id, layer, n,
                                 None if types_arr is None else types_arr.ctypes.data,
                                 None if grid_arr is None else grid_arr.ctypes.data,
                                 _ptr(k), _ptr(v), C.byref(slot0), _stream(stream)), "sv_cache_append")
    return slot0.value


def sv_cache_evict(handle: int, stream_id: int, n_sink: int, vision_window: int, text_window: int,
                   stream=None) -> int:
    n = C.c_int64(-1)
    _check(lib().sv_cache_evict(handle, stream_id, n_sink, vision_window, text_window, C.byref(n), _stream(stream)),
           "sv_cache_evict")
    return n.value


def sv_rope_apply(handle: int, stream_id: int, slot0: int, n: int, q, k, stream=None) -> None:
    _check(lib().sv_rope_apply(handle, stream_id, slot0, n, _ptr(q), _ptr(k), _stream(stream)), "sv_rope_apply")


def sv_attn_chunk(handle: int, stream_id: int, layer: int, q, n_q: int, o, causal: bool = True, stream=None) -> None:
    _check(lib().sv_attn_chunk(handle, stream_id, layer, _ptr(q), n_q, _ptr(o), 1 if causal else 0, _stream(stream)),
           "sv_attn_chunk")


def sv_attn_decode(handle: int, layer: int, stream_ids, q, o, stream=None) -> None:
    ids = np.ascontiguousarray(stream_ids, dtype=np.int32)
    _check(lib().sv_attn_decode(handle, layer, ids.ctypes.data, int(ids.shape[0]), _ptr(q), _ptr(o), _stream(stream)),
           "sv_attn_decode")


def sv_attn_decode_static(handle: int, layer: int, stream_ids, q, o, stream=None) -> None:
    ids = np.ascontiguousarray(stream_ids, dtype=np.int32)
    _check(lib().sv_attn_decode_static(handle, layer, ids.ctypes.data, int(ids.shape[0]), _ptr(q), _ptr(o),
                                       _stream(stream)), "sv_attn_decode_static")


def sv_decode_step(handle: int, layer: int, stream_ids, q, k, v, o, stream=None) -> None:
    ids = np.ascontiguousarray(stream_ids, dtype=np.int32)
    _check(lib().sv_decode_step(handle, layer, ids.ctypes.data, int(ids.shape[0]), _ptr(q), _ptr(k), _ptr(v), _ptr(o),
                                _stream(stream)), "sv_decode_step")


def sv_decode_step_layers(handle: int, stream_id: int, q, k, v, o, stream=None) -> None:
    _check(lib().sv_decode_step_layers(handle, stream_id, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _stream(stream)),
           "sv_decode_step_layers")


def sv_stream_step(handle: int, stream_id: int, n_sink: int, vision_window: int, text_window: int,
                   q_vision=None, k_vision=None, v_vision=None, o_vision=None, grid_thw=None,
                   q_text=None, k_text=None, v_text=None, o_text=None, decode_layers_batched=False, stream=None) -> int:
    """Tensors as laid out in include/sv.h (leading dimension = layers, resp. decode steps then layers)."""
    io = SvChunkIO()
    io.n_vision = 0 if q_vision is None else int(q_vision.shape[1])
    io.grid_thw = (C.c_int32 * 3)(*(grid_thw or (0, 0, 0)))
    io.q_vision, io.k_vision, io.v_vision, io.o_vision = _ptr(q_vision), _ptr(k_vision), _ptr(v_vision), _ptr(o_vision)
    io.n_text = 0 if q_text is None else int(q_text.shape[0])
    io.q_text, io.k_text, io.v_text, io.o_text = _ptr(q_text), _ptr(k_text), _ptr(v_text), _ptr(o_text)
    io.decode_layers_batched = 1 if decode_layers_batched else 0
    n = C.c_int64(-1)
    _check(lib().sv_stream_step(handle, stream_id, n_sink, vision_window, text_window, C.byref(io), C.byref(n),
                                _stream(stream)), "sv_stream_step")
    return n.value


def sv_cache_len(handle: int, stream_id: int) -> int:
    n = C.c_int64(-1)
    _check(lib().sv_cache_len(handle, stream_id, C.byref(n)), "sv_cache_len")
    return n.value


def sv_cache_retained(handle: int, stream_id: int, stream=None) -> Tuple[np.ndarray, np.ndarray]:
    """(arrival ids [n] int64, positions [n, 3] int32) in slot order; synchronous."""
    n = sv_cache_len(handle, stream_id)
    ids = np.empty(max(n, 1), dtype=np.int64)
    pos = np.empty((max(n, 1), 3), dtype=np.int32)
    got = C.c_int64(-1)
    _check(lib().sv_cache_retained(handle, stream_id, ids.ctypes.data, pos.ctypes.data, n, C.byref(got),
                                   _stream(stream)), "sv_cache_retained")
    return ids[:n], pos[:n]


def sv_cache_read_kv(handle: int, stream_id: int, layer: int, which: int, slot0: int, n: int, n_kv_heads: int,
                     head_dim: int, dtype: int, stream=None) -> np.ndarray:
    """Stored K (which=0, rotated) or V (which=1) rows as float32 [n, n_kv_heads, head_dim]; synchronous."""
    if dtype == SV_DTYPE_F32:
        buf = np.empty((max(n, 1), n_kv_heads, head_dim), dtype=np.float32)
    else:
        buf = np.empty((max(n, 1), n_kv_heads, head_dim), dtype=np.uint16)
    _check(lib().sv_cache_read_kv(handle, stream_id, layer, which, slot0, n, buf.ctypes.data, _stream(stream)),
           "sv_cache_read_kv")
    buf = buf[:n]
    if dtype == SV_DTYPE_BF16:
        buf = (buf.astype(np.uint32) << 16).view(np.float32)
    return buf


def sv_probe_rates(buf, stream=None):
    """(sustained dense bf16 MFMA TFLOP/s on constant operands, the same on pseudo-random operands, streaming HBM
    read GB/s) measured on `buf` (a device tensor)."""
    t, tr, g = C.c_double(0.0), C.c_double(0.0), C.c_double(0.0)
    _check(lib().sv_probe_rates(_ptr(buf), buf.numel() * buf.element_size(), C.byref(t), C.byref(tr), C.byref(g),
                                _stream(stream)), "sv_probe_rates")
    return t.value, tr.value, g.value


class Cache:
    """Owns the device arena (a torch tensor) and the handle; methods forward to the C calls."""

    def __init__(self, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, rope_mode: int,
                 rope_theta: float, mrope_sections=(0, 0, 0), n_streams: int = 1, capacity_tokens: int = 1024,
                 max_q_tokens: int = 256, device: str = "cuda:0", flags: int = 0):
        import torch
        self.cfg = SvConfig(n_layers, n_q_heads, n_kv_heads, head_dim, dtype, rope_mode, float(rope_theta),
                            (C.c_int32 * 3)(*mrope_sections), n_streams, capacity_tokens, max_q_tokens, flags)
        nbytes = sv_cache_bytes(self.cfg)
        if nbytes == 0:
            raise SvError(-1, "sv_cache_bytes")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.handle = sv_cache_create(self.cfg, self.arena)

    def close(self) -> None:
        if self.handle:
            sv_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, option: int, value: int) -> None:
        sv_cache_set_option(self.handle, option, value)

    def append(self, stream_id, layer, types, grid_thw, k, v) -> int:
        return sv_cache_append(self.handle, stream_id, layer, int(k.shape[0]), types, grid_thw, k, v)

    def evict(self, stream_id, n_sink, vision_window, text_window) -> int:
        return sv_cache_evict(self.handle, stream_id, n_sink, vision_window, text_window)

    def rope_apply(self, stream_id, slot0, n, q=None, k=None) -> None:
        sv_rope_apply(self.handle, stream_id, slot0, n, q, k)

    def attn_chunk(self, stream_id, layer, q, o, causal=True) -> None:
        sv_attn_chunk(self.handle, stream_id, layer, q, int(q.shape[0]), o, causal)

    def attn_decode(self, layer, stream_ids, q, o) -> None:
        sv_attn_decode(self.handle, layer, stream_ids, q, o)

    def attn_decode_static(self, layer, stream_ids, q, o) -> None:
        sv_attn_decode_static(self.handle, layer, stream_ids, q, o)

    def decode_step(self, layer, stream_ids, q, k, v, o) -> None:
        sv_decode_step(self.handle, layer, stream_ids, q, k, v, o)

    def decode_step_layers(self, stream_id, q, k, v, o) -> None:
        sv_decode_step_layers(self.handle, stream_id, q, k, v, o)

    def stream_step(self, stream_id, n_sink, vision_window, text_window, **tensors) -> int:
        return sv_stream_step(self.handle, stream_id, n_sink, vision_window, text_window, **tensors)

    def len(self, stream_id=0) -> int:
        return sv_cache_len(self.handle, stream_id)

    def retained(self, stream_id=0):
        return sv_cache_retained(self.handle, stream_id)

    def read_kv(self, stream_id, layer, which, slot0, n) -> np.ndarray:
        return sv_cache_read_kv(self.handle, stream_id, layer, which, slot0, n, self.cfg.n_kv_heads,
                                self.cfg.head_dim, self.cfg.dtype)
