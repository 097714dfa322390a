"""The C-ABI library builds, loads, and exports every function include/sv.h declares (no GPU needed)."""
import ctypes
import os
import re

import paper_2510_09608_amd as sv
from paper_2510_09608_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            names += re.findall(r"SV_API\s+[\w\s\*]+?\b(sv_\w+)\s*\(", open(os.path.join(inc, fn)).read())
    return names


def _lib():
    if not os.path.exists(sv.lib_path()):
        build.build(verbose=False)
    return ctypes.CDLL(sv.lib_path())


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert len(names) == 18 and "sv_cache_evict" in names and "sv_attn_decode" in names
    lib = _lib()
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.exported_names())     # the Python binding covers the same calls


def test_host_only_calls():
    """Calls that never touch the device: status text, arena sizing and configuration checks."""
    lib = _lib()
    lib.sv_strerror.restype = ctypes.c_char_p
    assert lib.sv_strerror(0) == b"ok" and b"capacity" in lib.sv_strerror(-2)
    lib.sv_cache_bytes.restype = ctypes.c_size_t
    lib.sv_cache_bytes.argtypes = [ctypes.POINTER(sv.SvConfig)]

    def cfg(**kw):
        base = dict(n_layers=28, n_q_heads=28, n_kv_heads=4, head_dim=128, dtype=1, rope_mode=1, rope_theta=1e6,
                    mrope_sections=(16, 24, 24), n_streams=1, capacity_tokens=5632, max_q_tokens=256)
        base.update(kw)
        base["mrope_sections"] = (ctypes.c_int32 * 3)(*base["mrope_sections"])
        return sv.SvConfig(**base)

    n = lib.sv_cache_bytes(ctypes.byref(cfg()))
    kv = 2 * 28 * 2 * 4 * 5632 * 128 * 2              # both ping-pong halves of K and V, all layers
    assert kv < n < kv + (96 << 20)
    assert lib.sv_cache_bytes(ctypes.byref(cfg(capacity_tokens=2 * 5632))) > 2 * kv
    for bad in (dict(n_q_heads=30), dict(head_dim=96), dict(mrope_sections=(16, 24, 23)), dict(n_layers=0),
                dict(dtype=3), dict(rope_mode=5), dict(capacity_tokens=0), dict(max_q_tokens=0), dict(rope_theta=0.0)):
        assert lib.sv_cache_bytes(ctypes.byref(cfg(**bad))) == 0, bad
    assert lib.sv_cache_bytes(None) == 0
    # a NULL handle is refused, not dereferenced
    lib.sv_cache_len.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    out = ctypes.c_int64(0)
    assert lib.sv_cache_len(None, 0, ctypes.byref(out)) == -1
    assert lib.sv_cache_destroy(None) == -1


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: any other --gpus exits with a message before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
