"""Build libsv.so (HIP, gfx950 only) next to this file.  Usage: python -m paper_2510_09608_amd.build"""
from __future__ import annotations

import concurrent.futures as cf
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libsv.so")
OBJDIR = os.path.join(ROOT, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
    # the first 16 dwords of a kernel's arguments arrive in SGPRs with the wavefront instead of being fetched by
    # its first instructions: the launch-latency-bound decode kernels start their memory round trip earlier
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function",
]


OUT_TIMELINE = os.path.join(HERE, "libsv_timeline.so")   # measurement build: decode kernels stamp a timeline


def _compile(src: str, extra=(), tag: str = "") -> str:
    obj = os.path.join(OBJDIR, os.path.basename(src) + tag + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def _link(out: str, objs) -> None:
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)


def build(verbose: bool = True) -> str:
    """libsv.so (the product) and libsv_timeline.so (the same sources with -DSV_TIMELINE: only bench.py's
    decode_timeline workload loads it)."""
    os.makedirs(OBJDIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with cf.ThreadPoolExecutor(max_workers=min(8, len(srcs) + 1)) as ex:
        objs = list(ex.map(_compile, srcs))
        dec = [s for s in srcs if s.endswith("sv_attn_decode.hip")][0]
        dec_tl = ex.submit(_compile, dec, ("-DSV_TIMELINE",), ".timeline").result()
    _link(OUT, objs)
    _link(OUT_TIMELINE, [dec_tl if o.endswith("sv_attn_decode.hip.o") else o for o in objs])
    if verbose:
        print(f"built {OUT} and {OUT_TIMELINE} from {len(srcs)} sources")
    return OUT


if __name__ == "__main__":
    build()
