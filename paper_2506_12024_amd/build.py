"""Builds libflexq.so (HIP, gfx950 only) in-tree with hipcc.

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is
installed.  Run as ``python -m paper_2506_12024_amd.build``.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libflexq.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["fq_api.hip", "fq_device.hip", "fq_noalloc.hip", "fq_probe.hip", "fq_quantize.hip", "fq_entropy.hip", "fq_decode.hip", "fq_staged.hip", "fq_skinny.hip", "fq_stream.hip", "fq_prefill.hip", "fq_w8a8.hip", "fq_sched.hip", "fq_lmhead.hip"]
HEADERS = [os.path.join(CSRC, "fq_internal.h"), os.path.join(CSRC, "fq_gemv.h"),
           os.path.join(os.path.dirname(HERE), "include", "flexq.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         # packed fp32 ops are kept off for device code (the host pass warns it does not know the feature)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str, force: bool) -> str:
    s = os.path.join(CSRC, src)
    o = os.path.join(OBJDIR, src + ".o")
    deps = [s] + HEADERS
    if force or not os.path.exists(o) or any(os.path.getmtime(d) > os.path.getmtime(o) for d in deps):
        subprocess.check_call(["hipcc"] + FLAGS + ["-c", s, "-o", o], stderr=subprocess.DEVNULL
                              if os.environ.get("FQ_QUIET") else None)
    return o


def build(force: bool = False) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
