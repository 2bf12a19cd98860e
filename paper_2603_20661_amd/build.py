"""Builds libwww.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2603_20661_amd.build` rebuilds."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libwww.so")
SOURCES = ["api.hip", "pack.hip", "decode.hip", "prefill.hip", "duel.hip", "sample.hip", "probe.hip", "sched.cpp", "ledger.cpp"]   # the .cpp files are host-only C++
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Wno-inline-asm",   # the LDS-copy assembly names M0 as clobbered, which clang reports as a reserved register
         "-fvisibility=hidden", "-fvisibility-inlines-hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    flags = FLAGS if src.endswith(".hip") else ["-O2", "-std=c++17", "-fPIC", "-Wall", "-fvisibility=hidden", "-fvisibility-inlines-hidden"]
    cmd = [HIPCC, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        print(err, file=sys.stderr)
    return obj


def build_library(force: bool = True) -> str:
    """Compile every HIP source for gfx950 and link the shared library."""
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp", ".h"))] + \
           [os.path.join(os.path.dirname(HERE), "include", "www.h")]
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in deps):
        return LIB
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-Bsymbolic", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build_library(True))
