"""Builds libsagekv.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsagekv.so")
SOURCES = ["api.hip", "score.hip", "select.hip", "prefilter.hip", "decode.hip"]
HEADERS = ["device_utils.h", "kernels.h", "radix_select.h", os.path.join("..", "..", "include", "sagekv.h"),
           os.path.join("..", "..", "include", "sagekv_bench.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every .hip source and link the shared library.  force=False rebuilds only when a
    source or header is newer than the library."""
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = ["hipcc", *FLAGS, *os.environ.get("SAGEKV_EXTRA_HIPCC_FLAGS", "").split(), "-c",
               os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB])
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
