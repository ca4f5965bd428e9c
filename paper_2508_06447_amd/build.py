"""Builds libslim.so (the method) and libslim_probe.so (bench.py's measurement probes) in-tree with hipcc for
gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libslim.so")
PROBE_LIB = os.path.join(HERE, "libslim_probe.so")
SOURCES = ("api.hip", "prune.hip", "norm_rope.hip", "gemm.hip", "attn.hip", "kvswap.hip", "decode.hip", "gemv.hip", "window.hip", "probe.hip")
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def build_lib(verbose: bool = True, extra_flags=()) -> str:
    """Compile every HIP source and link libslim.so; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        if verbose and out.strip():
            print(out)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    probe = [o for o in objs if os.path.basename(o) == "probe.o"]
    for lib, members in ((LIB, [o for o in objs if o not in probe]), (PROBE_LIB, probe)):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *members]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_lib()
    print("built", LIB)
    sys.exit(0)
