"""Builds libasynclm.so in-tree with hipcc for gfx950 (no torch dependency in the library)."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libasynclm.so")
ROOT = os.path.dirname(HERE)
PROBE_SRC = os.path.join(ROOT, "traffic_probe.hip")   # stand-alone C-ABI consumer for hardware-counter runs (beside bench.py)
PROBE = os.path.join(ROOT, "traffic_probe")
SOURCES = ["api.hip", "decode_kernels.hip", "decode_fused.hip", "chunk_kernels.hip"]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = False) -> str:
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-I", os.path.join(os.path.dirname(HERE), "include"),
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed")
    return LIB


def build_probe(verbose: bool = False) -> str:
    """Builds the counter-run program against the in-tree library.  Not part of the library build: measurement only."""
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wno-unused-command-line-argument",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", ROOT,
           PROBE_SRC, "-o", PROBE, "-L", HERE, "-lasynclm", "-Wl,-rpath," + HERE]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed (traffic_probe)")
    return PROBE


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True))
    if "--probe" in sys.argv[1:]:
        print(build_probe(verbose=True))
