"""Build libpoetx.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpoetx.so")
LIMITS = os.path.join(PKG, "poetx_limits")          # measurement tool (csrc/diag/limits.hip)

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unused-value"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, *sources(), "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    # the measurement tool: machine ceilings next to the dense kernel and its feed-less variants
    tool = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
            "-packed-fp32-ops", "-Wno-unused-value", "-Wno-unused-result", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
            os.path.join(CSRC, "diag", "limits.hip"), "-o", LIMITS]
    if verbose:
        print(" ".join(tool), flush=True)
    r = subprocess.run(tool, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed (poetx_limits):\n" + "\n".join(l for l in r.stderr.splitlines() if noise not in l))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
