"""Builds librapidgnn_hip.so (gfx950) in-tree with hipcc.

    python -m paper_2509_05207_amd.build
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "librapidgnn_hip.so")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + [os.path.join(ROOT, "include", "rapidgnn.h")]


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def stale_against(lib_path):
    t = os.path.getmtime(lib_path)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force=True, verbose=False, out=None, defines=()):
    """Builds the library; `out` and `defines` make another build of the same sources (the profiling build)."""
    if out is None and not force and not stale():
        return LIB
    out = out or LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",      # no packed-fp32 code generation
           "-Wall", "-Wno-unused-command-line-argument"] + ["-D" + d for d in defines] + [
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           "-o", out] + SOURCES
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    build(force=True, verbose=True)
    print("built", LIB)
