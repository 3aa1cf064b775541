"""Build the gfx950 shared library in-tree with hipcc.

    python -m paper_2411_08446_amd.build

Objects go to ``_build/`` at the repository root (git-ignored); the library
is written to ``paper_2411_08446_amd/lib/liblshmoe.so``.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB_DIR = os.path.join(PKG, "lib")
LIB_PATH = os.path.join(LIB_DIR, "liblshmoe.so")
PEAKS_LIB_PATH = os.path.join(LIB_DIR, "libpeaks.so")   # measured-peak probes of bench.py --peaks, not part of the path
BUILD_DIR = os.path.join(ROOT, "_build")

SOURCES = ["api.hip", "hash.hip", "group.hip", "centroid.hip", "restore.hip", "backward.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # the direct-to-LDS loads are inline assembly that sets M0 and says so in its clobber list
    "-Wno-inline-asm",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _compile(src: str) -> str:
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s\n%s" % (" ".join(cmd), res.stdout, res.stderr))
    warn = [l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    if warn:
        sys.stderr.write("\n".join(warn) + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed: %s\n%s\n%s" % (" ".join(cmd), res.stdout, res.stderr))
    peaks_obj = _compile("peaks.hip")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", peaks_obj, "-o", PEAKS_LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed: %s\n%s\n%s" % (" ".join(cmd), res.stdout, res.stderr))
    if verbose:
        print("built", LIB_PATH, "and", PEAKS_LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build()
