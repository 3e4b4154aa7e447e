"""Builds libhttm.so (the HIP kernels + C ABI) and libhttm_probe.so (bench.py's MFMA ceiling probe) for
gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libhttm.so")
PROBE_LIB_PATH = os.path.join(PKG_DIR, "libhttm_probe.so")   # measurement helper of bench.py, not the product
PROBE_SOURCES = ["mfma_probe.hip"]

SOURCES = ["api.hip", "geometry.cpp", "reorder_unmerge.hip", "match_merge.hip", "match_merge_big.hip", "outlier_filter.hip",
           "attention.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU ops
    "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP extension cannot be built")


def _compile(sources, target, verbose, extra_flags):
    srcs = []
    for s in sources:
        srcs += ["-x", "hip", os.path.join(CSRC, s)]
    tmp = target + ".tmp"
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, *srcs, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose:
        noise = "is not a recognized feature for this target"
        print("\n".join(l for l in res.stdout.splitlines() if noise not in l), flush=True)
    os.replace(tmp, target)


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source into paper_2511_21317_amd/libhttm.so (and the probe into libhttm_probe.so)
    and return the library's path."""
    _compile(SOURCES, LIB_PATH, verbose, extra_flags)
    _compile(PROBE_SOURCES, PROBE_LIB_PATH, verbose, extra_flags)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
