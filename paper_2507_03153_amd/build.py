"""Compiles the HIP library (libhgca.so) for gfx950 with hipcc, in-tree.

    python -m paper_2507_03153_amd.build [--force]
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libhgca.so")
SOURCES = ["hgca_api.hip", "attn_kernels.hip", "select_kernels.hip", "maw_kernels.hip", "cache_kernels.hip", "append_kernels.hip", "group_kernels.hip", "fused_kernels.hip"]
HEADERS = ["hgca_device.hpp", "hgca_launch.hpp", "threshold_compact.hpp", "row_map.hpp", "attn_device.hpp", "fold_device.hpp", "select_device.hpp", os.path.join("..", "..", "include", "hgca.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-FP32 instructions stay off (they are not written by hand either)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and up_to_date():
        return LIB
    cmd = [hipcc(), *FLAGS, "-o", LIB] + [os.path.join(CSRC, f) for f in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv or True, verbose=True))
