"""Build libosp.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libosp.so")
SOURCES = [os.path.join(CSRC, "osp_api.hip")]
HEADERS = [os.path.join(CSRC, h) for h in ("osp_stream_kernels.hpp", "osp_split_kernels.hpp",
                                            "osp_window_kernels.hpp", "osp_pack_kernels.hpp")]
HEADERS.append(os.path.join(os.path.dirname(HERE), "include", "osp.h"))

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # one rounding per fp32 operator: results must be bit-identical to a plain evaluation
    "-ffp-contract=off",
    # do not let the compiler form packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, extra_flags=()) -> str:
    if force or stale():
        cmd = [HIPCC, *FLAGS, *extra_flags, *SOURCES, "-o", LIB]
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
