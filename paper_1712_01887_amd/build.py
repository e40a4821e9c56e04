"""Compile libdgc.so (HIP, gfx950) next to this file.

    python -m paper_1712_01887_amd.build

hipcc cross-compiles without a GPU.  Flags that matter for correctness:
-ffp-contract=off keeps every binary32 operation separately rounded, and the
packed-FP32 instructions are switched off for the device pass.
"""

from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libdgc.so")
SOURCES = [os.path.join(HERE, "csrc", name) for name in
           ("dgc_api.hip", "dgc_compress.hip", "dgc_receive.hip", "dgc_wire.hip")]
HEADERS = [os.path.join(HERE, "csrc", "dgc_internal.h"), os.path.join(ROOT, "include", "dgc.h")]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def command(out: str = LIB_PATH) -> list:
    return [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            "-ffp-contract=off", "-fno-gpu-flush-denormals-to-zero",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-command-line-argument",
            "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
            *SOURCES, "-o", out]


def build_library(verbose: bool = True) -> str:
    cmd = command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    build_library()
    sys.exit(0)
