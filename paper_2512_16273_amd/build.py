"""Builds the C-ABI library `libtslt.so` for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libtslt.so")
SOURCES = [os.path.join(HERE, "csrc", "tslt.hip")]
HEADERS = [os.path.join(HERE, "csrc", n) for n in ("common.h", "truncate.h", "sample.h", "verify.h", "rowops.h", "exp64.h", "tree.h", "wire.h", "stats.h", "calib.h")] + \
          [os.path.join(ROOT, "include", "tslt.h")]


def hipcc_command(out: str = LIB_PATH) -> list:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
            # packed-fp32 instructions are kept out of the generated code
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-function",
            "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
            "-o", out] + SOURCES


def build_library(verbose: bool = True) -> str:
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.exists(s) and os.path.getmtime(s) > t for s in SOURCES + HEADERS)


if __name__ == "__main__":
    build_library()
    print(LIB_PATH)
    sys.exit(0)
