"""Build the gfx950 shared library from csrc/ with hipcc (in-tree, no JIT cache).

    python -m paper_2512_23087_amd.build          # rebuild everything
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
OBJ = PKG / "_build"
LIB = PKG / "libdvp_hip.so"
SOURCES = ["dvp_api.hip", "dvp_rows.hip", "dvp_lmhead.hip", "dvp_lmhead_lists.hip", "dvp_sequences.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _compile(src: str) -> Path:
    obj = OBJ / (src + ".o")
    subprocess.check_call([HIPCC, *FLAGS, "-c", str(CSRC / src), "-o", str(obj)])
    return obj


def build(verbose: bool = True) -> Path:
    """Compile every source for gfx950 and link libdvp_hip.so next to this file."""
    OBJ.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(5, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc",
                           "-o", str(tmp), *map(str, objs)])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
