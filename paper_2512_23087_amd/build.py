"""Build the gfx950 shared library from csrc/ with hipcc (in-tree, no JIT cache).

    python -m paper_2512_23087_amd.build            # rebuild everything
    python -m paper_2512_23087_amd.build --changed  # only the sources newer than their objects
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
SOURCES = ["dvp_api.hip", "dvp_rows.hip", "dvp_lmhead.hip", "dvp_lmhead_lists.hip", "dvp_sequences.hip", "dvp_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _compile(src: str) -> Path:
    obj = OBJ / (src + ".o")
    subprocess.check_call([HIPCC, *FLAGS, "-c", str(CSRC / src), "-o", str(obj)])
    return obj


def _stale(src: str) -> bool:
    """An object is up to date when it is newer than its source and every header."""
    obj = OBJ / (src + ".o")
    if not obj.exists():
        return True
    deps = [CSRC / src, *CSRC.glob("*.h"), *(PKG.parent / "include").glob("*.h")]
    return any(d.stat().st_mtime > obj.stat().st_mtime for d in deps)


def build(verbose: bool = True, only_changed: bool = False) -> Path:
    """Compile every source for gfx950 (or, with only_changed, the stale ones) and link
    libdvp_hip.so next to this file."""
    OBJ.mkdir(exist_ok=True)
    todo = [s for s in SOURCES if not only_changed or _stale(s)]
    with ThreadPoolExecutor(max_workers=min(6, max(1, len(todo)))) as ex:
        list(ex.map(_compile, todo))
    objs = [OBJ / (s + ".o") for s in SOURCES]
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc",
                           "-o", str(tmp), *map(str, objs)])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(only_changed="--changed" in sys.argv[1:])
    sys.exit(0)
