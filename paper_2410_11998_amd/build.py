"""Build libdadam.so (gfx950) in-tree with hipcc.  Cross-compiles without a GPU.

    python -m paper_2410_11998_amd.build [--incremental] [extra hipcc flags]

Each source is compiled to an object under _build/ and the objects are linked into
libdadam.so beside this file.  build() recompiles everything; --incremental skips sources whose
object is newer than the source and every header.
"""

from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdadam.so")

SOURCES = ["dadam_kernels.hip", "dadam_host.cpp"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-x", "hip",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = True, extra_flags=(), incremental: bool = False, lib: str = LIB) -> str:
    os.makedirs(OBJ, exist_ok=True)
    tag = "" if not extra_flags else "." + "".join(c if c.isalnum() else "_" for c in "".join(extra_flags))
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    objs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, s + tag + ".o")
        objs.append(obj)
        newest = max(os.path.getmtime(p) for p in [src, __file__] + headers)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > newest:
            continue
        _run([hipcc()] + FLAGS + list(extra_flags) + ["-c", src, "-o", obj], verbose)
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib], verbose)
    return lib


if __name__ == "__main__":
    argv = sys.argv[1:]
    inc = "--incremental" in argv
    build(extra_flags=[a for a in argv if a != "--incremental"], incremental=inc)
