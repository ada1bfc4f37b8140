"""Build libdadam.so (gfx950) in-tree with hipcc.  Cross-compiles without a GPU.

    python -m paper_2410_11998_amd.build [--incremental] [extra hipcc flags]

Each translation unit is compiled to an object under _build/ (several at a time) and the objects
are linked into libdadam.so beside this file.  The tile and direct kernels are compiled in sixteen
parts from one source (csrc/dadam_kernels_part.hip: a pair of element types, with or without the
streaming hint, pointer tables in the argument block or in device memory).  build() recompiles everything; --incremental skips units whose object is newer
than the source and every header.
"""

from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdadam.so")

TYPES = {"f32": "TF32", "bf16": "TBF16"}
# (object name, source, extra definitions)
UNITS = [("dadam_host", "dadam_host.cpp", []), ("dadam_place", "dadam_place.cpp", []), ("dadam_kernels", "dadam_kernels.hip", [])]
for _x in ("f32", "bf16"):
    for _g in ("f32", "bf16"):
        for _nt in (True, False):
            for _ext in (False, True):
                _name = f"{_x}_{_g}" + ("_nt" if _nt else "") + ("_ext" if _ext else "")
                UNITS.append((f"dadam_kernels_part_{_name}", "dadam_kernels_part.hip",
                              [f"-DDADAM_PART_XT={TYPES[_x]}", f"-DDADAM_PART_GT={TYPES[_g]}",
                               f"-DDADAM_PART_NT={'true' if _nt else 'false'}",
                               f"-DDADAM_PART_EXT={'true' if _ext else 'false'}", f"-DDADAM_PART_NAME={_name}"]))

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


def jobs() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(n, 16, int(os.environ.get("MAX_JOBS", "16") or 16)))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = True, extra_flags=(), incremental: bool = False, lib: str = LIB) -> str:
    os.makedirs(OBJ, exist_ok=True)
    tag = "" if not extra_flags else "." + "".join(c if c.isalnum() else "_" for c in "".join(extra_flags))
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    objs, todo = [], []
    for name, source, defs in UNITS:
        src = os.path.join(CSRC, source)
        obj = os.path.join(OBJ, name + tag + ".o")
        objs.append(obj)
        newest = max(os.path.getmtime(p) for p in [src, __file__] + headers)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > newest:
            continue
        todo.append([hipcc()] + FLAGS + list(extra_flags) + defs + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=jobs()) as pool:
        list(pool.map(lambda cmd: _run(cmd, verbose), todo))
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib], verbose)
    return lib


if __name__ == "__main__":
    argv = sys.argv[1:]
    inc = "--incremental" in argv
    build(extra_flags=[a for a in argv if a != "--incremental"], incremental=inc)
