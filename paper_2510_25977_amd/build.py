"""Build the svdmlp shared library (hipcc, gfx950 only) in-tree.

    python -m paper_2510_25977_amd.build [--force]

The library is built next to this file as ``libsvdmlp.so`` so that it travels with the source
tree; tests, ``bench.py`` and ``__graft_entry__.smoke()`` load that file and never compile.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libsvdmlp.so"
OBJDIR = HERE / "_build"

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # no packed-fp32 instructions (v_pk_*_f32) in generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(CSRC.glob("*.hip"))


def build(force: bool = True, verbose: bool = False) -> Path:
    """Compile every HIP source and link ``libsvdmlp.so``.  Always recompiles unless force=False and
    the library is newer than every source."""
    srcs = sources()
    deps = srcs + sorted(CSRC.glob("*.h")) + [HERE.parent / "include" / "svdmlp.h"]
    if not force and LIB.exists() and all(LIB.stat().st_mtime >= s.stat().st_mtime for s in deps):
        return LIB
    OBJDIR.mkdir(exist_ok=True)

    def compile_one(src: Path) -> Path:
        obj = OBJDIR / (src.stem + ".o")
        cmd = [HIPCC, *FLAGS, "-c", str(src), "-o", str(obj)]
        res = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src.name}:\n{out}")
        if verbose and out.strip():
            print(out)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(compile_one, srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(LIB), *map(str, objs)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    return LIB


if __name__ == "__main__":
    path = build(force=True, verbose=True)
    print(path)
