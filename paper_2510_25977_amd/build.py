"""Build the svdmlp shared library (hipcc, gfx950 only) in-tree.

    python -m paper_2510_25977_amd.build [--force]

The library is built next to this file as ``libsvdmlp.so`` so that it travels with the source
tree; tests, ``bench.py`` and ``__graft_entry__.smoke()`` load that file and never compile.
"""
from __future__ import annotations

import os
import re
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


_MEM_OP = re.compile(r"^(global_load_lds_\w+|global_store_\w+|global_load_\w+|global_atomic_\w+)\b(.*)$")
_SGPR_PAIR = re.compile(r"\bs\[(\d+):(\d+)\]")
_VALU_TO_SGPR = re.compile(r"^(v_readlane_b32|v_readfirstlane_b32)\s+s(\d+)\b")
_NOP = re.compile(r"^s_nop\s+(\d+)")
SGPR_TO_VMEM_WAIT_STATES = 5


def check_sgpr_hazards(asm: str) -> list:
    """Scan generated gfx950 assembly for a hazard the compiler cannot see: a vector-memory instruction INSIDE an
    inline-asm statement whose SGPR base address was written by a vector instruction (v_readfirstlane, or v_readlane
    when a spilled SGPR is restored) fewer than five wait states earlier.  The compiler inserts those wait states for
    instructions of its own, but an asm statement is opaque to it.  Returns one message per finding."""
    insts = []          # (text, inside_asm)
    inside = False
    for raw in asm.splitlines():
        line = raw.split(";")[0].strip() if not raw.strip().startswith(";;#ASM") else raw.strip()
        if line.startswith(";;#ASMSTART"):
            inside = True
            continue
        if line.startswith(";;#ASMEND"):
            inside = False
            continue
        if not line or line.startswith(".") or line.endswith(":"):
            continue
        insts.append((line, inside))
    found = []
    for i, (line, in_asm) in enumerate(insts):
        m = _MEM_OP.match(line)
        if not (in_asm and m):
            continue
        base = set()
        for a, b in _SGPR_PAIR.findall(m.group(2)):
            base.update(range(int(a), int(b) + 1))
        states, j = 0, i - 1
        while j >= 0 and states < SGPR_TO_VMEM_WAIT_STATES:
            prev = insts[j][0]
            w = _VALU_TO_SGPR.match(prev)
            if w and int(w.group(2)) in base:
                found.append(f"'{prev}' only {states} wait state(s) before '{line}'")
                break
            n = _NOP.match(prev)
            states += int(n.group(1)) + 1 if n else 1
            j -= 1
    return found


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

    def hazards_of(src: Path) -> list:
        asm = OBJDIR / (src.stem + ".s")
        res = subprocess.run([HIPCC, *FLAGS, "-S", "--cuda-device-only", str(src), "-o", str(asm)], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc -S failed on {src.name}:\n{res.stderr[-2000:]}")
        found = check_sgpr_hazards(asm.read_text())
        asm.unlink()
        return [f"{src.name}: {f}" for f in found]

    # sources with hand-written memory instructions that take an SGPR base: their generated assembly is checked
    asm_srcs = [s for s in srcs if re.search(r'asm volatile\("[^;]*global_(load|store)', s.read_text())]
    with ThreadPoolExecutor(max_workers=min(8, len(srcs) + len(asm_srcs))) as ex:
        hz = [ex.submit(hazards_of, s) for s in asm_srcs]
        objs = list(ex.map(compile_one, srcs))
        hazards = [f for h in hz for f in h.result()]
    if hazards:
        raise RuntimeError("SGPR-to-memory-address hazard inside inline asm (see check_sgpr_hazards):\n" + "\n".join(hazards))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(LIB), *map(str, objs)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    return LIB


if __name__ == "__main__":
    path = build(force=True, verbose=True)
    print(path)
