"""Build libtir.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

``python -m paper_2207_04296_amd.buildlib`` compiles every translation unit (in parallel) and
links ``paper_2207_04296_amd/libtir.so``.  Nothing is compiled at import time or inside tests.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
OBJ = PKG / "_build"
LIB = PKG / "libtir.so"
N_UNITS = 6

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-but-set-variable",
         "-Wno-unused-variable", "-Wno-unused-local-typedef", "-Wno-inline-asm",
         # packed fp32 instructions are kept off for every kernel of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         f"-I{INCLUDE}", f"-I{CSRC}"]


ALLOW_SCRATCH = False      # instrumented experiment builds may set this; the product build never does


def _compile(args):
    """Compile one unit.  The compiler reports every kernel's register and scratch use (-Rpass-analysis): a kernel
    that spills to scratch memory fails the build - a spill in a cold branch still makes every launch of the kernel
    carry a scratch allocation, and one in a main loop costs far more than the tile shape it came with can gain."""
    src, obj, extra = args
    cmd = [HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", *extra, "-c", str(src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    lines = r.stderr.splitlines()
    if r.returncode != 0:
        err = "\n".join(l for l in lines if "packed-fp32-ops" not in l and "remark:" not in l)
        raise RuntimeError(f"hipcc failed: {' '.join(cmd)}\n{err}")
    spilling, name = [], "?"
    for l in lines:
        if "remark: Function Name:" in l:
            name = l.split("Function Name:")[1].split("[-Rpass")[0].strip()
        elif "ScratchSize [bytes/lane]:" in l:
            n = int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if n > 0:
                spilling.append(f"{name}: {n} bytes of scratch per lane")
    if spilling and not ALLOW_SCRATCH:
        raise RuntimeError(f"{src.name} {' '.join(extra)}: kernels spill registers to scratch memory:\n  " + "\n  ".join(sorted(set(spilling))))
    # what is left to show: real warnings (the remarks and their source excerpts are dropped)
    keep, skip = [], 0
    for l in lines:
        if "remark:" in l:
            skip = 2            # the remark's source line and caret line follow
            continue
        if skip and (l.lstrip().startswith(("|", "^")) or "|" in l[:8]):
            skip -= 1
            continue
        skip = 0
        if "packed-fp32-ops" not in l and not l.startswith("In file included from") and "remarks generated" not in l:
            keep.append(l)
    return "\n".join(keep)


def sources():
    return sorted(CSRC.glob("*.hip")) + sorted(CSRC.glob("*.h")) + sorted(CSRC.glob("*.def")) + [INCLUDE / "tir.h"]


def is_stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    return any(s.stat().st_mtime > t for s in sources())


def build(verbose: bool = True, jobs: int | None = None, defines=(), lib: Path = LIB, tag: str = "") -> Path:
    """Compile and link.  `defines`, `lib` and `tag` let experiments build instrumented copies
    (extra -D flags, another output name) without touching the product library."""
    OBJ.mkdir(exist_ok=True)
    extra = [f"-D{d}" for d in defines]
    jobs_list = [(CSRC / "tir_api.hip", OBJ / f"tir_api{tag}.o", extra),
                 (CSRC / "tir_attn.hip", OBJ / f"tir_attn{tag}.o", extra)]
    for u in range(N_UNITS):
        jobs_list.append((CSRC / "tir_inst.hip", OBJ / f"tir_inst{u}{tag}.o", [f"-DTIR_UNIT={u}"] + extra))
    with ThreadPoolExecutor(max_workers=jobs or min(8, os.cpu_count() or 1)) as ex:
        for warn in ex.map(_compile, jobs_list):
            if verbose and warn.strip():
                print(warn, file=sys.stderr)
    objs = [str(j[1]) for j in jobs_list]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(lib), *objs]
    subprocess.run(cmd, check=True)
    if verbose:
        print(f"built {lib}")
    return lib


if __name__ == "__main__":
    build()
