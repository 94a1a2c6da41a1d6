"""Compile the HIP library for gfx950 into paper_2503_17911_amd/lib/ (in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
LIBDIR = PKG / "lib"
LIB = LIBDIR / "libann_gfx950.so"
SOURCES = ["host.hip", "sq.hip", "search.hip", "search_fast.hip", "search_general.hip", "search_fast_wide.hip", "search_general_wide.hip", "rerank.hip", "bruteforce.hip", "entry.hip", "schedule.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -ffp-contract=off: roundings are part of the results that must match a
# reference bit for bit; fused multiply-adds are written explicitly (fmaf).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-I", str(INCLUDE), "-I", str(CSRC),
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> Path:
    obj = LIBDIR / (src + ".o")
    cmd = [HIPCC, *FLAGS, "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        print(err, file=sys.stderr)
    return obj


def build(verbose: bool = True, only=None) -> Path:
    """Compile every source (or, for quick iterations, only those named in
    `only`, reusing the other object files) and link the library."""
    LIBDIR.mkdir(exist_ok=True)
    todo = [s for s in SOURCES if only is None or s in only or not (LIBDIR / (s + ".o")).exists()]
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as ex:
        list(ex.map(_compile, todo))
    objs = [LIBDIR / (s + ".o") for s in SOURCES]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *map(str, objs), "-o", str(LIB)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build(only=sys.argv[1:] or None)
