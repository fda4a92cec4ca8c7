"""Builds csrc/ into libspmv_mi355.so with hipcc for gfx950 (in-tree, no JIT cache)."""
from __future__ import annotations

import subprocess
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
LIB_PATH = PKG / "libspmv_mi355.so"
OBJ = PKG / "_build"   # objects only; never committed
SOURCES = [CSRC / "kernels.hip", CSRC / "spmm.hip", CSRC / "formats.hip", CSRC / "colblock.hip", CSRC / "twophase.hip", CSRC / "sell.hip", CSRC / "static_scratch.hip", CSRC / "capi.cpp", CSRC / "analysis.cpp"]
HEADERS = [CSRC / "kernels.h", CSRC / "device_common.h", CSRC / "row_phase.h", CSRC / "analysis.h", INCLUDE / "spmv_mi355.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # keep packed FP32 instructions out
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def is_stale() -> bool:
    if not LIB_PATH.exists():
        return True
    t = LIB_PATH.stat().st_mtime
    return any(p.stat().st_mtime > t for p in SOURCES + HEADERS)


def _run(cmd, verbose):
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the gfx feature name and says so once per file: harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if verbose or r.returncode != 0:
        print(" ".join(cmd))
        print(r.stdout + err)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)


def build(verbose: bool = False, incremental: bool = False) -> Path:
    """Compiles every source to an object of its own (in parallel) and links them.  incremental: sources older than
    their object and than every header are not compiled again (for work on one file; the default compiles all)."""
    OBJ.mkdir(exist_ok=True)
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    newest_header = max(p.stat().st_mtime for p in HEADERS)
    jobs = []
    for src in SOURCES:
        obj = OBJ / (src.name + ".o")
        if incremental and obj.exists() and obj.stat().st_mtime > max(src.stat().st_mtime, newest_header):
            continue
        jobs.append(["hipcc", *compile_flags, f"-I{INCLUDE}", f"-I{CSRC}", "-x", "hip", "-c", str(src), "-o", str(obj)])
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        for f in [pool.submit(_run, cmd, verbose) for cmd in jobs]:
            f.result()
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread",
          *[str(OBJ / (s.name + ".o")) for s in SOURCES], "-o", str(LIB_PATH)], verbose)
    return LIB_PATH


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv, incremental="-i" in sys.argv))
