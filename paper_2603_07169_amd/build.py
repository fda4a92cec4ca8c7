"""Builds csrc/ into libspmv_mi355.so with hipcc for gfx950 (in-tree, no JIT cache)."""
from __future__ import annotations

import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
LIB_PATH = PKG / "libspmv_mi355.so"
SOURCES = [CSRC / "kernels.hip", CSRC / "spmm.hip", CSRC / "formats.hip", CSRC / "colblock.hip", CSRC / "twophase.hip", CSRC / "capi.cpp", CSRC / "analysis.cpp"]
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


def build(verbose: bool = False) -> Path:
    cmd = ["hipcc", *HIPCC_FLAGS, f"-I{INCLUDE}", f"-I{CSRC}", "-x", "hip",
           *[str(s) for s in SOURCES], "-o", str(LIB_PATH)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the gfx feature name and says so once per file: harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if verbose or r.returncode != 0:
        print(" ".join(cmd))
        print(r.stdout + err)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
