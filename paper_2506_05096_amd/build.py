"""Builds libastraea.so (HIP, gfx950 only) next to this file."""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
LIB = PKG / "libastraea.so"
OBJ = PKG / "_build"

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed fp32 VALU forms are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", str(ROOT / "include"), "-I", str(CSRC),
]


def sources():
    return sorted(CSRC.glob("*.hip"))


def _compile(src: Path) -> Path:
    obj = OBJ / (src.stem + ".o")
    subprocess.run([HIPCC, *FLAGS, "-c", str(src), "-o", str(obj)], check=True)
    return obj


def build(verbose: bool = True) -> Path:
    """Compile every .hip file and link the shared library.  Always rebuilds."""
    OBJ.mkdir(exist_ok=True)
    srcs = sources()
    with cf.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(LIB), *map(str, objs)], check=True)
    if verbose:
        print(f"built {LIB}")
    return LIB


def ensure_built() -> Path:
    """Build only when no library is present (tests, smoke and bench load what is there)."""
    if not LIB.exists():
        build()
    return LIB


if __name__ == "__main__":
    build()
