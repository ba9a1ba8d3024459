"""Builds the gfx950 HIP library in-tree with hipcc (no GPU needed to compile)."""
from __future__ import annotations

import os
import shutil
import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
LIB = PKG / "libresq_hip.so"

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources() -> list[Path]:
    return sorted(CSRC.glob("*.hip"))


def _hipcc() -> str:
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build(verbose: bool = False, extra_flags: list[str] | None = None) -> Path:
    """Compile every HIP source into ``libresq_hip.so`` (always recompiles)."""
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    cmd = [_hipcc(), *HIPCC_FLAGS, *(extra_flags or []), f"-I{ROOT / 'include'}", f"-I{CSRC}",
           "-o", str(tmp), *map(str, sources())]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{res.stdout}\n{res.stderr}")
    if verbose and res.stderr:
        print(res.stderr)
    os.replace(tmp, LIB)
    return LIB


def ensure_built() -> Path:
    """Return the library path, compiling if no library is there or a source is newer than it
    (where there is no compiler, e.g. a box that only runs what was built, a library that is
    there is used as it is)."""
    if not LIB.exists():
        build()
    else:
        newest = max(p.stat().st_mtime for p in [*CSRC.iterdir(), ROOT / "include" / "resq.h"])
        if newest > LIB.stat().st_mtime and shutil.which("hipcc"):
            build()
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
