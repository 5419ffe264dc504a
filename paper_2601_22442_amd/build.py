"""Builds libasyncmesh.so (the C-ABI HIP library) in-tree for gfx950 with hipcc.

A digest of the library's source files is compiled into the library (am_version() ends with
"src:<digest>"); `source_hash()` recomputes it from the files, so that tests, the smoke check and
the benchmark can refuse a library that was not built from the sources beside it."""
from __future__ import annotations

import hashlib
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
SRC = PKG / "csrc" / "asyncmesh.hip"
DEPS = [SRC, PKG / "csrc" / "am_kernels.h", PKG / "csrc" / "am_device.h", PKG / "csrc" / "am_geometry.h",
        PKG / "csrc" / "am_host_logic.h", PKG.parent / "include" / "asyncmesh.h"]
LIB = PKG / "libasyncmesh.so"

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def source_hash() -> str:
    """First 16 hex digits of the SHA-256 over the library's source files (names and contents)."""
    h = hashlib.sha256()
    for f in sorted(DEPS, key=lambda q: q.name):
        h.update(f.name.encode())
        h.update(b"\0")
        h.update(f.read_bytes())
        h.update(b"\0")
    return h.hexdigest()[:16]


def stale() -> bool:
    return not LIB.exists() or any(LIB.stat().st_mtime < d.stat().st_mtime for d in DEPS)


def build_library(force: bool = True, verbose: bool = False) -> Path:
    if force or stale():
        cmd = ["hipcc", *HIPCC_FLAGS, f'-DAM_SOURCE_HASH="{source_hash()}"', "-o", str(LIB), str(SRC)]
        if verbose:
            cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
        subprocess.run(cmd, check=True)
    return LIB


def check_library_is_current(version: str) -> str:
    """Raise unless `version` (what am_version() of the loaded library says) carries the digest of
    the source files beside it; returns the digest."""
    want = source_hash()
    if not version.endswith("src:" + want):
        raise RuntimeError(f"libasyncmesh.so is stale: it says '{version}', the sources hash to {want}; "
                           "rebuild it (python -m paper_2601_22442_amd.build)")
    return want


if __name__ == "__main__":
    print(build_library(force=True, verbose="-v" in sys.argv))
