"""Builds libasyncmesh.so (the C-ABI HIP library) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
SRC = PKG / "csrc" / "asyncmesh.hip"
DEPS = [SRC, PKG / "csrc" / "am_kernels.h", PKG / "csrc" / "am_device.h", PKG.parent / "include" / "asyncmesh.h"]
LIB = PKG / "libasyncmesh.so"

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


PROBE_SRC = PKG / "csrc" / "hbm_copy_probe.hip"
PROBE = PKG / "hbm_copy_probe"


def build_probe() -> Path:
    """The plain-copy yardstick program (used only when profiling)."""
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    subprocess.run(["hipcc", *flags, "-o", str(PROBE), str(PROBE_SRC)], check=True)
    return PROBE


def stale() -> bool:
    return not LIB.exists() or any(LIB.stat().st_mtime < d.stat().st_mtime for d in DEPS)


def build_library(force: bool = True, verbose: bool = False) -> Path:
    if force or stale():
        cmd = ["hipcc", *HIPCC_FLAGS, "-o", str(LIB), str(SRC)]
        if verbose:
            cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose="-v" in sys.argv))
    print(build_probe())
