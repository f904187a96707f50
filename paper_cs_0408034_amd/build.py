"""Builds libplogp.so (the C-ABI HIP library) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libplogp.so"
SOURCES = [CSRC / "plogp_api.hip", CSRC / "plogp_kernels.hip", CSRC / "plogp_cutover.hip",
           CSRC / "plogp_robust.hip", CSRC / "plogp_profile.hip"]
HEADERS = [CSRC / "plogp_internal.hpp", CSRC / "plogp_handles.hpp", PKG.parent / "include" / "plogp.h",
           PKG.parent / "include" / "plogp_profile.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # the decision table must be reproducible bit for bit: no contraction, fma only where written
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build_library(force: bool = True, verbose: bool = False) -> Path:
    """Compile the library.  With force=False, only if it is missing or older
    than a source."""
    if not force and LIB.exists():
        newest = max(p.stat().st_mtime for p in SOURCES + HEADERS)
        if LIB.stat().st_mtime >= newest:
            return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", str(tmp)] + [str(s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
