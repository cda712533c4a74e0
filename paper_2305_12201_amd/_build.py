"""Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCE = os.path.join(_PKG, "csrc", "gravac.hip")
HOST_SOURCES = [os.path.join(_PKG, "csrc", "controller.cpp")]   # host-only parts of the same library
LIBRARY = os.path.join(_PKG, "libgravac.so")

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # acc = residual + grad stays one rounded add
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(force: bool = True) -> str:
    """Build ``libgravac.so`` in-tree.  With ``force=False`` only if it is missing or stale."""
    headers = [os.path.join(_ROOT, "include", h) for h in ("gravac.h", "gravac_profile.h", "gravac_controller.h")]
    if not force and os.path.exists(LIBRARY):
        newest = max(os.path.getmtime(f) for f in [SOURCE, *HOST_SOURCES, *headers])
        if os.path.getmtime(LIBRARY) >= newest:
            return LIBRARY
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(_ROOT, "include"), "-o", LIBRARY, SOURCE, *HOST_SOURCES]
    subprocess.run(cmd, check=True)
    return LIBRARY
