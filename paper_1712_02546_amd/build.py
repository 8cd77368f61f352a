"""Builds libconvslice.so (the C-ABI library of include/*.h) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libconvslice.so")
SOURCES = [os.path.join(CSRC, n) for n in ("convslice_api.hip", "convlayer_api.hip", "netlayers.hip")]
HEADERS = sorted(os.path.join(CSRC, n) for n in os.listdir(CSRC) if n.endswith(".h")) + [
    os.path.join(os.path.dirname(HERE), "include", n) for n in ("convslice.h", "convlayer.h", "convnet.h")]

# packed-fp32 VALU forms are switched off for all device code on purpose.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, extra_flags: list[str] | None = None) -> str:
    """Compile the library in-tree; returns its path."""
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        cmd = [hipcc] + HIPCC_FLAGS + (extra_flags or []) + ["-o", LIB] + SOURCES
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True, extra_flags=sys.argv[1:]))
