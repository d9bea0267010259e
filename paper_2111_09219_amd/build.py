"""Compiles the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libjpgd.so")
SOURCES = ["jpgd.hip", "jpgd_parse.cpp"]
HEADERS = ["jpgd_common.h", "jpgd_idct.h", "jpgd_kernels.h", "jpgd_lane.h", "jpgd_lut.h", "../../include/jpgd.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True) -> str:
    """Build libjpgd.so; with force=False only if it is missing or older than one of its sources (and a compiler
    is at hand: a box without hipcc runs what was built)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not force and os.path.exists(LIB) and (not stale() or not os.path.exists(hipcc)):
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass reports that it does not know the packed-fp32 feature; that is expected
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
