"""Compile the HIP sources under ``csrc/`` into ``libtdt_decode.so`` (gfx950 only)."""
from __future__ import annotations

import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libtdt_decode.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))


TIMERS_LIB = os.path.join(PKG, "libtdt_decode_timers.so")


def build_library(verbose: bool = False, defines=(), out: str = LIB) -> str:
    cmd = (["hipcc"] + HIPCC_FLAGS + [f"-D{d}" for d in defines] +
           ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc")] + sources() + ["-o", out])
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    return out


def build_timers_library(verbose: bool = False) -> str:
    """The profiling build: the decode kernel books wall-clock ticks per phase into the statistics."""
    return build_library(verbose, defines=("TDT_PHASE_TIMERS=1",), out=TIMERS_LIB)


if __name__ == "__main__":
    import sys
    if "--phase-timers" in sys.argv:
        print(build_timers_library(verbose=True))
    else:
        print(build_library(verbose=True))
