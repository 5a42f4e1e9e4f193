"""Builds librgc.so (the gfx950 HIP library behind include/rgc.h) in-tree with hipcc.

Build-time hooks (the library itself reads no environment variable): HIPCC names another compiler driver;
RGC_EXTRA_FLAGS appends flags for tuning experiments, e.g. -DRGC_CHUNK=4096 (wave-chunk size).
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librgc.so")
SOURCES = ["rgc_api.cpp", "rgc_compress.hip", "rgc_decompress.hip", "rgc_threshold.hip", "rgc_yardstick.hip"]
HEADERS = ["rgc_internal.h", "rgc_device.h", "rgc_exact.h", os.path.join("..", "..", "include", "rgc.h"),
           os.path.join("..", "..", "include", "rgc_diag.h")]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-ffp-contract=off",                       # the oracle is built the same way: no silent fma
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    for f in SOURCES + HEADERS:
        if os.path.getmtime(os.path.join(CSRC, f)) > t:
            return True
    return False


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not needs_build():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("RGC_EXTRA_FLAGS", "").split()      # tuning experiments only
    cmd = [hipcc] + FLAGS + extra + ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l)   # the host pass does not know the device feature
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print("built", LIB)
    sys.exit(0)
