"""Build libts.so (the HIP C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libts.so")
SOURCES = ["ts_runtime.hip", "ts_kmap.hip", "ts_conv.hip", "ts_elementwise.hip"]
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-result",
    # packed fp32 math is kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "ts_internal.h"), os.path.join(HERE, "..", "include", "ts.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile the library; returns the path of the shared object."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + sources() + ["-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libts.so")
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
