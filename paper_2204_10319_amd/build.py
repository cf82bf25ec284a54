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


OBJDIR = os.path.join(HERE, "_build")


def _object_stale(src: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    deps = [src, os.path.join(CSRC, "ts_internal.h"), os.path.join(HERE, "..", "include", "ts.h"),
            os.path.join(HERE, "..", "include", "ts_bench.h")]
    return any(os.path.exists(d) and os.path.getmtime(d) > t for d in deps)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile the library (one object per source, side by side, then one link); returns the path of the
    shared object.  With force every source is compiled again, otherwise only those older than what they
    include."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    jobs, objs = [], []
    for src in sources():
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
        objs.append(obj)
        if force or _object_stale(src, obj):
            jobs.append((src, subprocess.Popen([hipcc] + compile_flags + ["-c", src, "-o", obj],
                                               stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, proc in jobs:
        out, _ = proc.communicate()
        if verbose or proc.returncode != 0:
            print(out)
        if proc.returncode != 0:
            failed = True
            try:
                os.remove(os.path.join(OBJDIR, os.path.basename(src) + ".o"))
            except OSError:
                pass
    if failed:
        raise RuntimeError("hipcc failed building libts.so")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared"] + objs + ["-o", LIB],
                         capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed linking libts.so")
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
