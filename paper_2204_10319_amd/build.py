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


SAN_LIB = os.path.join(OBJDIR, "libts_hostsan.so")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-omit-frame-pointer", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def build_host_sanitized(force: bool = False) -> str:
    """The same library with its HOST code compiled under AddressSanitizer and UndefinedBehaviorSanitizer
    (device code as usual): for the host-side checks of tests/host/host_checks.cpp, which need no GPU.
    Goes to _build/, never next to the product library."""
    os.makedirs(OBJDIR, exist_ok=True)
    if not force and os.path.exists(SAN_LIB) and not any(_object_stale(src, SAN_LIB) for src in sources()):
        return SAN_LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f not in ("-O3", "-shared")] + ["-O1", "-g"] + SAN_FLAGS
    jobs, objs = [], []
    for src in sources():
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".san.o")
        objs.append(obj)
        jobs.append(subprocess.Popen([hipcc] + flags + ["-c", src, "-o", obj], stdout=subprocess.PIPE,
                                     stderr=subprocess.STDOUT, text=True))
    for proc in jobs:
        out, _ = proc.communicate()
        if proc.returncode != 0:
            print(out)
            raise RuntimeError("hipcc failed building the host-sanitized library")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-fsanitize=address", "-fsanitize=undefined",
                          "-fno-gpu-sanitize"] + objs + ["-o", SAN_LIB], capture_output=True, text=True)
    if res.returncode != 0:
        print(res.stdout, res.stderr)
        raise RuntimeError("hipcc failed linking the host-sanitized library")
    return SAN_LIB


def build_host_checks(force: bool = False) -> str:
    """tests/host/host_checks.cpp linked against the host-sanitized library; returns the executable's path."""
    lib = build_host_sanitized(force)
    exe = os.path.join(OBJDIR, "host_checks")
    src = os.path.join(HERE, "..", "tests", "host", "host_checks.cpp")
    if force or not os.path.exists(exe) or os.path.getmtime(exe) < max(os.path.getmtime(src), os.path.getmtime(lib)):
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        cmd = [hipcc, "-O1", "-g", "-std=c++17", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
               "-fno-sanitize-recover=undefined", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-x", "c++", src, "-x", "none", lib, "-Wl,-rpath," + OBJDIR, "-o", exe]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            print(res.stdout, res.stderr)
            raise RuntimeError("building tests/host/host_checks.cpp failed")
    return exe


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
