"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU needed).

A copy of libts.so whose host side is compiled with -fsanitize=address,undefined (device code as usual)
is linked into tests/host/host_checks.cpp, which walks the argument checks, the error texts, the host
arithmetic of ts_adaptive_groups and the NULL-safe releases.  Calls that would need a device must fail
with an error code; a bad read or an overflow in these paths stops the program.
"""
import os
import subprocess

from paper_2204_10319_amd import build


def test_host_paths_under_asan_and_ubsan():
    exe = build.build_host_checks()
    env = dict(os.environ)
    # the HIP runtime keeps process-lifetime allocations: leaks are not what this looks for
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert res.returncode == 0, res.stdout[-4000:] + res.stderr[-4000:]
    assert "host checks ok" in res.stdout
