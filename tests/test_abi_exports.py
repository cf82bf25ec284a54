"""The built library loads and exports every symbol declared in include/ts.h (no GPU needed)."""
import os
import re

from paper_2204_10319_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ts.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ts_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    declared = _declared_functions()
    assert "ts_build_kmap" in declared and "ts_sparse_conv" in declared and "ts_free" in declared
    assert sorted(binding.EXPORTS) == declared


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    for name in _declared_functions():
        assert hasattr(lib, name), name
    assert binding.ts_version().startswith("libts")


def test_constants_match_the_header():
    text = open(os.path.join(ROOT, "include", "ts.h")).read()
    for name in ("TS_BATCH_MAX", "TS_COORD_MIN", "TS_COORD_MAX"):
        val = int(re.search(rf"#define {name} \(?(-?\d+)\)?", text).group(1))
        assert getattr(binding, name) == val
    for name, val in re.findall(r"(TS_ERR_[A-Z_]+) = (-?\d+)", text):
        assert getattr(binding, name) == int(val)


def test_bench_refuses_more_than_one_gpu():
    """Everything here runs on one GPU; bench.py says so instead of starting ranks (no GPU needed for this)."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
