"""The built library loads and exports every symbol declared in include/*.h (no GPU needed)."""
import os
import re

from paper_2204_10319_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(ts_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_measurement_helpers_are_not_in_the_layer_header():
    text = open(os.path.join(ROOT, "include", "ts.h")).read()
    for name in ("ts_copy_bytes", "ts_mfma_loop", "ts_profile_enable", "ts_profile_read"):
        assert name not in text, name


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


def test_adaptive_groups_host_function_equals_the_oracle():
    """ts_adaptive_groups is host arithmetic (Appendix B, Alg. 4, first loop): same partition as the oracle's."""
    import numpy as np
    import pytest
    import oracle
    rng = np.random.Generator(np.random.PCG64(21))
    cases = [([], 0.3), ([0], 0.0), ([0, 0, 5], 0.0), ([100, 90, 60, 55, 10], 0.15)]
    for trial in range(400):
        n = int(rng.integers(1, 28))
        sizes = (rng.integers(0, 5, size=n) * 7).tolist() if trial % 4 == 0 else rng.integers(0, 100000, size=n).tolist()
        cases.append((sizes, float(rng.choice([0.0, 0.05, 0.2, 0.5, 0.75, 1.0]))))
    for sizes, eps in cases:
        expect = [0] * len(sizes)
        for g, members in enumerate(oracle.adaptive_groups(sizes, eps)):
            for i in members:
                expect[i] = g
        assert binding.ts_adaptive_groups(sizes, eps) == expect, (sizes, eps)
    for bad in (([1, 2], -0.1), ([1, 2], 1.5), ([1, -2], 0.5), (list(range(28)), 0.5)):
        with pytest.raises(binding.TsError) as e:
            binding.ts_adaptive_groups(*bad)
        assert e.value.code == binding.TS_ERR_INVALID_ARG


def test_tuner_picks_what_the_oracle_picks():
    """The product's search (Appendix B, Alg. 5) with a host cost function against the oracle's."""
    import numpy as np
    import oracle
    from paper_2204_10319_amd import tuner
    rng = np.random.Generator(np.random.PCG64(22))
    for trial in range(30):
        eps_space, S_space = list(tuner.DEFAULT_EPS_SPACE[: int(rng.integers(1, 9))]), list(tuner.DEFAULT_S_SPACE[: int(rng.integers(1, 5))])
        nd = int(rng.integers(1, 4))
        costs = {(d, e, S): float(rng.integers(1, 5 if trial % 2 else 10 ** 6)) for d in range(nd) for e in eps_space for S in S_space}
        f = lambda d, e, S: costs[(d, e, S)]
        eps, S, c, table = tuner.adaptive_group_search(range(nd), eps_space, S_space, f)
        assert (eps, S, c) == oracle.adaptive_group_search(range(nd), eps_space, S_space, f)
        assert len(table) == len(eps_space) * len(S_space)
