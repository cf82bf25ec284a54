"""CPU oracle for the sparse-convolution layer -- TEST INFRASTRUCTURE ONLY.

A thin ctypes wrapper around ``sparseconv_oracle.c`` (plain C, double precision,
sorted coordinates + binary search, direct evaluation of the paper's Eq. 1).
Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package; the GPU library never does, and this package never imports the
GPU library.

Paper passages each function follows:

* :func:`offsets`       - kernel-offset set Delta^3(K), Sec. 2
* :func:`out_coords`    - output coordinates, Sec. 2.1.1 / Alg. 3 (Appendix A)
* :func:`kmap`          - map search, Sec. 2.1.2 / Alg. 1
* :func:`conv`          - Eq. 1 evaluated per output row and per offset
* :func:`conv_transposed` - same pair set with in/out roles swapped (not in the paper)
* :func:`adaptive_groups` - partition of the weight indices by map size, first half of the
  grouped matmul of Appendix B (Alg. 4)
* :func:`adaptive_group_search` - exhaustive choice of the tolerance and threshold (Appendix B, Alg. 5)

Pins (see ``tests/test_oracle_pins.py``): the paper's worked stride-2 example and
printed offset sets, brute-force neighbour enumeration, dense 3-D convolution
masked to the active sites, the 1x1x1 == matmul identity, full-occupancy ==
zero-padded dense convolution, the submanifold symmetry of Sec. 4.2.1, and a
closed-form expectation of the map sizes on uniformly sampled grids.
:func:`adaptive_groups` is pinned by the special cases the paper names (tolerance 0 keeps only
equal sizes together, tolerance 1 makes one group), by the invariants of the partition (contiguous,
covering, every group within the tolerance, no group extensible) and by exhaustive comparison with
a search over all contiguous partitions on small inputs.  :func:`adaptive_group_search` is pinned by
numpy's argmin over a table of costs, ties included.
The comparison helpers are pinned too: :func:`rel_l2` and :func:`row_rel_err` by hand-computed
vectors (3-4-5 triangles, zero references, a single wrong row among many), :func:`round_to` by the
tie points of binary16 and binary32 written out by hand (round-to-nearest-even, overflow to inf),
:func:`sort_triples` by a hand-ordered list and by Python's ``sorted`` on the key ``(n, k, j)``.
Parity status: every function of this package is pinned by at least one of these.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparseconv_oracle.c")
_LIB = os.path.join(_HERE, "libsparseconv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP over output rows). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i64, i32p, f64p = ctypes.c_int64, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)
    ci = ctypes.c_int
    lib.orc_offset.argtypes = [ci, ci, i32p]
    lib.orc_offset.restype = None
    lib.orc_out_coords.argtypes = [i32p, i64, ci, ci, i32p, i32p, i64]
    lib.orc_out_coords.restype = i64
    lib.orc_kmap.argtypes = [i32p, i64, i32p, i64, ci, ci, i32p, i64]
    lib.orc_kmap.restype = i64
    lib.orc_conv.argtypes = [i32p, i64, i32p, i64, ci, ci, f64p, ci, f64p, ci, f64p, ci]
    lib.orc_conv.restype = ci
    lib.orc_conv_transposed.argtypes = [i32p, i64, i32p, i64, ci, ci, f64p, ci, f64p, ci, f64p, ci]
    lib.orc_conv_transposed.restype = ci
    lib.orc_max_threads.argtypes = []
    lib.orc_max_threads.restype = ci
    _lib = lib
    return lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check_coords(c):
    c = np.ascontiguousarray(c, dtype=np.int32)
    if c.ndim != 2 or c.shape[1] != 4:
        raise ValueError("coords must be [N,4] = (batch, x, y, z)")
    return c


def default_threads() -> int:
    """Threads the OpenMP loops use unless told otherwise (bounded by the CPU count)."""
    return max(1, min(os.cpu_count() or 1, _load().orc_max_threads()))


def offsets(K: int) -> np.ndarray:
    """``[K^3, 3]`` kernel offsets in weight-index order (Sec. 2)."""
    lib = _load()
    out = np.zeros((K ** 3, 3), dtype=np.int32)
    for n in range(K ** 3):
        d = (ctypes.c_int32 * 3)()
        lib.orc_offset(K, n, d)
        out[n] = list(d)
    return out


def out_coords(coords, K: int, s: int, boundary=None) -> np.ndarray:
    """Output coordinates of a (K, s) convolution (Alg. 3); sorted when ``s > 1``.

    ``boundary`` = (bx, by, bz): candidates outside ``0 <= u < s*b`` are dropped (Alg. 3's boundary
    check; ignored at stride 1, where the outputs are the inputs)."""
    lib = _load()
    c = _check_coords(coords)
    c, cp = _i32(c)
    bp = None
    if boundary is not None:
        b = np.ascontiguousarray(np.asarray(boundary, dtype=np.int32).reshape(3))
        bp = b.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    n_out = lib.orc_out_coords(cp, c.shape[0], K, s, bp, None, 0)
    if n_out < 0:
        raise MemoryError("oracle: allocation failed")
    out = np.zeros((n_out, 4), dtype=np.int32)
    out, op = _i32(out)
    lib.orc_out_coords(cp, c.shape[0], K, s, bp, op, n_out)
    return out


def kmap(in_coords, out_coords_, K: int, s: int) -> np.ndarray:
    """Kernel map as ``[M, 3]`` int32 triples ``(j, k, n)`` with ``p_j = s*q_k + delta_n`` (Alg. 1)."""
    lib = _load()
    a, ap = _i32(_check_coords(in_coords))
    b, bp = _i32(_check_coords(out_coords_))
    m = lib.orc_kmap(ap, a.shape[0], bp, b.shape[0], K, s, None, 0)
    if m == -2:
        raise ValueError("oracle: duplicate input coordinates")
    if m < 0:
        raise MemoryError("oracle: allocation failed")
    tri = np.zeros((m, 3), dtype=np.int32)
    tri, tp = _i32(tri)
    lib.orc_kmap(ap, a.shape[0], bp, b.shape[0], K, s, tp, m)
    return tri


def _check_rc(rc):
    if rc == -2:
        raise ValueError("oracle: duplicate input coordinates")
    if rc != 0:
        raise MemoryError("oracle: allocation failed")


def conv(in_coords, x, w, K: int, s: int, out_coords_=None, threads: int | None = None):
    """Forward sparse convolution, Eq. 1.  Returns ``(out_coords, y)`` with ``y`` in float64.

    ``x`` is ``[N_in, C_in]``, ``w`` is ``[K^3, C_in, C_out]``; both are converted to
    float64 exactly (float16/float32 values are representable).
    """
    lib = _load()
    a, ap = _i32(_check_coords(in_coords))
    q = out_coords(a, K, s) if out_coords_ is None else _check_coords(out_coords_)
    q, qp = _i32(q)
    x, xp = _f64(x)
    w, wp = _f64(w)
    if x.shape[0] != a.shape[0] or w.shape[0] != K ** 3 or w.shape[1] != x.shape[1]:
        raise ValueError("oracle: shape mismatch")
    y = np.zeros((q.shape[0], w.shape[2]), dtype=np.float64)
    y, yp = _f64(y)
    th = default_threads() if threads is None else int(threads)
    _check_rc(lib.orc_conv(ap, a.shape[0], qp, q.shape[0], K, s, xp, x.shape[1], wp, w.shape[2], yp, th))
    return q, y


def conv_transposed(fine_coords, x_coarse, w, K: int, s: int, coarse_coords=None,
                    threads: int | None = None):
    """Transposed sparse convolution onto ``fine_coords``.  Returns ``(coarse_coords, y)``.

    ``x_coarse`` is ``[N_coarse, C_in]`` with rows in the order of ``coarse_coords``
    (default: the sorted output coordinates of the forward (K, s) convolution of
    ``fine_coords``); ``y`` is ``[N_fine, C_out]`` float64.
    """
    lib = _load()
    f, fp = _i32(_check_coords(fine_coords))
    c = out_coords(f, K, s) if coarse_coords is None else _check_coords(coarse_coords)
    c, cp = _i32(c)
    x, xp = _f64(x_coarse)
    w, wp = _f64(w)
    if x.shape[0] != c.shape[0] or w.shape[0] != K ** 3 or w.shape[1] != x.shape[1]:
        raise ValueError("oracle: shape mismatch")
    y = np.zeros((f.shape[0], w.shape[2]), dtype=np.float64)
    y, yp = _f64(y)
    th = default_threads() if threads is None else int(threads)
    _check_rc(lib.orc_conv_transposed(fp, f.shape[0], cp, c.shape[0], K, s, xp, x.shape[1], wp,
                                      w.shape[2], yp, th))
    return c, y


def round_to(y: np.ndarray, dtype) -> np.ndarray:
    """One final round-to-nearest-even of the double result to the I/O dtype."""
    return np.asarray(y, dtype=np.float64).astype(dtype)


def rel_l2(y, y_ref) -> float:
    """``||y - y_ref||_F / ||y_ref||_F`` in float64 (0 when both are empty or zero)."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    if y.shape != y_ref.shape:
        raise ValueError(f"rel_l2: shapes differ, {y.shape} vs {y_ref.shape}")
    den = float(np.linalg.norm(y_ref))
    num = float(np.linalg.norm(y - y_ref))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


def row_rel_err(y, y_ref) -> np.ndarray:
    """Per-row error ``||y_k - ref_k|| / max(||ref_k||, ||ref||_F / sqrt(rows))`` in float64, one value
    per row: the whole-tensor norm of :func:`rel_l2` cannot see a handful of wrong rows among 10^5, this
    can.  The floor (the root-mean-square row norm) keeps rows that are nearly zero from dividing by
    nothing.  Empty input gives an empty array; an all-zero reference gives 0 where ``y`` is zero too
    and inf elsewhere."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    if y.shape != y_ref.shape or y.ndim != 2:
        raise ValueError("row_rel_err: two [rows, cols] arrays of one shape")
    if y.shape[0] == 0:
        return np.zeros(0)
    num = np.sqrt(((y - y_ref) ** 2).sum(axis=1))
    ref_rows = np.sqrt((y_ref ** 2).sum(axis=1))
    floor = float(np.sqrt((ref_rows ** 2).sum() / y.shape[0]))
    den = np.maximum(ref_rows, floor)
    out = np.zeros_like(num)
    nz = den > 0
    out[nz] = num[nz] / den[nz]
    out[~nz & (num > 0)] = np.inf
    return out


def adaptive_groups(sizes, eps: float) -> list[list[int]]:
    """Groups of consecutive weight indices whose map sizes are close enough to be padded to a
    common length (Appendix B, Alg. 4, first loop).

    ``sizes[i]`` is the map size of weight index ``i`` (for an odd kernel at stride 1 the caller
    passes the first floor(K^3/2) indices: each stands for itself and its mirror).  A group starts
    at the first index not yet grouped and takes following indices as long as
    ``1 - n_min / n_max <= eps`` over the sizes taken so far including the candidate (the share of
    padded, i.e. wasted, rows in the longest member's terms).  The listing prints ``n_min <- 0`` and
    never advances its outer index; read as ``n_min <- n_max <- len(M[W_i])`` and "continue after the
    last index taken".  Two empty maps count as equal (ratio 0).
    """
    sizes = [int(v) for v in sizes]
    groups, i = [], 0
    while i < len(sizes):
        n_min = n_max = sizes[i]
        group = [i]
        j = i + 1
        while j < len(sizes):
            lo, hi = min(n_min, sizes[j]), max(n_max, sizes[j])
            waste = 0.0 if hi == 0 else 1.0 - lo / hi
            if waste > eps:
                break
            n_min, n_max = lo, hi
            group.append(j)
            j += 1
        groups.append(group)
        i = j
    return groups


def adaptive_group_search(samples, eps_space, S_space, cost):
    """Pick the (tolerance, threshold) pair with the smallest cost summed over the samples
    (Appendix B, Alg. 5).  ``cost(sample, eps, S)`` stands for the elapsed time of the grouped matmul;
    pairs are tried with the tolerance in the outer loop and the first pair reaching the minimum is kept
    (the listing's ``c_min = 0`` only marks "nothing chosen yet").  Returns ``(eps, S, total_cost)``.
    """
    best = None
    for eps in eps_space:
        for S in S_space:
            c = 0.0
            for sample in samples:
                c = c + cost(sample, eps, S)
            if best is None or c < best[2]:
                best = (eps, S, c)
    return best


def sort_triples(tri: np.ndarray) -> np.ndarray:
    """Triples ``(j, k, n)`` in canonical order: by n, then k, then j."""
    tri = np.asarray(tri, dtype=np.int32).reshape(-1, 3)
    order = np.lexsort((tri[:, 0], tri[:, 1], tri[:, 2]))
    return np.ascontiguousarray(tri[order])
