"""Shared helpers for the GPU parity tests (comparison glue only, no method arithmetic)."""
import numpy as np
import torch

import oracle
from paper_2204_10319_amd import binding as ts

TOL = {torch.float32: 1e-5, torch.float16: 2e-3}   # max relative L2 error, whole output tensor


def np_dtype(dt):
    return np.float16 if dt == torch.float16 else np.float32


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_triples(kmap):
    """Sorted (in, out, offset) triples of a device kernel map."""
    sizes = kmap.sizes()
    a, b = kmap.pairs()
    n = np.repeat(np.arange(sizes.shape[0], dtype=np.int32), sizes)
    tri = np.stack([a.cpu().numpy(), b.cpu().numpy(), n], axis=1).astype(np.int32)
    return oracle.sort_triples(tri)


def oracle_map(coords, K, s, transposed=False, boundary=None):
    """(in_coords, out_coords, sorted triples) the library must reproduce for these arguments."""
    q = oracle.out_coords(coords, K, s, boundary=boundary)
    tri = oracle.kmap(coords, q, K, s)           # (j over coords, k over q, n)
    if transposed:
        tri = tri[:, [1, 0, 2]]                   # inputs are the coarse points, outputs the given fine points
        return q, np.asarray(coords, np.int32), oracle.sort_triples(tri)
    return np.asarray(coords, np.int32), q, oracle.sort_triples(tri)


def oracle_conv(coords, x, w, K, s, transposed=False, boundary=None):
    """float64 result of the layer on the same inputs."""
    q = oracle.out_coords(coords, K, s, boundary=boundary) if boundary is not None else None
    if transposed:
        _, y = oracle.conv_transposed(coords, x, w, K, s, coarse_coords=q)
    else:
        _, y = oracle.conv(coords, x, w, K, s, out_coords_=q)
    return y


def grid_of(coords, margin=0):
    """(lo, hi, batches) of a coordinate array, as the grid search wants its box stated."""
    c = np.asarray(coords)
    if c.shape[0] == 0:
        return (0, 0, 0), (0, 0, 0), 1
    return tuple(int(v) - margin for v in c[:, 1:].min(axis=0)), tuple(int(v) + margin for v in c[:, 1:].max(axis=0)), int(c[:, 0].max()) + 1


# Beside the whole-tensor norm (the bound the task states), two finer gates, because at 10^5 rows a few
# wrong rows or elements vanish in a norm:
#   per row      ||y_k - ref_k|| / max(||ref_k||, rms row norm)  (oracle.row_rel_err)
#   per element  |y - ref| <= 2 ulp(ref) + ELEM_FLOOR * rms(ref)
# fp16 in / fp32 accumulate: the stored value is the fp32 sum rounded once, the reference the fp64 sum
# rounded once; they differ by one ulp where the fp32 sum's own error (<= 2^-24 * sqrt(terms) * rms, terms
# <= 27 * 256) carries it across a rounding boundary, and by that error itself where the sum nearly
# cancels (an element far below the tensor's rms has a tiny ulp).  A single dropped product x * w is
# rms / sqrt(7 * C_in) >= 0.02 rms: two orders above the floor.
ROW_TOL = {torch.float32: 1e-5, torch.float16: 2e-3}
ELEM_FLOOR = {torch.float32: 5e-5, torch.float16: 1e-4}


def check_features(y_gpu, y_ref64, dtype, what="", elem_floor=None, row_tol=None, tol=None, pre_mag=None):
    """Whole-tensor relative L2 error, per-row error and per-element bound of a GPU result against the
    oracle's float64 result rounded once to the I/O dtype.  Returns the whole-tensor error; the worst row
    is printed (pytest -s shows it).

    ``pre_mag`` (array like the result, or None) is for results of layer + bias + residual + ReLU: there the
    layer's sum s is rounded to the I/O dtype before the elementwise step on both sides, so the two results
    may differ by one ulp of s, which exceeds two ulps of a result the residual has brought near zero.  It
    holds an upper bound of |s| per element (|result| + |bias| + |residual|), and one ulp of it is added to
    the element bound."""
    ndt = np_dtype(dtype)
    ref = oracle.round_to(y_ref64, ndt)
    got = y_gpu.detach().cpu().numpy()
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert got.dtype == ref.dtype, (what, got.dtype, ref.dtype)
    assert np.isfinite(got.astype(np.float64)).all(), what
    err = oracle.rel_l2(got, ref)
    tol = TOL[dtype] if tol is None else tol
    assert err <= tol, f"{what}: relative L2 error {err:.3e} > {tol:.1e}"
    if got.size == 0:
        return err
    rows = oracle.row_rel_err(got, ref)
    k = int(np.argmax(rows))
    print(f"{what}: rel L2 {err:.2e}, worst row {k} of {rows.shape[0]}: {rows[k]:.2e}")
    row_tol = ROW_TOL[dtype] if row_tol is None else row_tol
    assert rows[k] <= row_tol, f"{what}: row {k} is off by {rows[k]:.3e} > {row_tol:.1e} (relative to max(its norm, rms row norm))"
    ref64 = ref.astype(np.float64)
    rms = float(np.sqrt(np.mean(ref64 ** 2)))
    floor = (ELEM_FLOOR[dtype] if elem_floor is None else elem_floor) * rms
    bound = 2.0 * np.spacing(np.abs(ref)).astype(np.float64) + floor
    if pre_mag is not None:
        bound = bound + np.spacing(np.abs(np.asarray(pre_mag, np.float64)).astype(ndt)).astype(np.float64)
    diff = np.abs(got.astype(np.float64) - ref64)
    bad = diff > bound
    if bad.any():
        r, c = np.unravel_index(int(np.argmax(diff - bound)), diff.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} elements beyond 2 ulp + {floor:.2e}; worst at [{r}, {c}]: "
                             f"got {got[r, c]!r}, want {ref[r, c]!r}")
    return err
