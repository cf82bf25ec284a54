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


def check_features(y_gpu, y_ref64, dtype, what=""):
    ref = oracle.round_to(y_ref64, np_dtype(dtype))
    got = y_gpu.detach().cpu().numpy()
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got.astype(np.float64)).all(), what
    err = oracle.rel_l2(got, ref)
    assert err <= TOL[dtype], f"{what}: relative L2 error {err:.3e} > {TOL[dtype]:.1e}"
    return err
