"""Synthetic voxel sets, features and weights (inputs only, no method arithmetic).

The three coordinate recipes stand in for the paper's evaluation data (Sec. 5.1
uses real indoor/outdoor scans that are not available here):

* ``uniform_grid_coords``  - cells drawn uniformly without replacement from a cube.
* ``box_surface_coords``   - indoor-scene-like: surfaces of random axis-aligned boxes.
* ``lidar_scan_coords``    - outdoor-LiDAR-like: a simulated spinning multi-beam
  scanner over a ground plane with box obstacles, voxelized.
"""
from __future__ import annotations

import numpy as np

# seeds used for the five benchmark configurations (index = config number - 1)
CONFIG_SEEDS = (0, 1, 2, 3, 4)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def _first_occurrence_unique(rows: np.ndarray) -> np.ndarray:
    """Drop duplicate rows, keeping the first occurrence and the original order."""
    if rows.shape[0] == 0:
        return rows
    _, first = np.unique(rows, axis=0, return_index=True)
    first.sort()
    return rows[first]


def _with_batch(xyz: np.ndarray, batch: int = 0) -> np.ndarray:
    out = np.empty((xyz.shape[0], 4), dtype=np.int32)
    out[:, 0] = batch
    out[:, 1:] = xyz
    return np.ascontiguousarray(out)


def uniform_grid_coords(seed: int, n: int = 20000, grid: int = 64, batch: int = 0) -> np.ndarray:
    """``n`` distinct cells of a ``grid^3`` cube, in random order."""
    rng = _rng(seed)
    flat = rng.choice(grid ** 3, size=n, replace=False)
    x, y, z = np.unravel_index(flat, (grid, grid, grid))
    return _with_batch(np.stack([x, y, z], axis=1).astype(np.int32), batch)


def box_surface_coords(seed: int, n_boxes: int = 40, grid: int = 256,
                       side_min: int = 10, side_max: int = 80, batch: int = 0) -> np.ndarray:
    """Surface voxels of ``n_boxes`` random axis-aligned boxes inside ``grid^3``.

    Each box has integer side lengths uniform in ``[side_min, side_max]`` per axis and an
    origin uniform over the positions that keep it inside the grid.  Only voxels on the
    six faces are kept; duplicates (overlapping boxes) are removed, first occurrence wins.
    """
    rng = _rng(seed)
    chunks = []
    for _ in range(n_boxes):
        side = rng.integers(side_min, side_max + 1, size=3)
        org = np.array([rng.integers(0, grid - s + 1) for s in side])
        ax = [np.arange(org[a], org[a] + side[a]) for a in range(3)]
        for a in range(3):                      # two faces per axis
            b, c = [d for d in range(3) if d != a]
            gb, gc = np.meshgrid(ax[b], ax[c], indexing="ij")
            for face in (org[a], org[a] + side[a] - 1):
                pts = np.empty((gb.size, 3), dtype=np.int32)
                pts[:, a] = face
                pts[:, b] = gb.ravel()
                pts[:, c] = gc.ravel()
                chunks.append(pts)
    xyz = np.concatenate(chunks, axis=0) if chunks else np.zeros((0, 3), np.int32)
    return _with_batch(_first_occurrence_unique(xyz), batch)


def lidar_scan_coords(seed: int, n_sweeps: int = 1, n_beams: int = 64, n_azimuth: int = 2048,
                      elev_deg=(-25.0, 3.0), ground_z: float = -1.7, n_boxes: int = 30,
                      voxel: float = 0.05, xy_range: float = 51.2, z_range=(-3.0, 1.0),
                      sweep_step: float = 1.0, batch: int = 0) -> np.ndarray:
    """Voxelized hits of a simulated spinning scanner.

    The scene is a ground plane ``z = ground_z`` plus ``n_boxes`` random axis-aligned boxes
    standing on it.  A sweep casts ``n_beams x n_azimuth`` rays from the sensor (elevations
    linearly spaced over ``elev_deg``, azimuths over the full circle) and keeps the nearest
    hit.  ``n_sweeps`` sweeps are aggregated with the sensor moved ``sweep_step`` metres
    along +x between sweeps (a multi-frame input).  Hits are cropped to
    ``|x|,|y| < xy_range`` and ``z_range``, then quantized to ``voxel``-sized cells and
    shifted so all indices are non-negative.  Row order = order of first hit
    (sweep, beam, azimuth).
    """
    rng = _rng(seed)
    # scene
    bsz = np.stack([rng.uniform(1.5, 8.0, n_boxes), rng.uniform(1.5, 8.0, n_boxes),
                    rng.uniform(1.0, 3.5, n_boxes)], axis=1)
    rad = rng.uniform(6.0, 45.0, n_boxes)
    ang = rng.uniform(0.0, 2 * np.pi, n_boxes)
    ctr = np.stack([rad * np.cos(ang), rad * np.sin(ang)], axis=1)
    bmin = np.concatenate([ctr - bsz[:, :2] / 2, np.full((n_boxes, 1), ground_z)], axis=1)
    bmax = np.concatenate([ctr + bsz[:, :2] / 2, ground_z + bsz[:, 2:3]], axis=1)

    elev = np.deg2rad(np.linspace(elev_deg[0], elev_deg[1], n_beams))
    azim = np.linspace(0.0, 2 * np.pi, n_azimuth, endpoint=False)
    ce, se = np.cos(elev)[:, None], np.sin(elev)[:, None]
    d = np.stack([ce * np.cos(azim)[None, :], ce * np.sin(azim)[None, :],
                  np.broadcast_to(se, (n_beams, n_azimuth))], axis=-1).reshape(-1, 3)

    hits = []
    for sweep in range(n_sweeps):
        o = np.array([sweep * sweep_step, 0.0, 0.0])
        t = np.full(d.shape[0], np.inf)
        down = d[:, 2] < 0
        t[down] = (ground_z - o[2]) / d[down, 2]
        with np.errstate(divide="ignore", invalid="ignore"):
            inv = 1.0 / d
            for i in range(n_boxes):            # slab test per box
                t0 = (bmin[i] - o) * inv
                t1 = (bmax[i] - o) * inv
                tn = np.minimum(t0, t1).max(axis=1)
                tf = np.maximum(t0, t1).min(axis=1)
                ok = (tf >= tn) & (tn > 0)
                t = np.where(ok & (tn < t), tn, t)
        fin = np.isfinite(t)
        p = o[None, :] + d[fin] * t[fin, None]
        hits.append(p)
    p = np.concatenate(hits, axis=0)
    keep = ((np.abs(p[:, 0]) < xy_range) & (np.abs(p[:, 1]) < xy_range) &
            (p[:, 2] >= z_range[0]) & (p[:, 2] < z_range[1]))
    p = p[keep]
    lo = np.array([-xy_range, -xy_range, z_range[0]])
    ijk = np.floor((p - lo[None, :]) / voxel).astype(np.int32)
    return _with_batch(_first_occurrence_unique(ijk), batch)


def tile_batches(coords: np.ndarray, copies: int) -> np.ndarray:
    """Replicate a point cloud ``copies`` times with batch indices ``0..copies-1``."""
    outs = []
    for b in range(copies):
        c = coords.copy()
        c[:, 0] = b
        outs.append(c)
    return np.ascontiguousarray(np.concatenate(outs, axis=0))


def shuffle_rows(seed: int, *arrays: np.ndarray):
    """Apply one random row permutation to all arrays (same leading dimension)."""
    perm = _rng(seed).permutation(arrays[0].shape[0])
    out = tuple(np.ascontiguousarray(a[perm]) for a in arrays)
    return out if len(out) > 1 else out[0]


def features(seed: int, n: int, channels: int, dtype=np.float32) -> np.ndarray:
    """``[n, channels]`` standard-normal features, rounded to ``dtype``."""
    x = _rng(seed).standard_normal((n, channels))
    return np.ascontiguousarray(x.astype(dtype))


def conv_weights(seed: int, kernel_volume: int, c_in: int, c_out: int, dtype=np.float32,
                 gain: float = 1.0) -> np.ndarray:
    """``[kernel_volume, c_in, c_out]`` weights ~ N(0, gain / (kernel_volume * c_in))."""
    std = np.sqrt(gain / (kernel_volume * c_in))
    w = _rng(seed).standard_normal((kernel_volume, c_in, c_out)) * std
    return np.ascontiguousarray(w.astype(dtype))
