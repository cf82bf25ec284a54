"""Seeded synthetic inputs for the sparse-convolution workloads.

This module only *produces inputs* (voxel coordinates, feature matrices, weight
tensors).  It holds none of the method's arithmetic: no kernel maps, no hashing,
no convolution.  Both the CPU oracle's tests and the GPU path's tests/bench draw
their inputs from here, so the two sides see byte-identical arrays.

Every generator takes an explicit integer seed and uses
``numpy.random.Generator(numpy.random.PCG64(seed))``.

Coordinates are ``int32 [N, 4]`` with columns ``(b, x, y, z)``: batch index first,
then the three voxel indices.  Row order is whatever the generator produces; it
is *not* sorted unless stated (the paper treats a point cloud as an unordered
set, Sec. 2).
"""
from .generators import (  # noqa: F401
    uniform_grid_coords,
    box_surface_coords,
    lidar_scan_coords,
    tile_batches,
    features,
    conv_weights,
    shuffle_rows,
    CONFIG_SEEDS,
)
