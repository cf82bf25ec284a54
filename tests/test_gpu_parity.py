"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Kernel maps must equal the oracle's bit-exactly as sorted (in, out, offset) triples;
features must agree within a relative L2 error of 1e-5 (fp32) / 2e-3 (fp16 in, fp32 accumulate).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2204_10319_amd import binding as ts
from workloads import (uniform_grid_coords, box_surface_coords, lidar_scan_coords, features, conv_weights,
                       shuffle_rows)
from _util import TOL, np_dtype, to_dev, gpu_triples, oracle_map, oracle_conv, check_features, grid_of

pytestmark = pytest.mark.gpu


def _rand_coords(seed, n, lo, hi, batches=1):
    rng = np.random.Generator(np.random.PCG64(seed))
    side = hi - lo
    flat = rng.choice(batches * side ** 3, size=n, replace=False)
    b, x, y, z = np.unravel_index(flat, (batches, side, side, side))
    return np.stack([b, x + lo, y + lo, z + lo], axis=1).astype(np.int32)


def _check_map(coords, K, s, transposed=False, grid=None, boundary=None, wait=True, search=ts.TS_SEARCH_AUTO):
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed, wait=wait, grid=grid, boundary=boundary, search=search)
    in_c, out_c, tri = oracle_map(coords, K, s, transposed, boundary=boundary)
    assert kmap.num_in == in_c.shape[0]
    assert kmap.num_out == out_c.shape[0]
    assert kmap.kernel_volume == K ** 3
    assert np.array_equal(kmap.out_coords().cpu().numpy(), out_c)
    assert np.array_equal(kmap.in_coords().cpu().numpy(), in_c)
    assert kmap.num_pairs == tri.shape[0]
    assert np.array_equal(kmap.sizes(), np.bincount(tri[:, 2], minlength=K ** 3))
    assert np.array_equal(gpu_triples(kmap), tri)
    return kmap


MAP_CASES = [(1, 1, False), (3, 1, False), (2, 2, False), (3, 2, False), (1, 2, False), (2, 2, True), (3, 2, True)]


@pytest.mark.parametrize("K,s,transposed", MAP_CASES)
@pytest.mark.parametrize("n", [1, 37, 700, 5000])
def test_kmap_small(K, s, transposed, n):
    """Several tiles and a ragged tail, negative coordinates, three batch indices."""
    coords = _rand_coords(1000 + n + 10 * K + s, n, -9, 9, batches=3)
    _check_map(coords, K, s, transposed)


@pytest.mark.parametrize("K,s,transposed", MAP_CASES)
def test_kmap_empty(K, s, transposed):
    kmap = ts.ts_build_kmap(torch.zeros((0, 4), dtype=torch.int32, device="cuda"), K, s, transposed)
    assert kmap.num_in == 0 and kmap.num_out == 0 and kmap.num_pairs == 0
    assert kmap.sizes().sum() == 0


def test_kmap_extreme_coordinates():
    lo, hi = ts.TS_COORD_MIN, ts.TS_COORD_MAX
    coords = np.array([[0, lo, lo, lo], [0, lo + 1, lo, lo], [0, hi, hi, hi], [0, hi, hi - 1, hi],
                       [ts.TS_BATCH_MAX, 0, 0, 0], [ts.TS_BATCH_MAX, 0, 0, 1], [0, 0, 0, 0]], dtype=np.int32)
    for K, s, tr in MAP_CASES:
        _check_map(coords, K, s, tr)


@pytest.mark.parametrize("wait", [True, False])
def test_kmap_rows_start_clean_in_reused_memory(wait):
    """The neighbour rows of a 3x3x3 map are set to "no neighbour" by the build itself (the symmetric search
    writes hits only): a dense scene leaves a table full of entries in the library's pool, and a sparse scene of
    the same size built right after it, most likely into the same block, must show none of them.  Sizes on
    both sides of a whole number of 256-point workgroups."""
    for n in (255, 256, 257, 4096, 5000):
        dense = _rand_coords(7000 + n, n, 0, max(2, int(np.ceil(n ** (1 / 3))) + 1))      # nearly every cell taken
        _check_map(dense, 3, 1, wait=wait).free()
        sparse = _rand_coords(7100 + n, n, -60, 60)                                       # hardly any neighbours
        _check_map(sparse, 3, 1, wait=wait).free()


def test_kmap_errors():
    dup = np.array([[0, 1, 2, 3], [0, 5, 5, 5], [0, 1, 2, 3]], dtype=np.int32)
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(dup), 3, 1)
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(dup), 2, 2, True)
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
    far = np.array([[0, 1, 2, 3], [0, ts.TS_COORD_MAX + 1, 0, 0]], dtype=np.int32)
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(far), 3, 1)
    assert e.value.code == ts.TS_ERR_COORD_RANGE
    neg_batch = np.array([[-1, 1, 2, 3]], dtype=np.int32)
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(neg_batch), 2, 2)
    assert e.value.code == ts.TS_ERR_COORD_RANGE
    ok = to_dev(np.array([[0, 1, 2, 3]], dtype=np.int32))
    for K, s, tr in [(2, 1, False), (4, 1, False), (3, 3, False), (3, 1, True), (0, 1, False)]:
        with pytest.raises(ts.TsError) as e:
            ts.ts_build_kmap(ok, K, s, tr)
        assert e.value.code == ts.TS_ERR_INVALID_ARG
    # the library still works after the failures
    _check_map(_rand_coords(5, 100, 0, 6), 3, 1)


def _layer_case(coords, c_in, c_out, K, s, transposed, dtype, seed,
                dataflows=(ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FUSED_STAGED, ts.TS_DATAFLOW_FETCH, ts.TS_DATAFLOW_AUTO)):
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    x = features(seed, kmap.num_in, c_in, np_dtype(dtype))
    w = conv_weights(seed + 1, K ** 3, c_in, c_out, np_dtype(dtype))
    ref = oracle_conv(coords, x, w, K, s, transposed)
    errs = []
    for df in dataflows:
        y = ts.ts_sparse_conv(to_dev(x), to_dev(w), kmap, dataflow=df)
        torch.cuda.synchronize()
        errs.append(check_features(y, ref, dtype, f"dataflow {df} C {c_in}->{c_out} K{K} s{s} t{transposed}"))
    return errs


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("K,s,transposed", [(3, 1, False), (1, 1, False), (2, 2, False), (2, 2, True), (3, 2, False), (3, 2, True)])
@pytest.mark.parametrize("c_in,c_out", [(32, 32), (16, 64), (64, 96), (48, 128), (128, 256)])
def test_layer_small(dtype, K, s, transposed, c_in, c_out):
    coords = _rand_coords(77 + c_in + K, 1500, -7, 7, batches=2)
    _layer_case(coords, c_in, c_out, K, s, transposed, dtype, seed=c_in + c_out)


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("n", [1, 31, 129, 1000])
def test_layer_ragged_sizes(dtype, n):
    coords = _rand_coords(300 + n, n, 0, 11)
    _layer_case(coords, 32, 32, 3, 1, False, dtype, seed=n)


@pytest.mark.parametrize("c_in", [4, 8, 24])
def test_layer_narrow_input(c_in):
    """C_in below the MFMA operand step (the 4-channel stem) is zero-extended inside the library."""
    coords = _rand_coords(55, 900, 0, 10)
    _layer_case(coords, c_in, 32, 3, 1, False, torch.float16, seed=c_in)


@pytest.mark.parametrize("c_in,c_out", [(96, 96), (160, 64), (224, 32), (72, 32)])
@pytest.mark.parametrize("K,s,transposed", [(3, 1, False), (2, 2, True)])
def test_layer_channel_counts_that_are_odd_multiples_of_32(c_in, c_out, K, s, transposed):
    """Rows of 96, 160, 224 channels (and 72, padded to 96): chunking by 32 channels; nothing read past a
    row's end (the start of the next row) may count."""
    coords = _rand_coords(91 + c_in, 1300, -6, 6, batches=2)
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    x = features(910 + c_in, kmap.num_in, c_in, np.float16)
    w = conv_weights(911 + c_in, K ** 3, c_in, c_out, np.float16)
    ref = oracle_conv(coords, x, w, K, s, transposed)
    pw = ts.ts_weights_prepare(to_dev(w))
    for df in (ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH):
        check_features(ts.ts_sparse_conv(to_dev(x), to_dev(w), kmap, dataflow=df), ref, torch.float16, f"C {c_in}->{c_out} dataflow {df}")
    check_features(ts.ts_sparse_conv_prepared(to_dev(x), pw, kmap), ref, torch.float16, f"C {c_in}->{c_out} prepared")
    # a large value in the first channel of every row, with zero weights: a step that multiplied the next row's
    # start into the sums would show
    x2 = x.copy()
    x2[:, 0] = np.float16(60000.0)
    w2 = w.copy()
    w2[:, 0, :] = 0
    ref2 = oracle_conv(coords, x2, w2, K, s, transposed)
    check_features(ts.ts_sparse_conv(to_dev(x2), to_dev(w2), kmap, dataflow=ts.TS_DATAFLOW_FUSED), ref2, torch.float16, "large first channel")


@pytest.mark.parametrize("c_in,c_out", [(512, 512), (1024, 64), (64, 1024), (1024, 1024)])
def test_layer_widest_channels(c_in, c_out):
    """The widest layers the library accepts (1024 channels either side), every dataflow, fp16; beyond: an error."""
    coords = _rand_coords(600 + c_in, 400, -5, 5)
    _layer_case(coords, c_in, c_out, 3, 1, False, torch.float16, seed=c_in + c_out,
                dataflows=(ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_FETCH, ts.TS_DATAFLOW_AUTO))
    _layer_case(coords, c_in, c_out, 2, 2, True, torch.float16, seed=c_in + c_out + 1,
                dataflows=(ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT))


def test_layer_too_wide_is_refused():
    coords = _rand_coords(9, 200, 0, 8)
    kmap = ts.ts_build_kmap(to_dev(coords), 1, 1)
    for c_in, c_out in [(1056, 32), (32, 1056)]:
        with pytest.raises(ts.TsError) as e:
            ts.ts_sparse_conv(torch.zeros((200, c_in), dtype=torch.float16, device="cuda"),
                              torch.zeros((1, c_in, c_out), dtype=torch.float16, device="cuda"), kmap)
        assert e.value.code == ts.TS_ERR_UNSUPPORTED


def test_layer_empty():
    kmap = ts.ts_build_kmap(torch.zeros((0, 4), dtype=torch.int32, device="cuda"), 3, 1)
    x = torch.zeros((0, 32), dtype=torch.float16, device="cuda")
    w = torch.zeros((27, 32, 32), dtype=torch.float16, device="cuda")
    for df in (ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH):
        assert ts.ts_sparse_conv(x, w, kmap, dataflow=df).shape == (0, 32)


def test_layer_shape_errors():
    coords = _rand_coords(9, 200, 0, 8)
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    x = torch.zeros((200, 32), dtype=torch.float16, device="cuda")
    w = torch.zeros((27, 32, 32), dtype=torch.float16, device="cuda")
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv(x[:100].contiguous(), w, kmap)
    assert e.value.code == ts.TS_ERR_SHAPE
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv(x, w[:8].contiguous(), kmap)
    assert e.value.code == ts.TS_ERR_SHAPE
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv(x, w.float(), kmap)
    assert e.value.code == ts.TS_ERR_SHAPE
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv(x, torch.zeros((27, 32, 40), dtype=torch.float16, device="cuda"), kmap)
    assert e.value.code == ts.TS_ERR_UNSUPPORTED


def test_config1_uniform_grid_fp32():
    """20 000 of 64^3 cells, C 32->32, fp32, submanifold 3x3x3."""
    coords = uniform_grid_coords(0)
    kmap = _check_map(coords, 3, 1)
    assert abs(kmap.num_pairs - 58400) < 1500
    errs = _layer_case(coords, 32, 32, 3, 1, False, torch.float32, seed=100)
    print("config 1 rel L2:", errs)


def test_config2_box_surfaces_fp16():
    """~100k box-surface voxels in 256^3, C 64->64, fp16 with fp32 accumulation."""
    coords = box_surface_coords(1, n_boxes=9)
    assert 90000 <= coords.shape[0] <= 110000
    _check_map(coords, 3, 1)
    errs = _layer_case(coords, 64, 64, 3, 1, False, torch.float16, seed=200)
    print("config 2 rel L2:", errs)


@pytest.mark.timeout(600)
def test_config2b_box_surfaces_40_boxes_fp16():
    """The literal recipe of config 2 (40 boxes): ~470k box-surface voxels, C 64->64 fp16 - the map bit for bit,
    the fused layer row by row and element by element, on more tiles than any other single-layer case."""
    coords = box_surface_coords(1, n_boxes=40)
    assert 400000 <= coords.shape[0] <= 550000
    _check_map(coords, 3, 1)
    errs = _layer_case(coords, 64, 64, 3, 1, False, torch.float16, seed=210, dataflows=(ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT))
    print("config 2b rel L2:", errs)


@pytest.fixture(scope="module")
def lidar_coords():
    return lidar_scan_coords(2, n_sweeps=5)


def test_config3_lidar_map(lidar_coords):
    assert 135000 <= lidar_coords.shape[0] <= 165000
    _check_map(lidar_coords, 3, 1)


@pytest.mark.parametrize("c", [32, 64, 128])
def test_config3_lidar_fp16(lidar_coords, c):
    errs = _layer_case(lidar_coords, c, c, 3, 1, False, torch.float16, seed=300 + c)
    print(f"config 3 C={c} rel L2:", errs)


def test_config3_in_the_launch_configuration_of_the_benchmark(lidar_coords):
    """What bench.py times: the non-waiting build, weights prepared once, the fused layer at C = 64 on the
    full ~150k-voxel scene, several steps back to back with the maps freed in between; then the
    verdict of the builds and the whole output tensor against the oracle."""
    c = 64
    x_h, w_h = features(300 + c, lidar_coords.shape[0], c, np.float16), conv_weights(301 + c, 27, c, c, np.float16)
    coords, x, w = to_dev(lidar_coords), to_dev(x_h), to_dev(w_h)
    pw = ts.ts_weights_prepare(w)
    out = torch.empty((lidar_coords.shape[0], c), dtype=torch.float16, device="cuda")
    for _ in range(5):
        kmap = ts.ts_build_kmap(coords, 3, 1, wait=False)
        ts.ts_sparse_conv_prepared(x, pw, kmap, out=out)
        kmap.free()
    kmap = ts.ts_build_kmap(coords, 3, 1, wait=False)
    ts.ts_sparse_conv_prepared(x, pw, kmap, out=out)
    kmap.status()
    check_features(out, oracle_conv(lidar_coords, x_h, w_h, 3, 1), torch.float16, "bench configuration")
    _, _, tri = oracle_map(lidar_coords, 3, 1)
    assert np.array_equal(gpu_triples(kmap), tri)


def test_config4_down_up_pair(lidar_coords):
    """2x2x2 stride-2 conv 64->128 onto floor(coord/2), then the transposed conv 128->64 back."""
    dtype = torch.float16
    down = _check_map(lidar_coords, 2, 2)
    up = _check_map(lidar_coords, 2, 2, transposed=True)
    assert down.num_out == up.num_in
    x = features(400, lidar_coords.shape[0], 64, np.float16)
    w_down = conv_weights(401, 8, 64, 128, np.float16, gain=8.0)      # N(0, 1/fan_in), fan_in = 64
    w_up = conv_weights(402, 8, 128, 64, np.float16, gain=8.0)
    # the oracle runs the pair on its own: its down result, rounded to fp16, feeds its up layer
    ref_down = oracle_conv(lidar_coords, x, w_down, 2, 2)
    ref_up = oracle_conv(lidar_coords, oracle.round_to(ref_down, np.float16), w_up, 2, 2, transposed=True)
    for df in (ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH):
        y = ts.ts_sparse_conv(to_dev(x), to_dev(w_down), down, dataflow=df)
        check_features(y, ref_down, dtype, "down")
        # the up layer on the oracle's down result (held to the single-layer bounds), then chained on the
        # library's own (whose one-ulp rounding differences reach small elements of the sum: wider floor)
        z = ts.ts_sparse_conv(to_dev(oracle.round_to(ref_down, np.float16)), to_dev(w_up), up, dataflow=df)
        check_features(z, ref_up, dtype, "up")
        z = ts.ts_sparse_conv(y, to_dev(w_up), up, dataflow=df)
        check_features(z, ref_up, dtype, "up, chained", elem_floor=2e-3)


def test_stages_of_alg2(lidar_coords):
    """Gather, grouped matmul and scatter-accumulate on their own (Alg. 2), C 64->64 fp16."""
    coords = lidar_coords
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    tri = gpu_triples(kmap)                                  # sorted by (n, k, j) = the library's pair order
    sizes = kmap.sizes()
    offs = np.concatenate([[0], np.cumsum(sizes)])
    x = features(500, coords.shape[0], 64, np.float16)
    w = conv_weights(501, 27, 64, 64, np.float16)
    xd, wd = to_dev(x), to_dev(w)
    F = ts.ts_gather(xd, kmap).cpu().numpy()
    keep = tri[:, 2] != 13                                   # centre rows are not materialised
    assert np.array_equal(F[keep], x[tri[keep, 0]])
    G = ts.ts_grouped_matmul(to_dev(F), xd, wd, kmap)
    Gh = G.cpu().numpy().astype(np.float64)
    for n in (0, 4, 13, 22, 26):
        sel = slice(offs[n], offs[n + 1])
        ref = x[tri[sel, 0]].astype(np.float64) @ w[n].astype(np.float64)
        assert oracle.rel_l2(Gh[sel], ref) < 1e-6
    y = ts.ts_scatter_reduce(G, kmap, dtype=torch.float16)
    acc = np.zeros((coords.shape[0], 64))
    np.add.at(acc, tri[:, 1], Gh)
    assert oracle.rel_l2(y.cpu().numpy(), acc.astype(np.float16)) < 2e-3
    check_features(y, oracle_conv(coords, x, w, 3, 1), torch.float16, "staged")


@pytest.mark.parametrize("c,dtype", [(32, torch.float16), (64, torch.float16), (128, torch.float16), (256, torch.float16),
                                     (16, torch.float32), (64, torch.float32), (96, torch.float16)])
@pytest.mark.parametrize("n", [1, 700, 9000])
def test_gather_input_stationary_equals_output_order(c, dtype, n):
    """The locality-aware gather (Sec. 4.3.2: every input row read once, written wherever it is needed) fills
    the buffer F exactly as the output-order gather does, and as the oracle's pair list says: F[p] = X[in(p)]
    for every pair p outside the centre offset.  96 channels has no input-stationary kernel and runs in output
    order; a map of an asynchronous build gets its rank bitmaps on demand."""
    coords = _rand_coords(5000 + n + c, n, -9, 9, batches=2)
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1, wait=(n != 700))
    x_h = features(5100 + c, n, c, np_dtype(dtype))
    x = to_dev(x_h)
    tri = oracle_map(coords, 3, 1)[2]                         # sorted by (n, k, j): the library's pair order
    keep = tri[:, 2] != 13
    outs = []
    for order in (ts.TS_GATHER_INPUT_STATIONARY, ts.TS_GATHER_OUTPUT_ORDER, ts.TS_GATHER_AUTO):
        F = torch.full((kmap.num_pairs, c), -7.0, dtype=dtype, device="cuda")
        ts.ts_gather(x, kmap, F, order=order)
        Fh = F.cpu().numpy()
        assert np.array_equal(Fh[keep], x_h[tri[keep, 0]]), order
        assert (Fh[~keep] == -7.0).all(), "centre rows are not materialised"
        outs.append(Fh)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[1], outs[2])


# ---- grid map search (Sec. 4.4) and Alg. 3's boundary -----------------------------------------------------

@pytest.mark.parametrize("K,s,transposed", MAP_CASES)
@pytest.mark.parametrize("n", [1, 700, 5000])
def test_kmap_grid_search_small(K, s, transposed, n):
    """The grid yields the maps the hash table yields: negative coordinates, three batches, a box with slack."""
    coords = _rand_coords(2000 + n + 10 * K + s, n, -9, 9, batches=3)
    _check_map(coords, K, s, transposed, grid=grid_of(coords, margin=n % 3))


@pytest.mark.parametrize("K,s,transposed", [c for c in MAP_CASES if c[1] > 1])
@pytest.mark.parametrize("n", [1, 37, 5000])
def test_kmap_strided_hash_route(K, s, transposed, n):
    """Strided builds kept on the hash table (candidates sorted); the default measures its box and takes the grid."""
    coords = _rand_coords(2500 + n + 10 * K + s, n, -9, 9, batches=3)
    _check_map(coords, K, s, transposed, search=ts.TS_SEARCH_HASH)


def test_kmap_strided_box_too_large_for_the_grid():
    """Two far-apart clusters: the measured box exceeds what a build takes by itself, so it stays on the hash table."""
    a = _rand_coords(2601, 800, -8, 8)
    b = a.copy()
    b[:, 1:] += 40000
    coords = np.concatenate([a, b])
    for K, s, tr in [(2, 2, False), (3, 2, False), (2, 2, True)]:
        _check_map(coords, K, s, tr)


def test_kmap_strided_wide_box_through_the_bitmap():
    """Two clusters 700 cells apart: 3.7e8 cells of input box, 4.7e7 cells of output box.  The build marks its
    candidates in a bitmap over the output box (no coordinate grid over the input box is involved) and derives
    the map from the ranks of the marked cells; three batches, negative coordinates, a ragged last word."""
    a = _rand_coords(2611, 3000, -10, 10, batches=3)
    b = a.copy()
    b[:, 1:] += 700
    coords = np.concatenate([a, b[:1777]])
    for K, s, tr in MAP_CASES:
        if s > 1:
            _check_map(coords, K, s, tr)
            _check_map(coords, K, s, tr, wait=False)


def test_kmap_strided_duplicates_are_found_on_every_route():
    """Equal input points must be reported whether they share an output entry (forward), own a row each
    (transposed) or lose all their candidates to the boundary."""
    base = _rand_coords(2621, 500, 0, 12)
    dup = np.concatenate([base, base[17:18]])
    for K, s, tr, bnd in [(2, 2, False, None), (3, 2, False, None), (2, 2, True, None), (3, 2, True, None),
                          (3, 2, False, (3, 3, 3)), (3, 2, True, (3, 3, 3))]:
        for search in (ts.TS_SEARCH_AUTO, ts.TS_SEARCH_HASH):
            with pytest.raises(ts.TsError) as e:
                ts.ts_build_kmap(to_dev(dup), K, s, tr, boundary=bnd, search=search)
            assert e.value.code == ts.TS_ERR_DUPLICATE_COORD, (K, s, tr, bnd, search)
    # both copies outside the boundary (every candidate cut): still duplicates
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(np.concatenate([_rand_coords(2622, 50, 0, 4), np.array([[0, 11, 11, 11], [0, 11, 11, 11]], np.int32)])),
                         3, 2, False, boundary=(2, 2, 2))
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
    _check_map(base, 3, 2, boundary=(3, 3, 3))


@pytest.mark.parametrize("K", [2, 3])
def test_kmap_pyramid_with_the_box_handed_down(K):
    """A strided forward build reports a box holding its outputs; the next level's build takes it instead of
    measuring one.  Three levels, each map against the oracle; a box that misses a point is a range error."""
    coords = _rand_coords(2700 + K, 6000, -40, 40, batches=2)
    hint = None
    for level in range(3):
        kmap = ts.ts_build_kmap(to_dev(coords), K, 2, False, wait=False, box=hint)
        in_c, out_c, tri = oracle_map(coords, K, 2)
        assert np.array_equal(kmap.out_coords().cpu().numpy(), out_c)
        assert np.array_equal(gpu_triples(kmap), tri)
        hint = kmap.out_box()
        assert hint is not None
        lo, hi, batches = hint
        assert (out_c[:, 1:] >= np.array(lo)).all() and (out_c[:, 1:] <= np.array(hi)).all() and out_c[:, 0].max() < batches
        # stride-1 builds ignore a stated box on the default route
        sub = ts.ts_build_kmap(to_dev(out_c), 3, 1, box=((0, 0, 0), (0, 0, 0), 1))
        assert np.array_equal(gpu_triples(sub), oracle_map(out_c, 3, 1)[2])
        coords = out_c
    assert ts.ts_build_kmap(to_dev(coords), 3, 1).out_box() is None
    assert ts.ts_build_kmap(to_dev(coords), K, 2, True).out_box() is None
    lo, hi, batches = hint
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(coords), K, 2, False, box=(lo, tuple(h - 3 for h in hi), batches)).status()
    assert e.value.code == ts.TS_ERR_COORD_RANGE


def test_kmap_grid_is_clean_between_builds():
    """The cells are kept between builds: a build must not see the points of the one before, whatever the boxes
    (a smaller one, a larger one that makes the buffer grow, one that is moved), nor after a build that failed."""
    a = _rand_coords(41, 3000, -12, 12, batches=2)
    b = _rand_coords(42, 500, -5, 5)
    c = _rand_coords(43, 4000, -30, 30, batches=2)
    _check_map(a, 3, 1, grid=grid_of(a))
    _check_map(b, 3, 1, grid=grid_of(b))
    _check_map(b, 3, 1, grid=((-12, -12, -12), (12, 12, 12), 2))
    _check_map(c, 3, 2, grid=grid_of(c))
    _check_map(a, 2, 2, True, grid=grid_of(a, margin=2))
    _check_map(a, 3, 1, grid=grid_of(a), wait=False)
    with pytest.raises(ts.TsError) as e:            # a point outside the stated box
        ts.ts_build_kmap(to_dev(a), 3, 1, grid=((-12, -12, -12), (12, 12, 3), 2))
    assert e.value.code == ts.TS_ERR_COORD_RANGE
    _check_map(b, 3, 1, grid=grid_of(a))
    dup = np.concatenate([b, b[:1]])
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(dup), 3, 1, grid=grid_of(b))
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(dup), 2, 2, grid=grid_of(b))
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
    _check_map(b, 3, 1, grid=grid_of(b))
    with pytest.raises(ts.TsError) as e:            # more cells than the library is willing to hold
        ts.ts_build_kmap(to_dev(b), 3, 1, grid=((-5, -5, -5), (60000, 60000, 5), 1))
    assert e.value.code == ts.TS_ERR_UNSUPPORTED
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(b), 3, 1, grid=((5, -5, -5), (-5, 5, 5), 1))
    assert e.value.code == ts.TS_ERR_INVALID_ARG
    ts.ts_release_cache()
    _check_map(a, 3, 1, grid=grid_of(a))


def test_config3_lidar_map_grid(lidar_coords):
    """The full ~150k-voxel scene through the grid (a box of ~3e8 cells)."""
    _check_map(lidar_coords, 3, 1, grid=grid_of(lidar_coords))
    _check_map(lidar_coords, 3, 2, grid=grid_of(lidar_coords))


@pytest.mark.parametrize("K,s,transposed", [(2, 2, False), (3, 2, False), (2, 2, True), (3, 2, True)])
@pytest.mark.parametrize("route", ["auto", "hash", "grid"])
def test_kmap_boundary(K, s, transposed, route):
    """Alg. 3's boundary check: outputs on the grid [0, b) only; inputs beyond it feed nothing."""
    coords = _rand_coords(3000 + 7 * K + transposed, 4000, -6, 22, batches=2)
    b = (8, 11, 5)
    kmap = _check_map(coords, K, s, transposed, grid=grid_of(coords) if route == "grid" else None, boundary=b,
                      search=ts.TS_SEARCH_HASH if route == "hash" else ts.TS_SEARCH_AUTO)
    outs = (kmap.in_coords() if transposed else kmap.out_coords()).cpu().numpy()
    assert outs.shape[0] > 0 and (outs[:, 1:] >= 0).all() and (outs[:, 1:] < np.array(b)).all()
    free = oracle.out_coords(coords, K, s)
    assert outs.shape[0] < free.shape[0]


@pytest.mark.parametrize("K", [2, 3])
def test_transpose_of_a_map_with_boundary(K):
    """ts_kmap_transpose of a forward map built with a boundary: the transposed map the oracle gives for the same
    boundary (fine points all of whose candidates were cut are outputs without a neighbour)."""
    coords = _rand_coords(3200 + K, 3000, -6, 22, batches=2)
    b = (8, 11, 5)
    fwd = ts.ts_build_kmap(to_dev(coords), K, 2, boundary=b)
    tr = fwd.transpose()
    in_c, out_c, tri = oracle_map(coords, K, 2, True, boundary=b)
    assert tr.num_in == in_c.shape[0] and tr.num_out == out_c.shape[0] and tr.num_pairs == tri.shape[0]
    assert np.array_equal(tr.in_coords().cpu().numpy(), in_c)
    assert np.array_equal(tr.out_coords().cpu().numpy(), out_c)
    assert np.array_equal(gpu_triples(tr), tri)
    hit = np.zeros(coords.shape[0], bool)
    hit[tri[:, 1]] = True
    assert 0 < hit.sum() < coords.shape[0]


@pytest.mark.parametrize("seed", range(8))
def test_kmap_random_arguments_all_routes(seed):
    """Seeded random draws over what a build can be asked: size, extent and sign of the coordinates (dense
    blobs to scattered points), batches, (K, s, transposed), a boundary, the search route, waiting or not.
    Every map equals the oracle's, triple for triple."""
    rng = np.random.Generator(np.random.PCG64(8800 + seed))
    for case in range(10):
        K, s, tr = MAP_CASES[int(rng.integers(len(MAP_CASES)))]
        n = int(rng.choice([1, 2, 63, 64, 65, 129, 300, 1000, 2500]))
        side = int(rng.integers(max(2, int(np.ceil(n ** (1 / 3))) + 1), 40))
        lo = int(rng.integers(-30, 10))
        batches = int(rng.integers(1, 5))
        while batches * side ** 3 < n:
            side += 1
        coords = _rand_coords(int(rng.integers(1 << 30)), n, lo, lo + side, batches=batches)
        boundary = None
        if s == 2 and rng.random() < 0.4:
            boundary = tuple(int(v) for v in rng.integers(1, max(2, (lo + side) // 2 + 2), size=3))
        route = ["auto", "hash", "grid"][int(rng.integers(3))]
        wait = bool(rng.integers(2))
        print(f"seed {seed} case {case}: n={n} side={side} lo={lo} batches={batches} K={K} s={s} tr={tr} "
              f"boundary={boundary} route={route} wait={wait}", flush=True)
        _check_map(coords, K, s, tr, grid=grid_of(coords) if route == "grid" else None, boundary=boundary, wait=wait,
                   search=ts.TS_SEARCH_HASH if route == "hash" else ts.TS_SEARCH_AUTO).free()


def test_kmap_boundary_that_cuts_everything():
    coords = _rand_coords(3100, 500, 40, 60)
    for K, s, tr in [(2, 2, False), (3, 2, False), (2, 2, True), (3, 2, True)]:
        kmap = _check_map(coords, K, s, tr, boundary=(4, 4, 4))
        assert kmap.num_pairs == 0
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(coords), 3, 2, boundary=(0, 4, 4))
    assert e.value.code == ts.TS_ERR_INVALID_ARG


@pytest.mark.parametrize("transposed", [False, True])
def test_detector_style_downsampling_layer(transposed):
    """K = 3, s = 2 with a boundary on a LiDAR-like scene (the strided layer of a detection backbone, Sec. 5.1):
    map and features against the oracle, both dataflows."""
    coords = lidar_scan_coords(33, n_beams=32, n_azimuth=1024)
    lo, hi, _ = grid_of(coords)
    b = tuple((h + 1) // 2 * 3 // 4 for h in hi)                 # three quarters of the coarse extent: cuts a rim
    cin, cout = (32, 64) if not transposed else (64, 32)
    kmap = _check_map(coords, 3, 2, transposed, grid=grid_of(coords), boundary=b)
    n_in = kmap.num_in
    x = features(530, n_in, cin, np.float16)
    w = conv_weights(531, 27, cin, cout, np.float16)
    ref = oracle_conv(coords, x, w, 3, 2, transposed, boundary=b)
    for df in (ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH):
        y = ts.ts_sparse_conv(to_dev(x), to_dev(w), kmap, dataflow=df)
        check_features(y, ref, torch.float16, f"detector-style layer, dataflow {df}")


def _expected_launches(sizes, centre, eps, S):
    """Launch count of Appendix B, Alg. 4 from the oracle's partition (empty launches are not made)."""
    K3 = len(sizes)
    if eps < 0:
        return int(np.count_nonzero(sizes))
    idx = list(range(K3 // 2)) if centre >= 0 else list(range(K3))
    launches = 0
    for members in oracle.adaptive_groups([sizes[i] for i in idx], eps):
        n_max = max(sizes[i] for i in members)
        if n_max == 0:
            continue
        launches += 1 if n_max < S else sum(1 for i in members if sizes[i] > 0)
    return launches + (1 if centre >= 0 and sizes[centre] > 0 else 0)


@pytest.mark.parametrize("K,s", [(3, 1), (2, 2), (3, 2)])
def test_adaptive_grouping_same_result_in_the_launches_of_alg4(K, s):
    """Sec. 4.2.3 / Appendix B, Alg. 4: whatever the tolerance and the threshold, the partial sums are those of
    the single launch, bit for bit; the launches made and the padded rows follow the oracle's partition."""
    coords = lidar_scan_coords(31, n_beams=32, n_azimuth=1024)
    kmap = ts.ts_build_kmap(to_dev(coords), K, s)
    sizes = kmap.sizes()
    centre = 13 if (K, s) == (3, 1) else -1
    x = to_dev(features(520, coords.shape[0], 32, np.float16))
    w = to_dev(conv_weights(521, K ** 3, 32, 64, np.float16))
    F = ts.ts_gather(x, kmap)
    G = ts.ts_grouped_matmul(F, x if centre >= 0 else None, w, kmap)
    for eps, S in [(-1.0, 0), (0.0, 0), (0.0, 1 << 40), (0.3, 1 << 40), (0.5, int(np.median(sizes))), (1.0, 1 << 40), (1.0, 0)]:
        G2 = torch.full_like(G, float("nan"))
        G2, stats = ts.ts_grouped_matmul_adaptive(F, x if centre >= 0 else None, w, kmap, eps, S, G2)
        assert torch.equal(G, G2), (eps, S)
        assert stats["rows"] == kmap.num_pairs
        assert stats["launches"] == _expected_launches(sizes, centre, eps, S), (eps, S, stats)
        assert stats["padded_rows"] >= kmap.num_pairs
        if eps <= 0 or S == 0:
            assert stats["padded_rows"] == kmap.num_pairs            # equal sizes or no batching: nothing padded
    if centre >= 0:
        _, stats = ts.ts_grouped_matmul_adaptive(F, x, w, kmap, 1.0, 1 << 40)
        assert stats["launches"] == 2 and stats["padded_rows"] == 26 * int(sizes[:13].max()) + int(sizes[13])


@pytest.mark.parametrize("c", [32, 64, 128, 96])
def test_layers_on_a_map_nobody_waited_for(c):
    """A 3x3x3 stride-1 map from the asynchronous build, used in every order: fused first, fused again, explicit,
    accessors, an epilogue, sorted rows; whatever the build put off runs when it is first needed."""
    coords = lidar_scan_coords(35, n_beams=32, n_azimuth=1024)
    n = coords.shape[0]
    x_h, w_h = features(620 + c, n, c, np.float16), conv_weights(621 + c, 27, c, c, np.float16)
    x, w = to_dev(x_h), to_dev(w_h)
    ref = oracle_conv(coords, x_h, w_h, 3, 1)
    bias = to_dev(features(622, 1, c, np.float16)[0])
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1, wait=False)
    y1 = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_FUSED)
    check_features(y1, ref, torch.float16, "first fused layer")
    y2 = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_FUSED)
    assert torch.equal(y1, y2)
    y3 = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_EXPLICIT)
    check_features(y3, ref, torch.float16, "explicit afterwards")
    kmap.status()
    tri = oracle_map(coords, 3, 1)[2]
    assert np.array_equal(gpu_triples(kmap), tri)
    # with an epilogue, and a map used by the explicit dataflow or an accessor first
    k2 = ts.ts_build_kmap(to_dev(coords), 3, 1, wait=False)
    ya = ts.ts_sparse_conv_act(x, w, k2, bias=bias, relu=True)
    kw = ts.ts_build_kmap(to_dev(coords), 3, 1)
    assert torch.equal(ya, ts.ts_sparse_conv_act(x, w, kw, bias=bias, relu=True))
    k3 = ts.ts_build_kmap(to_dev(coords), 3, 1, wait=False)
    check_features(ts.ts_sparse_conv(x, w, k3, dataflow=ts.TS_DATAFLOW_EXPLICIT), ref, torch.float16, "explicit first")
    k4 = ts.ts_build_kmap(to_dev(coords), 3, 1, wait=False)
    assert k4.num_pairs == tri.shape[0]
    assert torch.equal(ts.ts_sparse_conv(x, w, k4, dataflow=ts.TS_DATAFLOW_FUSED), y1)
    k5 = ts.ts_build_kmap(to_dev(coords), 3, 1, wait=False).sort_rows()
    check_features(ts.ts_sparse_conv(x, w, k5, dataflow=ts.TS_DATAFLOW_FUSED), ref, torch.float16, "sorted rows on an asynchronous build")


def test_layer_on_an_asynchronous_build_with_bad_input():
    small = _rand_coords(62, 2000, -10, 10, batches=2)
    dup = np.concatenate([small, small[:1]])
    x = to_dev(features(630, dup.shape[0], 32, np.float16))
    w = to_dev(conv_weights(631, 27, 32, 32, np.float16))
    m = ts.ts_build_kmap(to_dev(dup), 3, 1, wait=False)
    ts.ts_sparse_conv(x, w, m, dataflow=ts.TS_DATAFLOW_FUSED)                  # runs (results meaningless), must not fault
    with pytest.raises(ts.TsError) as e:
        m.status()
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
    m.free()
    far = small.copy()
    far[3, 1] = ts.TS_COORD_MAX + 5
    m = ts.ts_build_kmap(to_dev(far), 3, 1, wait=False)
    ts.ts_sparse_conv(x[:2000].contiguous(), w, m, dataflow=ts.TS_DATAFLOW_FUSED)
    with pytest.raises(ts.TsError) as e:
        m.status()
    assert e.value.code == ts.TS_ERR_COORD_RANGE


def test_prepare_after_an_asynchronous_build(lidar_coords):
    """ts_kmap_prepare enqueues the put-off row pass of asynchronous builds; the maps, their sizes and the
    verdicts are those of the waiting build, also when several builds are prepared before any is asked."""
    small = _rand_coords(61, 3000, -10, 10, batches=2)
    dup = np.concatenate([small, small[:1]])
    ms = [ts.ts_build_kmap(to_dev(c), 3, 1, wait=False) for c in (lidar_coords, small, dup, small[:1])]
    for m in ms:
        m.prepare()
    for m in ms:
        m.prepare()                                   # a second call has nothing left to do
    for m, c in zip(ms, (lidar_coords, small, dup, small[:1])):
        if c is dup:
            with pytest.raises(ts.TsError) as e:
                m.status()
            assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
            continue
        m.status()
        tri = oracle_map(c, 3, 1)[2]
        assert m.num_pairs == tri.shape[0]
        assert np.array_equal(m.sizes(), np.bincount(tri[:, 2], minlength=27))
        assert np.array_equal(gpu_triples(m), tri)
    x = to_dev(features(610, small.shape[0], 32, np.float16))
    w = to_dev(conv_weights(611, 27, 32, 32, np.float16))
    ref = oracle_conv(small, x.cpu().numpy(), w.cpu().numpy(), 3, 1)
    for df in (ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH):
        check_features(ts.ts_sparse_conv(x, w, ms[1], dataflow=df), ref, torch.float16, f"prepared map, dataflow {df}")


def test_group_search_on_the_device():
    """Appendix B, Alg. 5 with the measured cost: the pair it returns is the cheapest of its own table."""
    from paper_2204_10319_amd import tuner
    coords = lidar_scan_coords(34, n_beams=16, n_azimuth=512)
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    x = to_dev(features(540, coords.shape[0], 32, np.float16))
    w = to_dev(conv_weights(541, 27, 32, 32, np.float16))
    F = ts.ts_gather(x, kmap)
    G = torch.empty((kmap.num_pairs, 32), dtype=torch.float32, device="cuda")
    eps, S, cost, table = tuner.adaptive_group_search([(F, x, w, kmap, G)], eps_space=(0.0, 0.5, 1.0), S_space=(0, 1 << 40),
                                                      cost=tuner.measured_cost(iters=3, warmup=1))
    assert len(table) == 6 and (eps, S) in table and cost == min(table.values()) and cost > 0
    assert torch.equal(G, ts.ts_grouped_matmul(F, x, w, kmap))


def test_reference_kernels_of_the_benchmark():
    """The copy and MFMA-loop kernels bench.py measures achievable rates with."""
    src = torch.arange(1 << 18, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    ts.ts_copy_bytes(dst, src)
    assert torch.equal(dst, src)
    sink = torch.zeros(1 << 18, dtype=torch.float32, device="cuda")
    flops = ts.ts_mfma_loop(16, sink)
    torch.cuda.synchronize()
    assert flops == 1024 * 4 * 16 * 8 * 2 * 16 * 16 * 32
    assert float(sink.abs().sum()) == 0.0


def test_results_are_deterministic(lidar_coords):
    kmap_a = ts.ts_build_kmap(to_dev(lidar_coords), 3, 1)
    kmap_b = ts.ts_build_kmap(to_dev(lidar_coords), 3, 1)
    pa, pb = kmap_a.pairs(), kmap_b.pairs()
    assert torch.equal(pa[0], pb[0]) and torch.equal(pa[1], pb[1])
    x = to_dev(features(600, lidar_coords.shape[0], 64, np.float16))
    w = to_dev(conv_weights(601, 27, 64, 64, np.float16))
    for df in (ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH):
        y1 = ts.ts_sparse_conv(x, w, kmap_a, dataflow=df)
        y2 = ts.ts_sparse_conv(x, w, kmap_b, dataflow=df)
        assert torch.equal(y1, y2)


def test_row_order_independence():
    coords = uniform_grid_coords(7, n=4000, grid=20)
    x = features(700, 4000, 32, np.float16)
    w = conv_weights(701, 27, 32, 32, np.float16)
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    y = ts.ts_sparse_conv(to_dev(x), to_dev(w), kmap).cpu().numpy()
    perm = np.random.Generator(np.random.PCG64(3)).permutation(4000)
    kmap_p = ts.ts_build_kmap(to_dev(coords[perm]), 3, 1)
    yp = ts.ts_sparse_conv(to_dev(x[perm]), to_dev(w), kmap_p).cpu().numpy()
    assert oracle.rel_l2(yp, y[perm]) < 1e-3


@pytest.mark.parametrize("K,s,transposed", [(3, 1, False), (2, 2, False), (2, 2, True)])
def test_sorted_rows_give_the_same_result(lidar_coords, K, s, transposed):
    """ts_kmap_sort_rows only regroups the output rows: every row's sum keeps its order, so the
    outputs are equal bit for bit; pairs and sizes are untouched; a second call is a no-op."""
    coords = lidar_coords[:60000]
    plain = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    grouped = ts.ts_build_kmap(to_dev(coords), K, s, transposed).sort_rows().sort_rows()
    assert np.array_equal(gpu_triples(plain), gpu_triples(grouped))
    for c_in, c_out in ((32, 64), (128, 128)):
        x = to_dev(features(800 + c_in, plain.num_in, c_in, np.float16))
        w = to_dev(conv_weights(801 + c_in, K ** 3, c_in, c_out, np.float16))
        y1 = ts.ts_sparse_conv(x, w, plain, dataflow=ts.TS_DATAFLOW_FUSED)
        y2 = ts.ts_sparse_conv(x, w, grouped, dataflow=ts.TS_DATAFLOW_FUSED)
        assert torch.equal(y1, y2)
    ref = oracle_conv(coords, features(832, plain.num_in, 32, np.float16), conv_weights(833, K ** 3, 32, 64, np.float16),
                      K, s, transposed)
    check_features(ts.ts_sparse_conv(to_dev(features(832, plain.num_in, 32, np.float16)),
                                     to_dev(conv_weights(833, K ** 3, 32, 64, np.float16)), grouped), ref, torch.float16,
                   "sorted rows")


def test_sorted_rows_many_distinct_masks():
    """Uniform random occupancy gives more distinct bitmasks than the mask table ranks (the radix-sort path)."""
    coords = _rand_coords(91, 120000, 0, 64)
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    x = to_dev(features(900, kmap.num_in, 32, np.float16))
    w = to_dev(conv_weights(901, 27, 32, 32, np.float16))
    y1 = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_FUSED)
    kmap.sort_rows()
    y2 = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_FUSED)
    assert torch.equal(y1, y2)
    y3 = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_EXPLICIT)
    assert oracle.rel_l2(y3.cpu().numpy(), y1.cpu().numpy()) < 1e-3


@pytest.mark.parametrize("n", [1, 63, 64, 65, 1000, 40000])
def test_identity_map_is_the_1x1x1_map_of_distinct_points(n):
    """ts_identity_kmap(n) = what the search finds for K = 1, s = 1 on n distinct points (Eq. 1 with delta = 0):
    same triples as the oracle's map, same sizes, and every dataflow gives the oracle's layer on it."""
    coords = _rand_coords(900 + n, n, -20, 20, batches=2)
    ident = ts.ts_identity_kmap(n)
    assert (ident.num_in, ident.num_out, ident.num_pairs, ident.kernel_volume) == (n, n, n, 1)
    _, _, want = oracle_map(coords, 1, 1)
    assert np.array_equal(gpu_triples(ident), want)
    assert ident.sizes().tolist() == [n]
    searched = ts.ts_build_kmap(to_dev(coords), 1, 1)
    for dtype in (torch.float16, torch.float32):
        nd = np_dtype(dtype)
        x = features(901, n, 48, nd)
        w = conv_weights(902, 1, 48, 64, nd)
        ref = oracle_conv(coords, x, w, 1, 1)
        for df in (ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH, ts.TS_DATAFLOW_AUTO):
            y = ts.ts_sparse_conv(to_dev(x), to_dev(w), ident, dataflow=df)
            check_features(y, ref, dtype, f"identity map, dataflow {df}")
            assert torch.equal(y, ts.ts_sparse_conv(to_dev(x), to_dev(w), searched, dataflow=df))
    ident.sort_rows()
    ident.prepare().status()
    with pytest.raises(ts.TsError):
        ident.out_coords()
    with pytest.raises(ts.TsError):
        ident.in_coords()
    with pytest.raises(ts.TsError):
        ident.transpose()
    ident.free()


def test_identity_map_of_nothing():
    m = ts.ts_identity_kmap(0)
    assert (m.num_in, m.num_out, m.num_pairs) == (0, 0, 0)
    x = torch.zeros((0, 32), dtype=torch.float16, device="cuda")
    w = torch.zeros((1, 32, 32), dtype=torch.float16, device="cuda")
    assert ts.ts_sparse_conv(x, w, m).shape == (0, 32)
    with pytest.raises(ts.TsError):
        ts.ts_identity_kmap(-1)


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("ca,cb,skip", [(96, 32, 0), (32, 256, 0), (20, 12, 0), (8, 8, 1), (4, 36, 3)])
def test_concat_cols_is_a_copy(dtype, ca, cb, skip):
    """ts_concat_cols moves bits (skip connections of a U-Net): whole 16-byte vectors where widths and
    addresses allow, element by element otherwise (odd widths; views that start off a 16-byte boundary)."""
    g = torch.Generator().manual_seed(ca * 100 + cb)
    a = torch.randn((1003 + skip, ca), generator=g).to(dtype).cuda()[skip:]
    b = torch.randn((1003 + skip, cb), generator=g).to(dtype).cuda()[skip:]
    assert torch.equal(ts.ts_concat_cols(a, b), torch.cat([a, b], dim=1))
    empty = ts.ts_concat_cols(a[:0], b[:0])
    assert empty.shape == (0, ca + cb)


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("c_in", [1, 3, 4, 9, 17, 40])
def test_layer_with_input_channels_that_need_padding(dtype, c_in):
    """C_in that is not a multiple of the operand step is zero-extended by the library (16-byte stores of
    8 elements): every dataflow against the oracle."""
    coords = _rand_coords(808 + c_in, 1100, -6, 6, batches=2)
    _layer_case(coords, c_in, 32, 3, 1, False, dtype, seed=800 + c_in)


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("K,s,transposed,c_in,c_out", [(3, 1, False, 64, 64), (3, 2, False, 24, 96), (2, 2, True, 256, 128), (1, 1, False, 128, 32)])
def test_fetch_dataflow_gives_the_bits_of_the_explicit_one(dtype, K, s, transposed, c_in, c_out):
    """TS_DATAFLOW_FETCH is Alg. 2 with the gather folded into the matmul: same products, same sums in the same
    order as the three-launch form; also as the first use of a map nobody waited for."""
    coords = _rand_coords(515 + K, 5000, -12, 12, batches=2)
    nd = np_dtype(dtype)
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    x = to_dev(features(516, kmap.num_in, c_in, nd))
    w = to_dev(conv_weights(517, K ** 3, c_in, c_out, nd))
    want = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_EXPLICIT)
    assert torch.equal(ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_FETCH), want)
    if not transposed:
        lazy = ts.ts_build_kmap(to_dev(coords), K, s, wait=False)
        assert torch.equal(ts.ts_sparse_conv(x, w, lazy, dataflow=ts.TS_DATAFLOW_FETCH), want)
    check_features(want, oracle_conv(coords, x.cpu().numpy(), w.cpu().numpy(), K, s, transposed), dtype, "fetch dataflow")


@pytest.mark.parametrize("K,s,transposed", [(3, 1, False), (2, 2, False), (2, 2, True), (1, 1, False)])
@pytest.mark.parametrize("c_in,c_out", [(32, 32), (4, 32), (32, 64)])
def test_narrow_layer_with_more_work_than_resident_waves(K, s, transposed, c_in, c_out):
    """C_in <= 32 -> C_out = 32 or 64 in fp16 on a 3x3x3 map runs in the kernel that keeps all weights in LDS
    and hands 32-row units to waves: enough rows here that units come out of the counters too; rows in input
    order and sorted by bitmask; with the epilogue; twice on one map (the counters rearm).  The other maps
    take the tile kernel on the same inputs."""
    coords = _rand_coords(4242 + K, 160000, 0, 90, batches=2)
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    assert kmap.num_out > 256 * 12 * 32 or K == 2 and not transposed
    x = features(77, kmap.num_in, c_in, np.float16)
    w = conv_weights(78, K ** 3, c_in, c_out, np.float16)
    ref = oracle_conv(coords, x, w, K, s, transposed)
    xd, wd = to_dev(x), to_dev(w)
    y = ts.ts_sparse_conv(xd, wd, kmap, dataflow=ts.TS_DATAFLOW_FUSED)
    check_features(y, ref, torch.float16, f"narrow layer K{K} s{s} t{transposed} C{c_in}")
    assert torch.equal(y, ts.ts_sparse_conv(xd, wd, kmap, dataflow=ts.TS_DATAFLOW_FUSED))
    assert oracle.rel_l2(ts.ts_sparse_conv(xd, wd, kmap, dataflow=ts.TS_DATAFLOW_FUSED_STAGED).cpu().numpy(), y.cpu().numpy()) < 1e-3
    bias = to_dev(features(79, 1, c_out, np.float16).reshape(-1))
    res = to_dev(features(80, kmap.num_out, c_out, np.float16))
    want = ts.ts_bias_act(y.clone(), bias, res, True)
    assert torch.equal(ts.ts_sparse_conv_act(xd, wd, kmap, bias, res, True), want)
    kmap.sort_rows()
    assert torch.equal(ts.ts_sparse_conv(xd, wd, kmap, dataflow=ts.TS_DATAFLOW_FUSED), y)
    assert torch.equal(ts.ts_sparse_conv_act(xd, wd, kmap, bias, res, True), want)


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("K,s,transposed,c_in,c_out", [(3, 1, False, 32, 64), (2, 2, False, 64, 96), (2, 2, True, 128, 32)])
def test_fused_epilogue_equals_two_calls(dtype, K, s, transposed, c_in, c_out):
    """ts_sparse_conv_act = ts_sparse_conv then ts_bias_act, bit for bit, with every subset of the extras."""
    coords = _rand_coords(55 + K, 3000, -9, 9, batches=2)
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    nd = np_dtype(dtype)
    x = to_dev(features(1000, kmap.num_in, c_in, nd))
    w = to_dev(conv_weights(1001, K ** 3, c_in, c_out, nd))
    bias = to_dev(features(1002, 1, c_out, nd).reshape(-1))
    res = to_dev(features(1003, kmap.num_out, c_out, nd))
    plain = ts.ts_sparse_conv(x, w, kmap)
    for b, r, relu in [(None, None, False), (bias, None, True), (None, res, False), (bias, res, True), (None, None, True)]:
        want = ts.ts_bias_act(plain.clone(), b, r, relu)
        got = ts.ts_sparse_conv_act(x, w, kmap, b, r, relu)
        assert torch.equal(got, want), (b is not None, r is not None, relu)
    ref = oracle_conv(coords, x.cpu().numpy(), w.cpu().numpy(), K, s, transposed)
    y = oracle.round_to(ref, nd).astype(np.float64) + bias.cpu().numpy().astype(np.float64)[None, :] + res.cpu().numpy().astype(np.float64)
    y = np.maximum(y, 0.0)
    # the layer's sum is rounded to the I/O dtype before the elementwise step on both sides: one ulp of it
    # is allowed on top of the element bound
    mag = np.abs(y) + np.abs(bias.cpu().numpy().astype(np.float64))[None, :] + np.abs(res.cpu().numpy().astype(np.float64))
    check_features(ts.ts_sparse_conv_act(x, w, kmap, bias, res, True), y, dtype, "fused epilogue vs oracle", pre_mag=mag)


@pytest.mark.parametrize("seed", range(6))
def test_layer_random_arguments_against_the_oracle(seed):
    """Seeded random draws over what a layer can be asked: map kind, point count, channel widths (multiples of
    32 up to 192, and the narrow 4 / 16-channel inputs the padding path takes), dtype, dataflow, prepared weights
    or not, and any subset of bias / residual / ReLU.  Every result is held to the oracle's with the layer bounds."""
    rng = np.random.Generator(np.random.PCG64(9900 + seed))
    for case in range(6):
        K, s, tr = [(3, 1, False), (2, 2, False), (2, 2, True), (1, 1, False), (3, 2, False), (3, 2, True)][int(rng.integers(6))]
        n = int(rng.choice([1, 100, 129, 1000, 4097, 9000]))
        side = max(int(np.ceil(n ** (1 / 3))) + 1, int(rng.integers(4, 36)))
        coords = _rand_coords(int(rng.integers(1 << 30)), n, -side // 2, -side // 2 + side, batches=int(rng.integers(1, 3)))
        dtype = torch.float16 if rng.random() < 0.75 else torch.float32
        nd = np_dtype(dtype)
        c_in = int(rng.choice([4, 16, 32, 64, 96, 128, 160, 192]))
        c_out = int(rng.choice([32, 64, 96, 128, 192]))
        df = [ts.TS_DATAFLOW_AUTO, ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH][int(rng.integers(4))]
        use_b, use_r, relu, prepared = (bool(rng.integers(2)) for _ in range(4))
        kmap = ts.ts_build_kmap(to_dev(coords), K, s, tr)
        x_h = features(int(rng.integers(1 << 30)), kmap.num_in, c_in, nd)
        w_h = conv_weights(int(rng.integers(1 << 30)), K ** 3, c_in, c_out, nd)
        b_h = features(int(rng.integers(1 << 30)), 1, c_out, nd).reshape(-1)
        r_h = features(int(rng.integers(1 << 30)), kmap.num_out, c_out, nd)
        print(f"seed {seed} case {case}: n={n} side={side} K={K} s={s} tr={tr} {c_in}->{c_out} {dtype} dataflow={df} "
              f"bias={use_b} residual={use_r} relu={relu} prepared={prepared}", flush=True)
        x, w = to_dev(x_h), to_dev(w_h)
        bias = to_dev(b_h) if use_b else None
        res = to_dev(r_h) if use_r else None
        if prepared:        # the library's own choice of dataflow, weights repacked once
            got = ts.ts_sparse_conv_prepared(x, ts.ts_weights_prepare(w), kmap, bias, res, relu)
        elif use_b or use_r or relu:
            got = ts.ts_sparse_conv_act(x, w, kmap, bias, res, relu)
        else:
            got = ts.ts_sparse_conv(x, w, kmap, dataflow=df)
        y = oracle.round_to(oracle_conv(coords, x_h, w_h, K, s, tr), nd).astype(np.float64)
        mag = np.abs(y)
        if use_b:
            y = y + b_h.astype(np.float64)[None, :]
            mag = mag + np.abs(b_h.astype(np.float64))[None, :]
        if use_r:
            y = y + r_h.astype(np.float64)
            mag = mag + np.abs(r_h.astype(np.float64))
        if relu:
            y = np.maximum(y, 0.0)
        check_features(got, y, dtype, f"seed {seed} case {case}", pre_mag=mag if (use_b or use_r or relu) else None)
        kmap.free()


@pytest.mark.parametrize("K", [1, 2, 3])
@pytest.mark.parametrize("n", [1, 700, 20000])
def test_transposed_map_derived_from_forward_map(K, n):
    """ts_kmap_transpose(forward map) is the map ts_build_kmap(..., transposed=1) searches for."""
    coords = _rand_coords(300 + n + K, n, -20, 20, batches=2)
    fwd = ts.ts_build_kmap(to_dev(coords), K, 2, False)
    built = ts.ts_build_kmap(to_dev(coords), K, 2, True)
    derived = fwd.transpose()
    _, _, tri = oracle_map(coords, K, 2, True)
    assert derived.num_in == built.num_in and derived.num_out == built.num_out and derived.num_pairs == built.num_pairs
    assert torch.equal(derived.in_coords(), built.in_coords()) and torch.equal(derived.out_coords(), built.out_coords())
    assert np.array_equal(derived.sizes(), built.sizes())
    assert np.array_equal(gpu_triples(derived), tri)
    pa, pb = derived.pairs(), built.pairs()
    assert torch.equal(pa[0], pb[0]) and torch.equal(pa[1], pb[1])
    x = to_dev(features(310, built.num_in, 64, np.float16))
    w = to_dev(conv_weights(311, K ** 3, 64, 32, np.float16))
    for df in (ts.TS_DATAFLOW_FUSED, ts.TS_DATAFLOW_EXPLICIT, ts.TS_DATAFLOW_FETCH):
        assert torch.equal(ts.ts_sparse_conv(x, w, derived, dataflow=df), ts.ts_sparse_conv(x, w, built, dataflow=df))
    fwd.free()   # the derived map does not depend on the forward map's memory
    assert torch.equal(ts.ts_sparse_conv(x, w, derived), ts.ts_sparse_conv(x, w, built))


def test_transpose_rejects_other_maps():
    ok = to_dev(_rand_coords(5, 100, 0, 6))
    for K, s, tr in [(3, 1, False), (2, 2, True)]:
        with pytest.raises(ts.TsError) as e:
            ts.ts_build_kmap(ok, K, s, tr).transpose()
        assert e.value.code == ts.TS_ERR_INVALID_ARG


@pytest.mark.parametrize("transposed", [False, True])
def test_strided_map_without_outputs(transposed):
    """K = 1, s = 2 on odd coordinates: no candidate passes the modular check of Alg. 3, the map has no pairs."""
    coords = np.array([[0, 1, 3, 5], [0, 7, 1, 1], [1, 3, 3, 3]], dtype=np.int32)
    kmap = _check_map(coords, 1, 2, transposed)
    assert kmap.num_pairs == 0
    x = to_dev(features(5, kmap.num_in, 32, np.float16))
    y = ts.ts_sparse_conv(x, to_dev(conv_weights(6, 1, 32, 32, np.float16)), kmap)
    assert y.shape == (kmap.num_out, 32) and not y.any()
    dup = np.array([[0, 1, 3, 5], [0, 1, 3, 5]], dtype=np.int32)
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(dup), 1, 2, transposed)
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("K,s,transposed,c_in,c_out,n", [(3, 1, False, 32, 64, 5000), (3, 1, False, 4, 32, 3000),
                                                          (2, 2, False, 64, 96, 4000), (2, 2, True, 256, 256, 3000),
                                                          (1, 1, False, 160, 96, 2000)])
def test_prepared_weights_give_the_same_result(dtype, K, s, transposed, c_in, c_out, n):
    coords = _rand_coords(66 + K + n, n, -9, 9, batches=2)
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    nd = np_dtype(dtype)
    x = to_dev(features(1100, kmap.num_in, c_in, nd))
    w = to_dev(conv_weights(1101, K ** 3, c_in, c_out, nd))
    bias = to_dev(features(1102, 1, c_out, nd).reshape(-1))
    res = to_dev(features(1103, kmap.num_out, c_out, nd))
    pw = ts.ts_weights_prepare(w)
    w_copy = w.clone()
    w.zero_()                                  # the prepared copy does not depend on the caller's tensor
    torch.cuda.synchronize()
    assert torch.equal(ts.ts_sparse_conv_prepared(x, pw, kmap), ts.ts_sparse_conv(x, w_copy, kmap))
    assert torch.equal(ts.ts_sparse_conv_prepared(x, pw, kmap, bias, res, True), ts.ts_sparse_conv_act(x, w_copy, kmap, bias, res, True))
    other = ts.ts_build_kmap(to_dev(coords), 1 if K != 1 else 3, 1)
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv_prepared(x, pw, other)
    assert e.value.code == ts.TS_ERR_SHAPE
    pw.free()


@pytest.mark.parametrize("K,s,transposed", [(3, 1, False), (1, 1, False), (2, 2, False), (2, 2, True)])
def test_async_build(K, s, transposed):
    """ts_build_kmap_async: same map, same layer output; a layer can run before anybody asked for the sizes."""
    coords = _rand_coords(400 + K, 6000, -12, 12, batches=2)
    sync = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    x = to_dev(features(410, sync.num_in, 32, np.float16))
    w = to_dev(conv_weights(411, K ** 3, 32, 64, np.float16))
    want = ts.ts_sparse_conv(x, w, sync, dataflow=ts.TS_DATAFLOW_FUSED)
    lazy = ts.ts_build_kmap(to_dev(coords), K, s, transposed, wait=False)
    got = ts.ts_sparse_conv(x, w, lazy, dataflow=ts.TS_DATAFLOW_FUSED)     # before any accessor
    assert torch.equal(got, want)
    lazy.status()
    assert lazy.num_pairs == sync.num_pairs and np.array_equal(lazy.sizes(), sync.sizes())
    assert np.array_equal(gpu_triples(lazy), gpu_triples(sync))
    assert torch.equal(ts.ts_sparse_conv(x, w, lazy, dataflow=ts.TS_DATAFLOW_EXPLICIT), ts.ts_sparse_conv(x, w, sync, dataflow=ts.TS_DATAFLOW_EXPLICIT))


def test_async_build_reports_bad_input_late():
    dup = np.concatenate([_rand_coords(5, 500, 0, 10), np.array([[0, 1, 2, 3], [0, 1, 2, 3]], np.int32)])
    kmap = ts.ts_build_kmap(to_dev(dup), 3, 1, wait=False)          # no error yet
    x = to_dev(features(1, dup.shape[0], 32, np.float16))
    w = to_dev(conv_weights(2, 27, 32, 32, np.float16))
    y = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_FUSED)   # runs, result meaningless but finite
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
    with pytest.raises(ts.TsError) as e:
        kmap.status()
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
    assert kmap.num_pairs == -1
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv(x, w, kmap)
    assert e.value.code == ts.TS_ERR_DUPLICATE_COORD
    far = np.array([[0, 1, 2, 3], [0, ts.TS_COORD_MAX + 1, 0, 0]], dtype=np.int32)
    with pytest.raises(ts.TsError) as e:
        ts.ts_build_kmap(to_dev(far), 3, 1, wait=False).status()
    assert e.value.code == ts.TS_ERR_COORD_RANGE
    # many maps whose sizes nobody asks for: the status slots are recycled
    ok = to_dev(_rand_coords(6, 300, 0, 8))
    maps = [ts.ts_build_kmap(ok, 3, 1, wait=False) for _ in range(200)]
    del maps
    fresh = ts.ts_build_kmap(ok, 3, 1, wait=False)
    assert fresh.num_pairs == ts.ts_build_kmap(ok, 3, 1).num_pairs


# ---- a layer on a two-part input (the skip connection of a U-Net decoder), the concatenation never formed ----

@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("K,s,transposed", [(3, 1, False), (1, 1, False), (2, 2, True), (2, 2, False)])
@pytest.mark.parametrize("c1,c2,c_out", [(96, 32, 96), (96, 64, 96), (128, 128, 128), (32, 96, 64), (64, 64, 32),
                                          (48, 16, 32), (24, 40, 64), (256, 256, 256)])
def test_two_part_input_equals_the_concatenated_input(dtype, K, s, transposed, c1, c2, c_out):
    """ts_sparse_conv_prepared2(a, b) against ts_sparse_conv_prepared([a | b]) bit for bit, and against the
    oracle on the concatenated input; widths the kernels read in place (multiples of 32), widths only the
    fetch-on-demand dataflow reads in place (multiples of 16 / 8: wide layers on few points take it), and
    widths that are concatenated in scratch (24 + 40); with and without the elementwise tail."""
    n = 600 if c1 + c2 >= 256 else 2500          # few points + wide layers: the library takes fetch-on-demand
    coords = _rand_coords(4000 + c1 + 3 * c2 + K, n, -8, 8, batches=2)
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    nd = np_dtype(dtype)
    a_h, b_h = features(4100 + c1, kmap.num_in, c1, nd), features(4200 + c2, kmap.num_in, c2, nd)
    w_h = conv_weights(4300 + c_out, K ** 3, c1 + c2, c_out, nd)
    a, b, w = to_dev(a_h), to_dev(b_h), to_dev(w_h)
    cat_h = np.concatenate([a_h, b_h], axis=1)
    cat = to_dev(cat_h)
    pw = ts.ts_weights_prepare(w)
    bias = to_dev(features(4400, 1, c_out, nd).reshape(-1))
    res = to_dev(features(4401, kmap.num_out, c_out, nd))
    for bb, rr, relu in [(None, None, False), (bias, res, True)]:
        want = ts.ts_sparse_conv_prepared(cat, pw, kmap, bb, rr, relu)
        got = ts.ts_sparse_conv_prepared2(a, b, pw, kmap, bb, rr, relu)
        assert torch.equal(got, want), (c1, c2, c_out, relu)
    assert torch.equal(ts.ts_sparse_conv_prepared2(cat, None, pw, kmap), ts.ts_sparse_conv_prepared(cat, pw, kmap))
    check_features(ts.ts_sparse_conv_prepared2(a, b, pw, kmap), oracle_conv(coords, cat_h, w_h, K, s, transposed), dtype,
                   f"two-part input {c1}+{c2}->{c_out} K{K} s{s} t{int(transposed)}")


def test_two_part_input_errors():
    coords = _rand_coords(4500, 300, 0, 8)
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    a = torch.zeros((300, 32), dtype=torch.float16, device="cuda")
    pw = ts.ts_weights_prepare(torch.zeros((27, 64, 32), dtype=torch.float16, device="cuda"))
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv_prepared2(a, torch.zeros((299, 32), dtype=torch.float16, device="cuda"), pw, kmap)
    assert e.value.code == ts.TS_ERR_SHAPE
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv_prepared2(a, torch.zeros((300, 32), dtype=torch.float32, device="cuda"), pw, kmap)
    assert e.value.code == ts.TS_ERR_SHAPE
    with pytest.raises(ts.TsError) as e:
        ts.ts_sparse_conv_prepared2(a, torch.zeros((300, 64), dtype=torch.float16, device="cuda"), pw, kmap)
    assert e.value.code == ts.TS_ERR_SHAPE          # 32 + 64 channels against weights prepared for 64


def test_callers_allocator_owns_the_librarys_memory():
    """ts_set_allocator: with PyTorch's caching allocator behind it the library's maps, temporaries and scratch
    show up in torch's statistics, results are the ones the library's own pool gives, and everything goes back
    when the maps are freed; maps made under one setting are released correctly under the other."""
    coords = _rand_coords(6000, 20000, -30, 30, batches=2)
    x_h, w_h = features(6001, 20000, 64, np.float16), conv_weights(6002, 27, 64, 96, np.float16)
    x, w, cd = to_dev(x_h), to_dev(w_h), to_dev(coords)
    own = ts.ts_build_kmap(cd, 3, 1)
    want = ts.ts_sparse_conv(x, w, own, dataflow=ts.TS_DATAFLOW_EXPLICIT)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ts.use_torch_allocator(True)
    try:
        theirs = ts.ts_build_kmap(cd, 3, 1)
        down = ts.ts_build_kmap(cd, 2, 2, wait=False)
        assert torch.cuda.memory_allocated() > before + 20000 * 128      # at least the neighbour table
        got = ts.ts_sparse_conv(x, w, theirs, dataflow=ts.TS_DATAFLOW_EXPLICIT)
        assert torch.equal(got, want)
        assert np.array_equal(gpu_triples(theirs), oracle_map(coords, 3, 1)[2])
        assert np.array_equal(gpu_triples(down), oracle_map(coords, 2, 2)[2])
        own.free()                      # a block of the library's pool, released while the caller's allocator is set
    finally:
        ts.use_torch_allocator(False)
    theirs.free()                       # and the other way round
    down.free()
    del got
    torch.cuda.synchronize()
    ts.ts_release_cache()
    # what remains allocated in torch: this test's own tensors only (scratch areas taken from torch went back with the cache)
    assert torch.cuda.memory_allocated() <= before + want.numel() * 2 + 4096
    check_features(ts.ts_sparse_conv(x, w, ts.ts_build_kmap(cd, 3, 1)), oracle_conv(coords, x_h, w_h, 3, 1), torch.float16, "after the switch back")
