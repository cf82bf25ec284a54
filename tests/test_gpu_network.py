"""Config 5: the MinkUNet-style forward pass, GPU library vs. CPU oracle, tensor by tensor.

The oracle runs the whole network on its own (no value of the GPU run enters it); every
intermediate tensor and the output are compared.  The end-to-end value has no closed form:
it is pinned only through the per-layer pins of the oracle ("parity unpinned" beyond that).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2204_10319_amd import binding as ts
from paper_2204_10319_amd.network import SparseNet
from workloads import lidar_scan_coords, features
from workloads.minkunet import build_plan, make_params
from _net_oracle import run_plan
from _util import to_dev, check_features

pytestmark = pytest.mark.gpu


def _run_both(coords, seed, box=None):
    ops, output = build_plan(4)
    params = make_params(seed, ops)
    x = features(seed + 1, coords.shape[0], 4, np.float16)
    ref = {}
    y_ref, levels = run_plan(ops, output, params, coords, x, hook=lambda n, v: ref.__setitem__(n, v))
    net = SparseNet(ops, output, {k: (to_dev(w), to_dev(b)) for k, (w, b) in params.items()})
    maps, dev_levels = net.build_maps(to_dev(coords), box=box)
    for level, c in levels.items():
        assert np.array_equal(dev_levels[level].cpu().numpy(), c), f"level {level} coordinates"
    got = {}
    y = net.forward(maps, to_dev(x), hook=lambda n, v: got.__setitem__(n, v.cpu().numpy()))
    torch.cuda.synchronize()
    # without a hook nobody asks for the concatenated tensors: the layers behind a skip connection read its two
    # parts in place, and the pass must give the same bits
    y_plain = net.forward(maps, to_dev(x))
    assert torch.equal(y_plain, y), "the concat-free pass differs from the pass that forms the concatenations"
    # (1) the free-running pass: every tensor within the stated norm; its rows within ten times that (the
    # two runs have drifted apart by the rounding differences of up to 45 layers, so rows are not held to
    # the single-layer bound here; a row that lost a neighbour term is off by tens of percent)
    worst = 0.0
    for name, r in ref.items():
        g = got[name]
        assert g.shape == r.shape, name
        assert np.isfinite(g.astype(np.float64)).all(), name
        rms = float(np.sqrt(np.mean(r.astype(np.float64) ** 2)))
        assert 2.0 ** -6 < rms < 2.0 ** 6, f"{name}: activation RMS {rms} out of the fp16 comfort range"
        err = oracle.rel_l2(g, r)
        worst = max(worst, err)
        assert err <= 2e-3, f"{name}: relative L2 error {err:.3e}"
        rows = oracle.row_rel_err(g, r)
        k = int(np.argmax(rows))
        assert rows[k] <= 2e-2, f"{name}: row {k} off by {rows[k]:.3e}"
    assert oracle.rel_l2(y.cpu().numpy(), y_ref) <= 2e-3
    # (2) layer by layer on the ORACLE's activations: each GPU layer gets the oracle's input (and residual)
    # tensor, so its output is held to the single-layer bounds, row by row and element by element (plus one
    # ulp of the layer's sum, which both sides round to fp16 before bias / residual / ReLU).
    dev = {"input": to_dev(x)}
    def on_dev(name):
        if name not in dev:
            dev[name] = to_dev(ref[name])
        return dev[name]
    cat_parts = {}
    for kind, op in ops:
        if kind == "concat":
            g = ts.ts_concat_cols(on_dev(op["a"]), on_dev(op["b"]))
            assert np.array_equal(g.cpu().numpy(), ref[op["dst"]]), op["dst"]
            cat_parts[op["dst"]] = (op["a"], op["b"])
            continue
        _, b = net.params[op["name"]]
        res = on_dev(op["residual"]) if op["residual"] else None
        if op["src"] in cat_parts:      # as the network driver runs it: the two parts read in place
            pa, pb = cat_parts[op["src"]]
            g = ts.ts_sparse_conv_prepared2(on_dev(pa), on_dev(pb), net.prepared[op["name"]], maps[op["map"]], b, res, op["relu"])
            g1 = ts.ts_sparse_conv_prepared(on_dev(op["src"]), net.prepared[op["name"]], maps[op["map"]], b, res, op["relu"])
            assert torch.equal(g, g1), f"{op['name']}: two-part input differs from the concatenated one"
        else:
            g = ts.ts_sparse_conv_prepared(on_dev(op["src"]), net.prepared[op["name"]], maps[op["map"]], b, res, op["relu"])
        r = ref[op["dst"]].astype(np.float64)
        mag = np.abs(r) + np.abs(params[op["name"]][1].astype(np.float64))[None, :]
        if op["residual"]:
            mag = mag + np.abs(ref[op["residual"]].astype(np.float64))
        check_features(g, r, torch.float16, f"{op['name']} on the oracle's input", pre_mag=mag)
    torch.cuda.synchronize()
    SparseNet.free_maps(maps)
    return worst, len(ref)


def test_network_small_scene():
    """One sweep (~58k voxels): all 45 convs, 4 concats, every intermediate tensor checked."""
    coords = lidar_scan_coords(4, n_sweeps=1)
    worst, n = _run_both(coords, seed=40)
    print(f"config 5 (1 sweep): {n} tensors, worst rel L2 {worst:.2e}")


def test_network_maps_through_the_coordinate_grid():
    """The same pass with every map built through the grid over the recipe's voxel grid (2048 x 2048 x 80 cells)."""
    coords = lidar_scan_coords(4, n_sweeps=1)
    worst, n = _run_both(coords, seed=41, box=((0, 0, 0), (2047, 2047, 79), 1))
    print(f"config 5 (1 sweep, grid search): {n} tensors, worst rel L2 {worst:.2e}")


@pytest.mark.timeout(600)
def test_config5_full_scene():
    """Config 3's input (5 sweeps, ~150k voxels), 4 input channels."""
    coords = lidar_scan_coords(2, n_sweeps=5)
    worst, n = _run_both(coords, seed=50)
    print(f"config 5 (full): {n} tensors, worst rel L2 {worst:.2e}")


def test_graph_replay_equals_eager():
    """The forward pass captured in a HIP graph gives the eager result on every replay, with other
    work of the library (a map build, a layer) and synchronisations between the replays."""
    coords = lidar_scan_coords(4, n_sweeps=1)
    ops, output = build_plan(4)
    params = make_params(60, ops)
    net = SparseNet(ops, output, {k: (to_dev(w), to_dev(b)) for k, (w, b) in params.items()})
    maps, _ = net.build_maps(to_dev(coords))
    xs = [to_dev(features(61 + i, coords.shape[0], 4, np.float16)) for i in range(3)]
    eager = [net.forward(maps, x).clone() for x in xs]
    torch.cuda.synchronize()
    graph, static_in, static_out = net.capture(maps, xs[0])
    for rep in range(2):
        for x, want in zip(xs, eager):
            static_in.copy_(x)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(static_out, want)
            other = ts.ts_build_kmap(to_dev(coords[:5000]), 3, 1)      # eager library work in between
            ts.ts_sparse_conv(to_dev(features(70, 5000, 32, np.float16)), to_dev(np.zeros((27, 32, 32), np.float16)), other)
            torch.cuda.synchronize()
            other.free()
        if rep == 0:
            # An eager layer that outgrows every scratch area the graph recorded (buffers F and G of the explicit
            # dataflow at 256 channels on the whole scene, its repacked weights): the areas the graph addresses
            # must stay untouched, whatever is built and freed afterwards.
            big = ts.ts_build_kmap(to_dev(coords), 3, 1)
            ts.ts_sparse_conv(to_dev(features(71, coords.shape[0], 256, np.float16)), to_dev(np.ones((27, 256, 256), np.float16)), big,
                              dataflow=ts.TS_DATAFLOW_EXPLICIT)
            torch.cuda.synchronize()
            big.free()
            for i in range(4):
                ts.ts_build_kmap(to_dev(coords[: 20000 * (i + 1)]), 3, 1).free()
    del graph
    SparseNet.free_maps(maps)


def test_scratch_cannot_grow_under_capture_and_says_so():
    """A layer whose scratch areas have no room yet fails cleanly while its stream is being captured (nothing
    may allocate there); after one eager call the same capture works and replays the eager result."""
    coords = lidar_scan_coords(4, n_sweeps=1)[:20000]
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    x = to_dev(features(80, 20000, 64, np.float16))
    w = to_dev(features(81, 27 * 64, 64, np.float16).reshape(27, 64, 64) * np.float16(0.05))
    out = torch.zeros((20000, 64), dtype=torch.float16, device="cuda")
    torch.cuda.synchronize()
    ts.ts_release_cache()                       # the areas are gone: the next layer call must allocate
    side = torch.cuda.Stream()
    err = None
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        try:
            ts.ts_sparse_conv(x, w, kmap, out)  # the plain call repacks its weights into library scratch
        except ts.TsError as e:
            err = e
    assert err is not None and err.code == ts.TS_ERR_UNSUPPORTED and "captured" in str(err)
    del graph
    with torch.cuda.stream(side):
        want = ts.ts_sparse_conv(x, w, kmap).clone()   # sizes the area
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ts.ts_sparse_conv(x, w, kmap, out)
    out.zero_()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    del graph
    kmap.free()
