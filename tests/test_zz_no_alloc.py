"""ts_sparse_conv_static - the layer for callers that cannot allocate - against ts_sparse_conv, through the C ABI.

Both run the same kernels, so the results must be equal bit for bit (and both are held to the oracle's
bounds).  Two calls in a row share the library's fixed staging array, the second with a smaller input:
nothing of the first may leak into it.  Device memory in use must not change across a call.
"""
import numpy as np
import pytest
import torch

from paper_2204_10319_amd import binding as ts
from workloads import features, conv_weights
from _util import np_dtype, to_dev, oracle_conv, check_features

pytestmark = pytest.mark.gpu


def _coords(seed, n, side, batches=1):
    rng = np.random.Generator(np.random.PCG64(seed))
    flat = rng.choice(batches * side ** 3, size=n, replace=False)
    b, x, y, z = np.unravel_index(flat, (batches, side, side, side))
    return np.stack([b, x - side // 2, y - side // 2, z - side // 2], axis=1).astype(np.int32)


def _case(coords, c_in, c_out, K, s, transposed, dtype, seed):
    nd = np_dtype(dtype)
    kmap = ts.ts_build_kmap(to_dev(coords), K, s, transposed)
    x_h, w_h = features(seed, kmap.num_in, c_in, nd), conv_weights(seed + 1, K ** 3, c_in, c_out, nd)
    x, w = to_dev(x_h), to_dev(w_h)
    want = ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_FUSED)
    out = torch.full((kmap.num_out, c_out), float("nan"), dtype=dtype, device="cuda")
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    print(f"ts_sparse_conv_static N={coords.shape[0]} C {c_in}->{c_out} K{K} s{s} t{int(transposed)} {dtype}", flush=True)
    ts.ts_sparse_conv_static(x, w, kmap, out)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory in use changed across the call"
    assert torch.equal(out, want)
    check_features(out, oracle_conv(coords, x_h, w_h, K, s, transposed), dtype, "static entry point")
    kmap.free()


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
def test_two_calls_in_a_row_the_second_smaller(dtype):
    """A layer with large weights on several tiles, then a narrower layer on fewer points: the second call's
    packed weights cover only the start of what the first left in the array."""
    _case(_coords(1, 5000, 24, batches=2), 64, 96, 3, 1, False, dtype, seed=10)
    _case(_coords(2, 700, 12), 32, 32, 3, 1, False, dtype, seed=20)
    _case(_coords(3, 37, 6), 32, 64, 2, 2, True, dtype, seed=30)


def test_other_map_kinds_and_the_resident_weight_kernel():
    _case(_coords(4, 3000, 20), 32, 32, 3, 1, False, torch.float16, seed=40)     # weights resident in LDS
    _case(_coords(5, 3000, 20), 128, 64, 2, 2, False, torch.float16, seed=50)
    _case(_coords(6, 2000, 16), 256, 256, 1, 1, False, torch.float16, seed=60)
    _case(_coords(7, 1, 4), 32, 32, 3, 1, False, torch.float16, seed=70)


def test_limits_are_reported_not_exceeded():
    coords = _coords(8, 500, 10)
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    def call(c_in, c_out, dtype):
        x = torch.zeros((500, c_in), dtype=dtype, device="cuda")
        w = torch.zeros((27, c_in, c_out), dtype=dtype, device="cuda")
        out = torch.zeros((500, c_out), dtype=dtype, device="cuda")
        return ts.ts_sparse_conv_static(x, w, kmap, out)
    call(256, 256, torch.float16)                       # 27 * 256 * 256 * 2 = 3.375 MiB: fits
    for c_in, c_out, dtype in [(288, 288, torch.float16), (256, 256, torch.float32), (16, 32, torch.float16),
                               (4, 32, torch.float32)]:
        with pytest.raises(ts.TsError) as e:
            call(c_in, c_out, dtype)
        assert e.value.code == ts.TS_ERR_UNSUPPORTED, (c_in, c_out, dtype)
    empty = ts.ts_build_kmap(torch.zeros((0, 4), dtype=torch.int32, device="cuda"), 3, 1)
    out = torch.zeros((0, 32), dtype=torch.float16, device="cuda")
    ts.ts_sparse_conv_static(torch.zeros((0, 32), dtype=torch.float16, device="cuda"),
                             torch.zeros((27, 32, 32), dtype=torch.float16, device="cuda"), empty, out)


def test_under_graph_capture():
    """What the entry point is for: recorded into a HIP graph (nothing may allocate there) and replayed, with new
    features copied in between the replays and other library work in between; every replay equals the eager result."""
    coords = _coords(9, 4000, 22, batches=2)
    kmap = ts.ts_build_kmap(to_dev(coords), 3, 1)
    w = to_dev(conv_weights(91, 27, 64, 64, np.float16))
    xs = [to_dev(features(92 + i, 4000, 64, np.float16)) for i in range(3)]
    want = [ts.ts_sparse_conv(x, w, kmap, dataflow=ts.TS_DATAFLOW_FUSED).clone() for x in xs]
    static_in = xs[0].clone()
    static_out = torch.zeros((4000, 64), dtype=torch.float16, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ts.ts_sparse_conv_static(static_in, w, kmap, static_out)     # the first call on the device looks the array's address up
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ts.ts_sparse_conv_static(static_in, w, kmap, static_out)
    for rep in range(2):
        for x, y in zip(xs, want):
            static_in.copy_(x)
            static_out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(static_out, y)
            other = ts.ts_build_kmap(to_dev(coords[:1000]), 3, 1)      # eager library work between the replays
            ts.ts_sparse_conv_static(to_dev(features(99, 1000, 32, np.float16)), to_dev(conv_weights(98, 27, 32, 32, np.float16)), other,
                                     torch.zeros((1000, 32), dtype=torch.float16, device="cuda"))
            torch.cuda.synchronize()
            other.free()
            # the eager call above has overwritten the shared array: the graph's own repacking kernel restores it on replay
    del graph
    assert torch.cuda.mem_get_info()[0] >= free_before - (64 << 20)    # nothing of note was allocated by capture or replays
    kmap.free()
