"""Pins for the CPU oracle: it is checked against things other than itself.

Each test names what fixes the expected value: a value the paper prints, a
closed form, a brute-force enumeration written here in plain Python, or a
library routine (dense 3-D convolution, matmul) that the sparse convolution
must reduce to on special inputs.
"""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from workloads import uniform_grid_coords, features, conv_weights, shuffle_rows

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _random_coords(seed, n, lo, hi, batches=1):
    """n distinct (b,x,y,z) rows with x,y,z in [lo,hi) and b in [0,batches)."""
    rng = _rng(seed)
    side = hi - lo
    flat = rng.choice(batches * side ** 3, size=n, replace=False)
    b, x, y, z = np.unravel_index(flat, (batches, side, side, side))
    return np.stack([b, x + lo, y + lo, z + lo], axis=1).astype(np.int32)


# ---------------------------------------------------------------- offsets (Sec. 2)

def _read_offset_sets():
    sets = []
    with open(os.path.join(GOLDEN, "offset_sets.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, vals = line.split(":")
            d, k = (int(t) for t in head.split())
            sets.append((d, k, [int(t) for t in vals.split()]))
    return sets


def test_offset_sets_match_the_paper():
    """Delta^3(3) = {-1,0,1}^3 and the per-axis range of K=5 is {-2..2} (paper, Sec. 2)."""
    for d, k, axis_vals in _read_offset_sets():
        off = oracle.offsets(k)
        assert off.shape == (k ** 3, 3)
        # per-axis value range is what the paper prints (its K=5 example is 2-D; the per-axis set is the same)
        for a in range(3):
            assert sorted(set(off[:, a].tolist())) == axis_vals
        assert len({tuple(r) for r in off.tolist()}) == k ** 3
        if d == 3:
            assert {tuple(r) for r in off.tolist()} == set(itertools.product(axis_vals, repeat=3))


@pytest.mark.parametrize("K", [1, 3, 5])
def test_offset_index_order_odd(K):
    """x slowest, z fastest; the mirrored offset of index n has index K^3-1-n; the centre is in the middle."""
    off = oracle.offsets(K)
    r = (K - 1) // 2
    expect = np.array(list(itertools.product(range(-r, r + 1), repeat=3)), dtype=np.int32)
    assert np.array_equal(off, expect)
    assert np.array_equal(off[::-1], -off)
    assert tuple(off[(K ** 3 - 1) // 2]) == (0, 0, 0)


def test_offset_set_even_kernel():
    """Even K (reading, the paper gives odd examples only): Delta^3(2) = {0,1}^3."""
    off = oracle.offsets(2)
    assert np.array_equal(off, np.array(list(itertools.product((0, 1), repeat=3)), dtype=np.int32))


# ---------------------------------------------------------------- output coordinates (Alg. 3)

def _read_example():
    vals = {}
    with open(os.path.join(GOLDEN, "stride2_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=")
            vals[k.strip()] = [int(t) for t in v.split()]
    return vals


def test_paper_worked_example_stride2():
    """Input (3,5), stride 2: offset (1,1) gives output (1,2); offset (0,0) gives none (Sec. 2.1.1)."""
    ex = _read_example()
    s = ex["stride"][0]
    px, py = ex["input"]
    coords = np.array([[0, px, py, 0]], dtype=np.int32)     # embed the 2-D example at z = 0
    out = oracle.out_coords(coords, 3, s)
    got = {tuple(r) for r in out.tolist()}
    ox, oy = ex["output"]
    assert (0, ox, oy, 0) in got
    # 3 and 5 are odd, 0 is even: x,y each admit offsets -1 and +1, z only 0  => exactly four outputs
    assert got == {(0, 1, 2, 0), (0, 1, 3, 0), (0, 2, 2, 0), (0, 2, 3, 0)}
    # the map entry that produces (1,2) carries the offset the paper names, and no entry carries (0,0)
    tri = oracle.kmap(coords, out, 3, s)
    off = oracle.offsets(3)
    k_12 = out.tolist().index([0, ox, oy, 0])
    deltas_12 = [tuple(off[n]) for j, k, n in tri.tolist() if k == k_12]
    dx, dy = ex["offset_with_output"]
    assert deltas_12 == [(dx, dy, 0)]
    zx, zy = ex["offset_without_output"]
    assert all(tuple(off[n][:2]) != (zx, zy) for _, _, n in tri.tolist())


def _brute_out_coords(coords, K, s):
    if s == 1:
        return [tuple(r) for r in coords.tolist()]
    r = (K - 1) // 2
    rng_ = range(-r, K - r)
    out = set()
    for b, x, y, z in coords.tolist():
        for dx in rng_:
            for dy in rng_:
                for dz in rng_:
                    u = (x - dx, y - dy, z - dz)
                    if all(v % s == 0 for v in u):          # Python's % is the mathematical one
                        out.add((b, u[0] // s, u[1] // s, u[2] // s))
    return sorted(out)


@pytest.mark.parametrize("K,s", [(2, 2), (3, 2), (3, 3), (5, 2), (2, 1), (3, 1)])
def test_out_coords_brute_force_with_negative_coords(K, s):
    coords = _random_coords(11 + K * 7 + s, 60, -6, 6, batches=2)
    got = [tuple(r) for r in oracle.out_coords(coords, K, s).tolist()]
    assert got == _brute_out_coords(coords, K, s)


@pytest.mark.parametrize("K,s", [(2, 2), (3, 2), (3, 3), (5, 2)])
def test_out_coords_boundary(K, s):
    """Alg. 3's boundary check, three ways: the unbounded result cut to the grid [0, b) afterwards (u < s*b
    with s | u is q < b), a brute-force enumeration that tests u itself, and a boundary too large to cut."""
    coords = _random_coords(31 + K + s, 80, -4, 9, batches=2)
    b = (3, 4, 2)
    free = oracle.out_coords(coords, K, s)
    got = oracle.out_coords(coords, K, s, boundary=b)
    keep = np.all((free[:, 1:] >= 0) & (free[:, 1:] < np.array(b)), axis=1)
    assert 0 < keep.sum() < free.shape[0]
    assert np.array_equal(got, free[keep])
    r = (K - 1) // 2
    brute = set()
    for bb, x, y, z in coords.tolist():
        for dx in range(-r, K - r):
            for dy in range(-r, K - r):
                for dz in range(-r, K - r):
                    u = (x - dx, y - dy, z - dz)
                    if all(v % s == 0 and 0 <= v < s * lim for v, lim in zip(u, b)):
                        brute.add((bb, u[0] // s, u[1] // s, u[2] // s))
    assert [tuple(row) for row in got.tolist()] == sorted(brute)
    if K <= 3:      # radius 1: from non-negative inputs no candidate below zero passes the modular check
        nonneg = coords[np.all(coords[:, 1:] >= 0, axis=1)]
        assert np.array_equal(oracle.out_coords(nonneg, K, s, boundary=(100, 100, 100)), oracle.out_coords(nonneg, K, s))
    assert np.array_equal(oracle.out_coords(coords, 3, 1, boundary=b), coords)      # stride 1: outputs are the inputs


def test_out_coords_k2s2_closed_form():
    """K=2,s=2: every input has exactly one admissible offset (p mod 2) and its output is floor(p/2)."""
    coords = _random_coords(5, 500, -20, 20, batches=3)
    expect = np.unique(np.concatenate([coords[:, :1], np.floor_divide(coords[:, 1:], 2)], axis=1), axis=0)
    got = oracle.out_coords(coords, 2, 2)
    assert np.array_equal(got, expect)
    tri = oracle.kmap(coords, got, 2, 2)
    assert tri.shape[0] == coords.shape[0]
    assert sorted(tri[:, 0].tolist()) == list(range(coords.shape[0]))
    par = np.mod(coords[:, 1:], 2)
    n_expect = (par[:, 0] * 2 + par[:, 1]) * 2 + par[:, 2]
    assert np.array_equal(n_expect[tri[:, 0]], tri[:, 2])
    assert np.array_equal(got[tri[:, 1], 1:], np.floor_divide(coords[tri[:, 0], 1:], 2))


# ---------------------------------------------------------------- kernel maps (Alg. 1)

def _brute_kmap(in_c, out_c, K, s):
    """All (j,k,n) with p_j == s*q_k + delta_n by plain enumeration: no sorting, no searching."""
    r = (K - 1) // 2
    deltas = list(itertools.product(range(-r, K - r), repeat=3))
    tri = []
    ins, outs = in_c.tolist(), out_c.tolist()
    for k, q in enumerate(outs):
        for j, p in enumerate(ins):
            if p[0] != q[0]:
                continue
            for n, d in enumerate(deltas):
                if all(p[1 + a] == s * q[1 + a] + d[a] for a in range(3)):
                    tri.append((j, k, n))
    return tri


@pytest.mark.parametrize("K,s", [(1, 1), (3, 1), (5, 1), (2, 2), (3, 2), (3, 3)])
def test_kmap_brute_force(K, s):
    coords = _random_coords(100 + 13 * K + s, 90, -4, 4, batches=2)
    out = oracle.out_coords(coords, K, s)
    got = oracle.sort_triples(oracle.kmap(coords, out, K, s))
    expect = oracle.sort_triples(np.array(_brute_kmap(coords, out, K, s), dtype=np.int32).reshape(-1, 3))
    assert np.array_equal(got, expect)
    assert got.shape[0] > 0


@pytest.mark.parametrize("K", [3, 5])
def test_submanifold_symmetry_and_centre(K):
    """Odd K, stride 1 (Sec. 4.2.1): (j,k,n) in M  <=>  (k,j,K^3-1-n) in M; the centre map is the identity."""
    coords = uniform_grid_coords(3, n=3000, grid=24)
    tri = oracle.kmap(coords, coords, K, 1)
    K3 = K ** 3
    fwd = {tuple(t) for t in tri.tolist()}
    assert len(fwd) == tri.shape[0]
    assert {(k, j, K3 - 1 - n) for j, k, n in fwd} == fwd
    centre = tri[tri[:, 2] == (K3 - 1) // 2]
    assert np.array_equal(centre[:, 0], centre[:, 1])
    assert sorted(centre[:, 0].tolist()) == list(range(coords.shape[0]))
    sizes = np.bincount(tri[:, 2], minlength=K3)
    assert np.array_equal(sizes, sizes[::-1])
    # every output appears at most once per offset
    assert len({(k, n) for _, k, n in fwd}) == len(fwd)


def test_kmap_sizes_match_closed_form_on_uniform_grid():
    """20000 of 64^3 cells without replacement: E[M_delta] = N(N-1)/(V-1) * prod_a(1 - |delta_a|/64)."""
    N, G = 20000, 64
    coords = uniform_grid_coords(0, n=N, grid=G)
    tri = oracle.kmap(coords, coords, 3, 1)
    sizes = np.bincount(tri[:, 2], minlength=27)
    off = oracle.offsets(3)
    V = G ** 3
    for n in range(27):
        if n == 13:
            assert sizes[n] == N
            continue
        mean = N * (N - 1) / (V - 1) * np.prod(1 - np.abs(off[n]) / G)
        assert abs(sizes[n] - mean) < 6 * np.sqrt(mean), (n, sizes[n], mean)
    assert abs(int(sizes.sum()) - 58400) < 1500


def test_kmap_rejects_duplicates():
    coords = np.array([[0, 1, 2, 3], [0, 4, 4, 4], [0, 1, 2, 3]], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.kmap(coords, coords, 3, 1)
    with pytest.raises(ValueError):
        oracle.conv(coords, np.ones((3, 2)), np.ones((27, 2, 2)), 3, 1)


def test_batches_do_not_interact():
    a = _random_coords(21, 200, 0, 8)
    b = _random_coords(22, 150, 0, 8)
    b2 = b.copy()
    b2[:, 0] = 1
    both = np.concatenate([a, b2])
    t_both = oracle.kmap(both, both, 3, 1)
    t_a = oracle.kmap(a, a, 3, 1)
    t_b = oracle.kmap(b, b, 3, 1)
    t_b_shift = t_b.copy()
    t_b_shift[:, :2] += a.shape[0]
    expect = oracle.sort_triples(np.concatenate([t_a, t_b_shift]))
    assert np.array_equal(oracle.sort_triples(t_both), expect)


# ---------------------------------------------------------------- features (Eq. 1)

def _densify(coords, x, shape):
    """[1, C, X, Y, Z] float64 tensor holding x at the active sites and zeros elsewhere."""
    C = x.shape[1]
    vol = torch.zeros((1, C) + tuple(shape), dtype=torch.float64)
    c = torch.from_numpy(coords.astype(np.int64))
    vol[0, :, c[:, 1], c[:, 2], c[:, 3]] = torch.from_numpy(np.asarray(x, dtype=np.float64)).T
    return vol


def _dense_weight(w, K):
    """[K^3, Cin, Cout] -> [Cout, Cin, K, K, K] with the offset index unravelled x-slowest."""
    c_in, c_out = w.shape[1], w.shape[2]
    return torch.from_numpy(np.asarray(w, dtype=np.float64)).reshape(K, K, K, c_in, c_out).permute(4, 3, 0, 1, 2).contiguous()


@pytest.mark.parametrize("K", [3, 5])
def test_submanifold_equals_masked_dense_conv(K):
    """Densify, run a dense cross-correlation with zero padding, read it at the active sites."""
    G, c_in, c_out = 10, 5, 7
    coords = uniform_grid_coords(7 + K, n=260, grid=G)
    x = features(1, coords.shape[0], c_in, np.float64)
    w = conv_weights(2, K ** 3, c_in, c_out, np.float64)
    q, y = oracle.conv(coords, x, w, K, 1)
    assert np.array_equal(q, coords)
    dense = F.conv3d(_densify(coords, x, (G, G, G)), _dense_weight(w, K), padding=(K - 1) // 2)
    expect = dense[0][:, coords[:, 1], coords[:, 2], coords[:, 3]].T.numpy()
    assert np.allclose(y, expect, rtol=1e-12, atol=1e-12)
    assert np.abs(expect).max() > 0.1


def test_full_occupancy_equals_dense_conv_everywhere():
    G, c_in, c_out = 6, 4, 3
    grid = np.array(list(itertools.product(range(G), repeat=3)), dtype=np.int32)
    coords = np.concatenate([np.zeros((G ** 3, 1), np.int32), grid], axis=1)
    coords = shuffle_rows(5, coords)
    x = features(3, G ** 3, c_in, np.float64)
    w = conv_weights(4, 27, c_in, c_out, np.float64)
    _, y = oracle.conv(coords, x, w, 3, 1)
    dense = F.conv3d(_densify(coords, x, (G, G, G)), _dense_weight(w, 3), padding=1)
    expect = dense[0][:, coords[:, 1], coords[:, 2], coords[:, 3]].T.numpy()
    assert np.allclose(y, expect, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("K,s,pad", [(2, 2, 0), (3, 2, 1)])
def test_strided_equals_masked_dense_conv(K, s, pad):
    G, c_in, c_out = 12, 4, 6
    coords = uniform_grid_coords(31 + K, n=300, grid=G)
    x = features(5, coords.shape[0], c_in, np.float64)
    w = conv_weights(6, K ** 3, c_in, c_out, np.float64)
    q, y = oracle.conv(coords, x, w, K, s)
    big = G + 4                                              # room so every output index exists in the dense result
    dense = F.conv3d(_densify(coords, x, (big, big, big)), _dense_weight(w, K), stride=s, padding=pad)
    occ = F.conv3d(_densify(coords, np.ones((coords.shape[0], 1)), (big, big, big)),
                   torch.ones((1, 1, K, K, K), dtype=torch.float64), stride=s, padding=pad)
    # the output set is exactly where the receptive field holds at least one input
    sites = torch.nonzero(occ[0, 0] > 0.5).numpy().astype(np.int32)
    assert np.array_equal(q[:, 1:], sites)                   # nonzero() is lexicographic, like the oracle's Unique
    expect = dense[0][:, q[:, 1], q[:, 2], q[:, 3]].T.numpy()
    assert np.allclose(y, expect, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("K,s,pad", [(2, 2, 0), (3, 2, 1)])
def test_transposed_equals_masked_dense_conv_transpose(K, s, pad):
    G, c_in, c_out = 12, 6, 4
    fine = uniform_grid_coords(41 + K, n=300, grid=G)
    coarse = oracle.out_coords(fine, K, s)
    x = features(7, coarse.shape[0], c_in, np.float64)
    w = conv_weights(8, K ** 3, c_in, c_out, np.float64)
    c2, y = oracle.conv_transposed(fine, x, w, K, s)
    assert np.array_equal(c2, coarse)
    big = G // 2 + 3
    vol = _densify(coarse, x, (big, big, big))
    # conv_transpose3d weight layout is [Cin, Cout, K, K, K]; out[s*q + t - pad] += in[q] * w[t]
    wt = torch.from_numpy(w).reshape(K, K, K, c_in, c_out).permute(3, 4, 0, 1, 2).contiguous()
    dense = F.conv_transpose3d(vol, wt, stride=s, padding=pad)
    expect = dense[0][:, fine[:, 1], fine[:, 2], fine[:, 3]].T.numpy()
    assert np.allclose(y, expect, rtol=1e-12, atol=1e-12)
    assert np.abs(expect).max() > 0.1


def test_kernel_size_one_is_a_matmul():
    coords = _random_coords(9, 400, -10, 10, batches=2)
    x = features(9, 400, 12, np.float64)
    w = conv_weights(10, 1, 12, 20, np.float64)
    q, y = oracle.conv(coords, x, w, 1, 1)
    assert np.array_equal(q, coords)
    assert np.allclose(y, x @ w[0], rtol=1e-13, atol=1e-13)


def test_single_pair_picks_the_right_weight_slice():
    """Two points one step apart along +y: output 0 sees input 1 through delta=(0,1,0) only (plus the centre)."""
    coords = np.array([[0, 5, 5, 5], [0, 5, 6, 5]], dtype=np.int32)
    x = np.array([[1.0, 0.0], [0.0, 1.0]])
    w = np.arange(27 * 2 * 3, dtype=np.float64).reshape(27, 2, 3)
    _, y = oracle.conv(coords, x, w, 3, 1)
    n_plus_y = (1 * 3 + 2) * 3 + 1      # delta = (0,+1,0)
    n_minus_y = (1 * 3 + 0) * 3 + 1     # delta = (0,-1,0)
    assert np.array_equal(y[0], x[0] @ w[13] + x[1] @ w[n_plus_y])
    assert np.array_equal(y[1], x[1] @ w[13] + x[0] @ w[n_minus_y])


def test_conv_agrees_with_sum_over_its_own_map():
    """Alg. 2 (gather, matmul, scatter-accumulate over the map) gives the same result as Eq. 1."""
    coords = _random_coords(77, 300, -5, 5, batches=2)
    x = features(11, 300, 6, np.float64)
    for K, s in [(3, 1), (2, 2), (3, 2)]:
        w = conv_weights(12, K ** 3, 6, 5, np.float64)
        q, y = oracle.conv(coords, x, w, K, s)
        tri = oracle.kmap(coords, q, K, s)
        acc = np.zeros_like(y)
        for n in range(K ** 3):
            sel = tri[tri[:, 2] == n]
            np.add.at(acc, sel[:, 1], x[sel[:, 0]] @ w[n])
        assert np.allclose(y, acc, rtol=1e-12, atol=1e-12)
        # transposed: same pairs, roles swapped
        xc = features(13, q.shape[0], 6, np.float64)
        _, yt = oracle.conv_transposed(coords, xc, w, K, s)
        acc_t = np.zeros_like(yt)
        for n in range(K ** 3):
            sel = tri[tri[:, 2] == n]
            np.add.at(acc_t, sel[:, 0], xc[sel[:, 1]] @ w[n])
        assert np.allclose(yt, acc_t, rtol=1e-12, atol=1e-12)


def test_row_order_does_not_matter():
    coords = uniform_grid_coords(15, n=500, grid=12)
    x = features(16, 500, 4, np.float64)
    w = conv_weights(17, 27, 4, 4, np.float64)
    _, y = oracle.conv(coords, x, w, 3, 1)
    perm = _rng(18).permutation(500)
    _, yp = oracle.conv(coords[perm], x[perm], w, 3, 1)
    assert np.allclose(yp, y[perm], rtol=1e-12, atol=1e-13)
    w2 = conv_weights(19, 8, 4, 4, np.float64)
    q, y2 = oracle.conv(coords, x, w2, 2, 2)
    qp, y2p = oracle.conv(coords[perm], x[perm], w2, 2, 2)
    assert np.array_equal(q, qp)
    assert np.allclose(y2, y2p, rtol=1e-12, atol=1e-13)


def test_threads_do_not_change_the_result():
    coords = uniform_grid_coords(20, n=2000, grid=16)
    x = features(21, 2000, 8, np.float64)
    w = conv_weights(22, 27, 8, 8, np.float64)
    _, y1 = oracle.conv(coords, x, w, 3, 1, threads=1)
    _, y4 = oracle.conv(coords, x, w, 3, 1, threads=4)
    assert np.array_equal(y1, y4)


def test_empty_input():
    coords = np.zeros((0, 4), dtype=np.int32)
    assert oracle.out_coords(coords, 2, 2).shape == (0, 4)
    assert oracle.kmap(coords, coords, 3, 1).shape == (0, 3)
    q, y = oracle.conv(coords, np.zeros((0, 4)), np.zeros((27, 4, 3)), 3, 1)
    assert y.shape == (0, 3)


# ---- adaptive grouping (Appendix B, Alg. 4) ------------------------------------------------------------

def _waste(sizes, group):
    hi = max(sizes[i] for i in group)
    return 0.0 if hi == 0 else 1.0 - min(sizes[i] for i in group) / hi


def test_adaptive_groups_special_cases_named_by_the_paper():
    """Sec. 4.2.3: tolerance 1 is dense computation (one group), tolerance 0 groups only equal sizes
    (with mirrored offsets that is symmetric grouping: every index alone with its mirror)."""
    sizes = [8705, 58030, 8790, 26968, 79418, 26855, 8771, 49826, 8594, 30917, 84057, 30973, 49787]
    assert oracle.adaptive_groups(sizes, 1.0) == [list(range(13))]
    assert oracle.adaptive_groups(sizes, 0.0) == [[i] for i in range(13)]
    assert oracle.adaptive_groups([5, 5, 5, 7, 7, 0, 0], 0.0) == [[0, 1, 2], [3, 4], [5, 6]]
    # a downsampling layer: all sizes similar -> one group at a small tolerance
    assert oracle.adaptive_groups([19000, 19100, 18900, 19050, 19120, 18870, 19010, 18990], 0.02) == [list(range(8))]
    # worked by hand: 100,90 (waste 0.1) | 60 would give 0.4 -> new group; 60,55 (0.083) | 10
    assert oracle.adaptive_groups([100, 90, 60, 55, 10], 0.15) == [[0, 1], [2, 3], [4]]


def test_adaptive_groups_invariants():
    rng = np.random.Generator(np.random.PCG64(11))
    for trial in range(300):
        n = int(rng.integers(1, 14))
        sizes = rng.integers(0, 50, size=n).tolist() if trial % 3 else (rng.integers(0, 4, size=n) * 10).tolist()
        eps = float(rng.choice([0.0, 0.1, 0.25, 0.5, 0.9, 1.0]))
        groups = oracle.adaptive_groups(sizes, eps)
        assert [i for g in groups for i in g] == list(range(n))                    # contiguous and covering
        for gi, g in enumerate(groups):
            assert _waste(sizes, g) <= eps + 1e-12                                  # within the tolerance
            if gi + 1 < len(groups):                                                # greedy: could not take the next index
                assert _waste(sizes, g + [groups[gi + 1][0]]) > eps


def test_adaptive_groups_equals_greedy_by_exhaustive_search():
    """Among all contiguous partitions within the tolerance, the greedy one is the one whose groups are,
    from left to right, as long as possible: found here by enumerating every partition of small inputs."""
    from itertools import product
    rng = np.random.Generator(np.random.PCG64(12))
    for _ in range(60):
        n = int(rng.integers(1, 9))
        sizes = rng.integers(1, 30, size=n).tolist()
        eps = float(rng.choice([0.0, 0.2, 0.5, 0.8]))
        best = None
        for cuts in product([0, 1], repeat=n - 1):
            groups, cur = [], [0]
            for i, c in enumerate(cuts, start=1):
                if c:
                    groups.append(cur)
                    cur = []
                cur.append(i)
            groups.append(cur)
            if all(_waste(sizes, g) <= eps + 1e-12 for g in groups):
                key = tuple(len(g) for g in groups)
                if best is None or key > best[0]:
                    best = (key, groups)
        assert oracle.adaptive_groups(sizes, eps) == best[1]


def test_adaptive_group_search_is_the_argmin_of_the_summed_cost():
    """Appendix B, Alg. 5 against numpy's argmin over the table of summed costs (first minimum in search order)."""
    rng = np.random.Generator(np.random.PCG64(13))
    for trial in range(50):
        ne, ns, nd = int(rng.integers(1, 6)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
        costs = rng.integers(1, 6 if trial % 2 else 1000, size=(nd, ne, ns)).astype(float)     # small range: ties
        eps_space, S_space = [0.1 * i for i in range(ne)], [1000 * i for i in range(ns)]
        got = oracle.adaptive_group_search(range(nd), eps_space, S_space,
                                           lambda d, e, S: costs[d, eps_space.index(e), S_space.index(S)])
        total = costs.sum(axis=0)
        ie, js = np.unravel_index(np.argmin(total), total.shape)
        assert got == (eps_space[ie], S_space[js], total[ie, js])


# ---------------------------------------------------------------------------------------------
# The comparison helpers every feature-parity assertion goes through.  Expected values are worked
# out by hand (Pythagorean triples, binary16/binary32 tie points), not recomputed with the formula.
# ---------------------------------------------------------------------------------------------

def test_rel_l2_hand_computed():
    # ||(3,4) - (0,0)|| / ||(0,0)||: nothing to divide by and a non-zero difference
    assert oracle.rel_l2([3.0, 4.0], [0.0, 0.0]) == float("inf")
    assert oracle.rel_l2([0.0, 0.0], [0.0, 0.0]) == 0.0
    assert oracle.rel_l2(np.zeros((0, 8)), np.zeros((0, 8))) == 0.0
    # difference (0,1) has norm 1, reference (1,0) has norm 1
    assert oracle.rel_l2([1.0, 1.0], [1.0, 0.0]) == 1.0
    # the reference is the second argument: difference (0,1), reference (1,1) of norm sqrt 2
    assert oracle.rel_l2([1.0, 0.0], [1.0, 1.0]) == pytest.approx(1.0 / np.sqrt(2.0), rel=1e-15)
    # the norm itself, not its square: difference (3,4) -> 5, reference (6,8) -> 10
    assert oracle.rel_l2([9.0, 12.0], [6.0, 8.0]) == 0.5
    # Frobenius over all entries of a matrix: difference [[3,0],[0,4]] -> 5, reference [[0,5],[12,0]] -> 13
    assert oracle.rel_l2([[3.0, 5.0], [12.0, 4.0]], [[0.0, 5.0], [12.0, 0.0]]) == pytest.approx(5.0 / 13.0, rel=1e-15)
    # no silent broadcasting of a mismatched shape into a small number
    with pytest.raises(ValueError):
        oracle.rel_l2(np.ones((4, 3)), np.ones((4, 2)))
    with pytest.raises(ValueError):
        oracle.rel_l2(np.ones((4, 3)), np.ones((1, 3)))
    # half-precision inputs are widened before the subtraction (65504 - (-65504) overflows fp16)
    a = np.array([65504.0], np.float16)
    assert oracle.rel_l2(a, -a) == 2.0


def test_row_rel_err_hand_computed():
    ref = np.array([[3.0, 4.0], [0.0, 0.0], [6.0, 8.0], [0.0, 5.0]])
    # row norms 5, 0, 10, 5 -> squares 25 + 0 + 100 + 25 = 150, rms row norm sqrt(150 / 4)
    floor = np.sqrt(37.5)
    got = ref.copy()
    got[0] += [0.0, 1.0]        # error 1 on a row of norm 5 (below the floor 6.12)
    got[1] += [0.6, 0.8]        # error 1 on a zero row: divided by the floor
    got[2] += [3.0, 4.0]        # error 5 on a row of norm 10 (above the floor)
    want = np.array([1.0 / floor, 1.0 / floor, 0.5, 0.0])
    assert np.allclose(oracle.row_rel_err(got, ref), want, rtol=1e-15, atol=0)
    # one wrong row among 10 000 is invisible to the whole-tensor norm and plain here
    rng = _rng(5)
    ref = rng.standard_normal((10000, 16))
    got = ref.copy()
    got[1234] = 0.0
    assert oracle.rel_l2(got, ref) < 2e-2
    e = oracle.row_rel_err(got, ref)
    assert int(np.argmax(e)) == 1234 and e[1234] > 0.5 and np.count_nonzero(e) == 1
    assert oracle.row_rel_err(np.zeros((0, 4)), np.zeros((0, 4))).shape == (0,)
    z = oracle.row_rel_err(np.array([[0.0, 0.0], [1.0, 0.0]]), np.zeros((2, 2)))
    assert z[0] == 0.0 and z[1] == np.inf
    with pytest.raises(ValueError):
        oracle.row_rel_err(np.ones((3, 2)), np.ones((3, 1)))


def test_round_to_is_round_to_nearest_even_once():
    # binary16 has 11 significant bits: spacing 2^-10 in [1, 2), 1 in [1024, 2048), 2 in [2048, 4096)
    h = 2.0 ** -11
    cases16 = [
        (1.0 + h, 1.0),                      # tie between 1 and 1 + 2^-10: the even mantissa is 1
        (1.0 + 3 * h, 1.0 + 2.0 ** -9),      # tie between 1 + 2^-10 (odd) and 1 + 2^-9 (even)
        (1.0 + h + 2.0 ** -30, 1.0 + 2.0 ** -10),   # just above the tie: up
        (1.0 + h - 2.0 ** -30, 1.0),                # just below: down
        (2049.0, 2048.0), (2051.0, 2052.0),  # ties at spacing 2
        (-2049.0, -2048.0),
        (65519.0, 65504.0),                  # below the overflow threshold 65520: largest finite value
        (65520.0, np.inf),                   # the tie at the top rounds to infinity
        (2.0 ** -25, 0.0),                   # half the smallest subnormal 2^-24: tie to even = 0
        (3 * 2.0 ** -25, 2.0 ** -23),        # tie between 2^-24 (odd) and 2^-23 (even)
    ]
    for x, want in cases16:
        got = oracle.round_to(np.array([x], np.float64), np.float16)
        assert got.dtype == np.float16
        assert float(got[0]) == want, (x, float(got[0]), want)
    # binary32: 24 significant bits, spacing 2^-23 in [1, 2)
    g = 2.0 ** -24
    for x, want in [(1.0 + g, 1.0), (1.0 + 3 * g, 1.0 + 2.0 ** -22), (1.0 + g + 2.0 ** -50, 1.0 + 2.0 ** -23),
                    (16777217.0, 16777216.0), (16777219.0, 16777220.0)]:
        got = oracle.round_to(np.array([x], np.float64), np.float32)
        assert got.dtype == np.float32 and float(got[0]) == want, (x, float(got[0]), want)
    # one rounding, not two: 1 + 2^-11 + 2^-26 is above the binary16 tie and must go up, while rounding
    # to binary32 first (spacing 2^-23) would land exactly on the tie and then go down to 1
    x = 1.0 + 2.0 ** -11 + 2.0 ** -26
    assert float(oracle.round_to(np.array([x]), np.float16)[0]) == 1.0 + 2.0 ** -10
    assert float(np.array([x]).astype(np.float32).astype(np.float16)[0]) == 1.0
    # shape is kept
    assert oracle.round_to(np.zeros((3, 5)), np.float16).shape == (3, 5)


def test_sort_triples_orders_by_offset_then_output_then_input():
    tri = np.array([[5, 1, 2], [0, 7, 0], [9, 0, 2], [3, 1, 2], [4, 7, 0], [1, 0, 26], [2, 3, 1]], np.int32)
    want = np.array([[0, 7, 0], [4, 7, 0], [2, 3, 1], [9, 0, 2], [3, 1, 2], [5, 1, 2], [1, 0, 26]], np.int32)
    got = oracle.sort_triples(tri)
    assert got.dtype == np.int32 and got.flags["C_CONTIGUOUS"]
    assert np.array_equal(got, want)
    # against Python's sorted on the key (n, k, j), random triples with repeats
    rng = _rng(17)
    tri = rng.integers(0, 6, size=(500, 3)).astype(np.int32)
    want = np.array(sorted(map(tuple, tri.tolist()), key=lambda t: (t[2], t[1], t[0])), np.int32)
    assert np.array_equal(oracle.sort_triples(tri), want)
    assert oracle.sort_triples(np.zeros((0, 3), np.int32)).shape == (0, 3)
    # a flat list of 3k numbers is read as k triples
    assert np.array_equal(oracle.sort_triples(np.array([1, 1, 1, 0, 0, 0])), np.array([[0, 0, 0], [1, 1, 1]], np.int32))
