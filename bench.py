#!/usr/bin/env python3
"""Benchmark of the sparse-convolution hot path on one MI355X.

A "step" is one pass of the whole path over the ~150k-voxel LiDAR-like workload
(config 3): the kernel-map build in its non-waiting form (keys packed and inserted into the
hash table, the symmetric map search that fills the out-major neighbour table; the per-offset
counts, rank bitmaps and pair lists are derived only when something asks for them, and the fused
layer does not) followed by the fused output-stationary layer kernel, C_in = C_out = 64,
fp16 in / fp32 accumulate, inputs resident in HBM, no host round trip inside a step.
`ms_per_step_waiting` is the same step with the waiting build (row pass, scan, sizes and error
flags brought to the host) in its place.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--channels C] [--no-cpu-baseline]
    python bench.py --pmc-run      # short run for `rocprofv3 --pmc ...`: a few steps plus three
                                   # 256 MiB plain copies that calibrate the byte counters
    python bench.py --no-sweep     # leaves out the 10x / 100x scenes (batch-tiled config 3)
    python bench.py --no-configs   # leaves out the per-config rows (configs 1, 2, 2b, 4)
    python bench.py --step-only    # the timed steps and nothing else (what the kernel-trace profile runs)
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16 MFMA, vendor figure
F32_PEAK_TFLOPS = 157.3        # fp32 (vector and matrix), vendor figure
COPY_BYTES = 256 << 20


def fused_conv_bytes(n_in, n_out, m, c_in, c_out, k3, b):
    """Algorithmic HBM bytes of one fused layer: X_in read once, X_out written once, the map's
    (in, out) index pairs, the weights."""
    return n_in * c_in * b + n_out * c_out * b + 8 * m + k3 * c_in * c_out * b


def explicit_stage_bytes(n_in, n_out, m, m_moved, c_in, c_out, k3, b):
    """Algorithmic bytes of the three explicit stages (gather / grouped matmul / scatter)."""
    gather = n_in * c_in * b + 4 * m_moved + m_moved * c_in * b
    matmul = m * c_in * b + k3 * c_in * c_out * b + m * c_out * 4
    scatter = m * c_out * 4 + 4 * m + n_out * c_out * b
    return gather, matmul, scatter


def kmap_bytes(n, m, k3, table_slots):
    """Algorithmic bytes of the stride-1 map build that is timed (ts_build_kmap, waiting form): coordinates
    in, table init + fill, one 8-byte probe per (point, half of the offsets), and what it writes: one
    4-byte neighbour entry per pair, a bitmask word per row, and the rank bitmaps (12 bytes per offset and
    64-row block).  The offset-major pair lists are not part of it: they are derived on first use.
    table_slots is counted as the smallest power of two that keeps the table half empty (2 n or more): the
    library allocates twice that because shorter probe chains pay for it, which is its choice, not work the
    method asks for."""
    return 16 * n + 12 * table_slots + 12 * n + (k3 - 1) // 2 * n * 8 + 4 * m + 4 * n + 12 * k3 * ((n + 63) // 64)


def source_tag():
    """First 12 hex digits of the SHA-256 of the layer kernels' source: what a measured traffic figure
    belongs to."""
    import hashlib
    path = os.path.join(ROOT, "paper_2204_10319_amd", "csrc", "ts_conv.hip")
    return hashlib.sha256(open(path, "rb").read()).hexdigest()[:12]


def read_traffic(kernel, workload):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, calibrated); kept in
    profiles/traffic.txt as 'kernel workload fetch_bytes write_bytes source_tag'.  A figure counted on
    another version of the kernel source is not reported: (None, its tag)."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        parts = line.split()
        if len(parts) == 5 and parts[0] == kernel and parts[1] == workload:
            if parts[4] != source_tag():
                return None, parts[4]
            return int(float(parts[2]) + float(parts[3])), parts[4]
    return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--channels", type=int, default=64)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-run", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-configs", action="store_true")
    ap.add_argument("--step-only", action="store_true")
    ap.add_argument("--network-run", action="store_true",
                    help="only 10 passes of the config-5 network (17 map builds + 45 layers each), for profiling")
    ap.add_argument("--build-run", type=int, default=0, metavar="COPIES",
                    help="only 4 waiting 3x3x3 stride-1 map builds of the config-3 scene tiled COPIES times over the batch index, then exit (for counter passes)")
    ap.add_argument("--strided-run", action="store_true",
                    help="20 builds each of the K=2,s=2 and K=3,s=2 (with boundary) maps of config 3, then exit (for the kernel-trace profile)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2204_10319_amd import binding as ts
    from workloads import lidar_scan_coords, tile_batches, features, conv_weights, uniform_grid_coords, box_surface_coords

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    ts.load_library()

    C = args.channels
    K, K3 = 3, 27
    coords_h = lidar_scan_coords(2, n_sweeps=5)
    N = coords_h.shape[0]
    x_h = features(300 + C, N, C, np.float16)
    w_h = conv_weights(301 + C, K3, C, C, np.float16)
    coords = torch.from_numpy(coords_h).cuda()
    x = torch.from_numpy(x_h).cuda()
    w = torch.from_numpy(w_h).cuda()
    out = torch.empty((N, C), dtype=torch.float16, device="cuda")

    pw = ts.ts_weights_prepare(w)   # layer constants: repacked for the kernels once, outside the step

    def step():
        # the build does not wait for its sizes to reach the host (nothing in this step needs them): map
        # build and layer run back to back on the device
        kmap = ts.ts_build_kmap(coords, K, 1, wait=False)
        ts.ts_sparse_conv_prepared(x, pw, kmap, out=out)
        return kmap

    def step_waiting():
        kmap = ts.ts_build_kmap(coords, K, 1)      # waits: row pass, scan, sizes and error flags on the host
        ts.ts_sparse_conv_prepared(x, pw, kmap, out=out)
        return kmap

    if args.pmc_run:
        src = torch.zeros(COPY_BYTES // 4, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            step().free()
        for _ in range(3):
            ts.ts_copy_bytes(dst, src)
        for _ in range(5):
            step().free()
        torch.cuda.synchronize()
        print(json.dumps({"pmc_run": True, "copy_bytes": COPY_BYTES, "N": int(N)}))
        return

    if args.network_run:
        from paper_2204_10319_amd.network import SparseNet
        from workloads.minkunet import build_plan, make_params
        ops, net_out = build_plan(4)
        params = {k: (torch.from_numpy(wt).cuda(), torch.from_numpy(bs).cuda()) for k, (wt, bs) in make_params(50, ops).items()}
        net = SparseNet(ops, net_out, params)
        x4 = torch.from_numpy(features(51, N, 4, np.float16)).cuda()
        for _ in range(10):
            maps, _ = net.build_maps(coords)
            net.forward(maps, x4)
            SparseNet.free_maps(maps)
        torch.cuda.synchronize()
        print(json.dumps({"network_run": True, "N": int(N), "passes": 10}))
        return

    if args.build_run:
        # map builds of the batch-tiled scene (waiting form), for the counter passes of the large build
        big = torch.from_numpy(tile_batches(coords_h, args.build_run)).cuda()
        for _ in range(4):
            ts.ts_build_kmap(big, K, 1).free()
        torch.cuda.synchronize()
        print(json.dumps({"build_run": True, "copies": args.build_run, "N": int(big.shape[0])}))
        return

    if args.strided_run:
        hi = coords_h[:, 1:].max(axis=0)
        bnd = tuple(int(h + 2) // 2 for h in hi)
        for _ in range(20):
            ts.ts_build_kmap(coords, 2, 2).free()
            ts.ts_build_kmap(coords, 3, 2, boundary=bnd).free()
        torch.cuda.synchronize()
        print(json.dumps({"strided_run": True, "N": int(N), "boundary": bnd}))
        return

    # The device's clocks and caches, the library's memory pool and the allocator settle over the first few
    # dozen steps of a process; a fixed number of steps runs before the W warm-up steps the caller asked for,
    # so that a short run (W = 5, K = 20) times the same steady state as a long one.
    PRE_WARM_STEPS = 100
    for _ in range(PRE_WARM_STEPS + args.warmup):
        step().free()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps; the dominant kernel is bracketed by HIP events
    # recorded by the library on its stream
    dominant = "k_conv_"   # k_conv_tile, or k_conv_res for layers of at most 32 channels
    ts.ts_profile_enable(True, dominant)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        kmap = step()
        kmap.free()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = ts.ts_profile_read()
    ts.ts_profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    dom_name = [k for k in prof if k.startswith(dominant)][0]
    launches, total_ms = prof[dom_name]
    dom_us = total_ms * 1e3 / launches

    for _ in range(5):
        step_waiting().free()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_waiting().free()
    torch.cuda.synchronize()
    ms_per_step_waiting = (time.perf_counter() - t0) * 1e3 / args.steps

    kmap = ts.ts_build_kmap(coords, K, 1)
    M = kmap.num_pairs
    sizes = kmap.sizes()
    if args.step_only:
        fb = fused_conv_bytes(N, N, M, C, C, K3, 2)
        print(json.dumps({"step_only": True, "ms_per_step": round(ms_per_step, 4), "kernel": dom_name,
                          "avg_us": round(dom_us, 2), "GBs": round(fb / dom_us * 1e-3, 1), "N": int(N), "M": int(M)}))
        return

    # ---- untimed extras: per-kernel breakdown of a step, copy reference, the layer at several widths
    ts.ts_profile_enable(True)
    for _ in range(20):
        step().free()
    per_kernel = {k: round(v[1] * 1e3 / 20, 2) for k, v in ts.ts_profile_read().items()}   # us per step
    src = torch.zeros(COPY_BYTES // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(13):
        ts.ts_copy_bytes(dst, src)
    cp = ts.ts_profile_read()["k_copy_bytes"]
    copy_gbs = 2 * COPY_BYTES / (cp[1] / cp[0] * 1e-3) * 1e-9
    # achievable MFMA rate: register-only loop of the instruction the layer kernels use
    sink = torch.zeros(1 << 18, dtype=torch.float32, device="cuda")
    for _ in range(6):
        mfma_flops = ts.ts_mfma_loop(4096, sink)
    ml = ts.ts_profile_read()["k_mfma_loop"]
    mfma_loop_tflops = mfma_flops / (ml[1] / ml[0] * 1e-3) * 1e-12
    ts.ts_profile_enable(False)
    del src, dst, sink

    # spread of single steps: each step bracketed by an event pair of its own
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
    for a_ev, b_ev in evs:
        a_ev.record()
        step().free()
        b_ev.record()
    torch.cuda.synchronize()
    step_us = np.sort(np.array([a_ev.elapsed_time(b_ev) * 1e3 for a_ev, b_ev in evs]))
    step_spread = {"p10_us": round(float(step_us[20]), 1), "p50_us": round(float(step_us[100]), 1),
                   "p90_us": round(float(step_us[180]), 1), "n": 200}

    # the same step with the map searched through the coordinate grid over the recipe's voxel grid (Sec. 4.4:
    # the choice the paper makes per layer); not the headline, which stays on the hash table
    vgrid = ((0, 0, 0), (2047, 2047, 79), 1)

    def step_grid():
        km = ts.ts_build_kmap(coords, K, 1, wait=False, grid=vgrid)
        ts.ts_sparse_conv_prepared(x, pw, km, out=out)
        return km

    for _ in range(10):
        step_grid().free()
    torch.cuda.synchronize()
    g0 = time.perf_counter()
    for _ in range(200):
        step_grid().free()
    torch.cuda.synchronize()
    step_grid_ms = (time.perf_counter() - g0) * 1e3 / 200

    def time_calls(fn, iters=50):
        for _ in range(5):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / iters   # us

    def layer_report(km, n, m, c, device_features=False):
        if device_features:   # timing only, at sizes where drawing the features on the host would take longer than the run
            gen = torch.Generator(device="cuda")
            gen.manual_seed(300 + c)
            xc = torch.randn((n, c), generator=gen, device="cuda", dtype=torch.float32).to(torch.float16)
        else:
            xc = torch.from_numpy(features(300 + c, n, c, np.float16)).cuda()
        wc = torch.from_numpy(conv_weights(301 + c, K3, c, c, np.float16)).cuda()
        oc = torch.empty((n, c), dtype=torch.float16, device="cuda")
        fused_us = time_calls(lambda: ts.ts_sparse_conv(xc, wc, km, oc, ts.TS_DATAFLOW_FUSED), 30)
        expl_us = time_calls(lambda: ts.ts_sparse_conv(xc, wc, km, oc, ts.TS_DATAFLOW_EXPLICIT), 30)
        fetch_us = time_calls(lambda: ts.ts_sparse_conv(xc, wc, km, oc, ts.TS_DATAFLOW_FETCH), 30)
        ts.ts_profile_enable(True)
        for _ in range(20):
            ts.ts_sparse_conv(xc, wc, km, oc, ts.TS_DATAFLOW_EXPLICIT)
            ts.ts_sparse_conv(xc, wc, km, oc, ts.TS_DATAFLOW_FUSED)
        pk = {k: v[1] * 1e3 / v[0] for k, v in ts.ts_profile_read().items()}
        ts.ts_profile_enable(False)
        fused_name = [k for k in pk if k.startswith("k_conv_") or k.startswith("k_fused")][0]
        gname = [k for k in pk if k.startswith("k_gather")][0]     # k_gather (output order) or k_gather_in (input-stationary)
        # the gather stage in both orders (Sec. 4.3.2), on its own
        Fb = torch.empty((m, c), dtype=torch.float16, device="cuda")
        g_out = time_calls(lambda: ts.ts_gather(xc, km, Fb, order=ts.TS_GATHER_OUTPUT_ORDER), 20)
        g_in = time_calls(lambda: ts.ts_gather(xc, km, Fb, order=ts.TS_GATHER_INPUT_STATIONARY), 20)
        del Fb
        fu = pk[fused_name]
        gb, mb, sb = explicit_stage_bytes(n, n, m, m - n, c, c, K3, 2)   # the centre offset is not gathered
        fb = fused_conv_bytes(n, n, m, c, c, K3, 2)
        flops = 2.0 * m * c * c
        return {
            "fused_layer_us": round(fused_us, 2), "explicit_layer_us": round(expl_us, 2), "fetch_layer_us": round(fetch_us, 2),
            "fused_kernel": fused_name, "k_fused_us": round(fu, 2),
            "k_fused_GBs": round(fb / fu * 1e-3, 1), "k_fused_frac_hbm": round(fb / fu * 1e-3 / HBM_PEAK_GBS, 4),
            "k_fused_TFLOPs": round(flops / fu * 1e-6, 1),
            "k_fused_frac_mfma": round(flops / fu * 1e-6 / MFMA_F16_PEAK_TFLOPS, 4),
            "gather_kernel": gname, "k_gather_us": round(pk[gname], 2), "k_gather_GBs": round(gb / pk[gname] * 1e-3, 1),
            "k_gather_frac_hbm": round(gb / pk[gname] * 1e-3 / HBM_PEAK_GBS, 4),
            "gather_output_order_us": round(g_out, 2), "gather_input_stationary_us": round(g_in, 2),
            "k_grouped_mm_us": round(pk["k_grouped_mm"], 2),
            "k_grouped_mm_GBs": round(mb / pk["k_grouped_mm"] * 1e-3, 1),
            "k_grouped_mm_TFLOPs": round(flops / pk["k_grouped_mm"] * 1e-6, 1),
            "k_grouped_mm_frac_mfma": round(flops / pk["k_grouped_mm"] * 1e-6 / MFMA_F16_PEAK_TFLOPS, 4),
            "k_scatter_reduce_us": round(pk["k_scatter_reduce"], 2),
            "k_scatter_reduce_GBs": round(sb / pk["k_scatter_reduce"] * 1e-3, 1),
            "k_scatter_reduce_frac_hbm": round(sb / pk["k_scatter_reduce"] * 1e-3 / HBM_PEAK_GBS, 4),
            "k_grouped_mm_frac_hbm": round(mb / pk["k_grouped_mm"] * 1e-3 / HBM_PEAK_GBS, 4),
        }

    kmap_us = time_calls(lambda: ts.ts_build_kmap(coords, K, 1).free(), 30)
    layers = {f"C{c}": layer_report(kmap, N, M, c) for c in (32, 64, 128)}
    # ---- grouping ablation (Sec. 4.2.3; Appendix B, Alg. 4): the matmul stage of the explicit dataflow in the
    # launches adaptive grouping prescribes, next to the single tile-scheduled launch the library uses
    def grouping_report(km, n_in, c):
        xc = torch.from_numpy(features(300 + c, n_in, c, np.float16)).cuda()
        wc = torch.from_numpy(conv_weights(301 + c, km.kernel_volume, c, c, np.float16)).cuda()
        has_centre = km.kernel_volume == 27 and km.num_in == km.num_out
        fc = ts.ts_gather(xc, km)
        gc = torch.empty((km.num_pairs, c), dtype=torch.float32, device="cuda")
        xarg = xc if has_centre else None
        rows = {"single_launch": {"us": round(time_calls(lambda: ts.ts_grouped_matmul(fc, xarg, wc, km, gc), 30), 2),
                                  "launches": 1, "padded_over_needed": 1.0}}
        huge = 1 << 40
        for tag, eps, thr in (("separate", -1.0, 0), ("symmetric_eps0", 0.0, 0), ("adaptive_eps0.1", 0.1, huge),
                              ("adaptive_eps0.3", 0.3, huge), ("adaptive_eps0.5", 0.5, huge),
                              ("adaptive_eps0.5_S30000", 0.5, 30000), ("dense_eps1", 1.0, huge)):
            _, st = ts.ts_grouped_matmul_adaptive(fc, xarg, wc, km, eps, thr, gc)
            us = time_calls(lambda: ts.ts_grouped_matmul_adaptive(fc, xarg, wc, km, eps, thr, gc), 30)
            rows[tag] = {"us": round(us, 2), "launches": int(st["launches"]),
                         "padded_over_needed": round(st["padded_rows"] / max(st["rows"], 1), 3)}
        from paper_2204_10319_amd import tuner
        eps, thr, us, _ = tuner.adaptive_group_search([(fc, xarg, wc, km, gc)])
        rows["tuned_alg5"] = {"us": round(us, 2), "epsilon": eps, "S": int(thr),
                              "search_space": len(tuner.DEFAULT_EPS_SPACE) * len(tuner.DEFAULT_S_SPACE)}
        return rows

    grouping = {"config3_C64_K3s1": grouping_report(kmap, N, 64)}
    kdown = ts.ts_build_kmap(coords, 2, 2)
    grouping["config3_C64_K2s2"] = grouping_report(kdown, N, 64)
    kdown.free()
    # ---- map search ablation (Sec. 4.4): hash table against the coordinate grid, per level of the network's
    # pyramid (coordinates halved level by level), submanifold 3x3x3 and the K=3, s=2 strided map with a boundary
    def grid_box(c_h):
        return (tuple(int(v) for v in c_h[:, 1:].min(axis=0)), tuple(int(v) for v in c_h[:, 1:].max(axis=0)),
                int(c_h[:, 0].max()) + 1)

    search = {}
    level_h = coords_h
    for level in range(5):
        cd = torch.from_numpy(np.ascontiguousarray(level_h)).cuda()
        box = grid_box(level_h)
        cells = box[2] * int(np.prod([h - l + 1 for l, h in zip(box[0], box[1])]))
        bnd = tuple((h + 2) // 2 for h in box[1])
        ts.ts_build_kmap(cd, 3, 1, grid=box).free()          # grows the grid's buffer outside the timing
        row = {"N": int(level_h.shape[0]), "grid_cells": cells,
               "K3s1_hash_us": round(time_calls(lambda: ts.ts_build_kmap(cd, 3, 1).free(), 20), 1),
               "K3s1_grid_us": round(time_calls(lambda: ts.ts_build_kmap(cd, 3, 1, grid=box).free(), 20), 1),
               "K3s2_boundary_hash_us": round(time_calls(lambda: ts.ts_build_kmap(cd, 3, 2, boundary=bnd, search=ts.TS_SEARCH_HASH).free(), 20), 1),
               "K3s2_boundary_grid_us": round(time_calls(lambda: ts.ts_build_kmap(cd, 3, 2, grid=box, boundary=bnd).free(), 20), 1),
               "K3s2_boundary_auto_us": round(time_calls(lambda: ts.ts_build_kmap(cd, 3, 2, boundary=bnd).free(), 20), 1),
               "K2s2_hash_us": round(time_calls(lambda: ts.ts_build_kmap(cd, 2, 2, search=ts.TS_SEARCH_HASH).free(), 20), 1),
               "K2s2_auto_us": round(time_calls(lambda: ts.ts_build_kmap(cd, 2, 2).free(), 20), 1)}
        search[f"level{level}_stride{2 ** level}"] = row
        nxt = np.unique(np.concatenate([level_h[:, :1], level_h[:, 1:] // 2], axis=1), axis=0).astype(np.int32)
        level_h = nxt
    # optional ordering of the output rows by offset bitmask (for maps that serve several layers)
    sort_us = time_calls(lambda: ts.ts_build_kmap(coords, K, 1).sort_rows().free(), 20) - kmap_us
    ksorted = ts.ts_build_kmap(coords, K, 1).sort_rows()
    sorted_rows = {"sort_rows_us": round(sort_us, 1)}
    for c in (32, 64, 128):
        xc = torch.from_numpy(features(300 + c, N, c, np.float16)).cuda()
        wc = torch.from_numpy(conv_weights(301 + c, K3, c, c, np.float16)).cuda()
        oc = torch.empty((N, c), dtype=torch.float16, device="cuda")
        sorted_rows[f"C{c}_fused_layer_us"] = round(time_calls(lambda: ts.ts_sparse_conv(xc, wc, ksorted, oc), 30), 2)
    ksorted.free()
    table_slots = 1 << int(np.ceil(np.log2(2 * N)))
    kb = kmap_bytes(N, M, K3, table_slots)
    breakdown = {"kmap_build_us": round(kmap_us, 1), "kmap_algorithmic_bytes": int(kb),
                 "kmap_GBs": round(kb / kmap_us * 1e-3, 1), "copy_kernel_GBs": round(copy_gbs, 1),
                 "mfma_loop_TFLOPs": round(mfma_loop_tflops, 1), "step_spread": step_spread,
                 "step_with_grid_search_ms": round(step_grid_ms, 4),
                 "per_kernel_us_per_step": per_kernel, "layers": layers, "grouping_ablation": grouping,
                 "map_search_ablation": search,
                 "sorted_rows": sorted_rows}

    # ---- config 5: MinkUNet-style forward pass on the same scene (maps built once, then the 45 convs)
    from paper_2204_10319_amd.network import SparseNet
    from workloads.minkunet import build_plan, make_params
    ops, net_out = build_plan(4)
    params = {k: (torch.from_numpy(wt).cuda(), torch.from_numpy(bs).cuda()) for k, (wt, bs) in make_params(50, ops).items()}
    net = SparseNet(ops, net_out, params)
    x4 = torch.from_numpy(features(51, N, 4, np.float16)).cuda()
    net_report = {"convs": sum(1 for k, _ in ops if k == "conv"), "maps": 17}
    for tag, srt in (("", False), ("_sorted_rows", True)):
        maps_us = time_calls(lambda: SparseNet.free_maps(net.build_maps(coords, srt)[0]), 5)
        maps, _ = net.build_maps(coords, srt)
        fwd_us = time_calls(lambda: net.forward(maps, x4), 10)
        graph, _, _ = net.capture(maps, x4)
        graph_us = time_calls(graph.replay, 20)
        del graph
        if not srt:
            # where a pass spends its time: launches and microseconds per kernel (HIP events around every launch)
            ts.ts_profile_enable(True)
            for _ in range(3):
                net.forward(maps, x4)
            net_report["forward_kernels"] = {k: {"launches": v[0] // 3, "us": round(v[1] * 1e3 / 3, 1)}
                                             for k, v in ts.ts_profile_read().items()}
            ts.ts_profile_enable(False)
        SparseNet.free_maps(maps)
        net_report["maps_build_ms" + tag] = round(maps_us * 1e-3, 3)
        if not srt:
            # the same maps through the coordinate grid over the voxel grid of the recipe (2048 x 2048 x 80 cells)
            vbox = ((0, 0, 0), (2047, 2047, 79), 1)
            SparseNet.free_maps(net.build_maps(coords, False, vbox)[0])
            net_report["maps_build_ms_grid"] = round(time_calls(lambda: SparseNet.free_maps(net.build_maps(coords, False, vbox)[0]), 5) * 1e-3, 3)
        net_report["forward_ms" + tag] = round(fwd_us * 1e-3, 3)
        net_report["forward_graph_ms" + tag] = round(graph_us * 1e-3, 3)
    breakdown["config5_network"] = net_report

    if not args.no_sweep:
        big_h = tile_batches(coords_h, 10)
        big = torch.from_numpy(big_h).cuda()
        kbig = ts.ts_build_kmap(big, K, 1)
        breakdown["sweep_10x"] = {"N": int(big_h.shape[0]), "M": int(kbig.num_pairs),
                                  "kmap_build_us": round(time_calls(lambda: ts.ts_build_kmap(big, K, 1).free(), 10), 1),
                                  "C64": layer_report(kbig, big_h.shape[0], kbig.num_pairs, 64, True)}
        sl = 1 << int(np.ceil(np.log2(2 * big_h.shape[0])))
        kb10 = kmap_bytes(big_h.shape[0], breakdown["sweep_10x"]["M"], K3, sl)
        breakdown["sweep_10x"]["kmap_frac_hbm"] = round(kb10 / breakdown["sweep_10x"]["kmap_build_us"] * 1e-3 / HBM_PEAK_GBS, 4)
        kbig.free()
        del big
        huge_h = tile_batches(coords_h, 100)
        huge = torch.from_numpy(huge_h).cuda()
        khuge = ts.ts_build_kmap(huge, K, 1)
        breakdown["sweep_100x"] = {"N": int(huge_h.shape[0]), "M": int(khuge.num_pairs),
                                   "kmap_build_us": round(time_calls(lambda: ts.ts_build_kmap(huge, K, 1).free(), 5), 1),
                                   "C64": layer_report(khuge, huge_h.shape[0], khuge.num_pairs, 64, True)}
        sl = 1 << int(np.ceil(np.log2(2 * huge_h.shape[0])))
        kb100 = kmap_bytes(huge_h.shape[0], breakdown["sweep_100x"]["M"], K3, sl)
        breakdown["sweep_100x"]["kmap_frac_hbm"] = round(kb100 / breakdown["sweep_100x"]["kmap_build_us"] * 1e-3 / HBM_PEAK_GBS, 4)
        khuge.free()
        del huge

    # ---- one row per benchmark configuration other than the headline: sizes, map build, layer, fractions of the
    # rooflines, and the oracle on the host beside them
    def config_row(coords_c, K_, s_, transposed, c_in, c_out, np_dt, seed, gain=1.0):
        import oracle
        f16 = np_dt == np.float16
        cd = torch.from_numpy(np.ascontiguousarray(coords_c)).cuda()
        build_us = time_calls(lambda: ts.ts_build_kmap(cd, K_, s_, transposed).free(), 20)
        km = ts.ts_build_kmap(cd, K_, s_, transposed)
        n_in, n_out, m = km.num_in, km.num_out, km.num_pairs
        xh = features(seed, n_in, c_in, np_dt)
        wh = conv_weights(seed + 1, K_ ** 3, c_in, c_out, np_dt, gain=gain)
        xc, wc = torch.from_numpy(xh).cuda(), torch.from_numpy(wh).cuda()
        oc = torch.empty((n_out, c_out), dtype=xc.dtype, device="cuda")
        layer_us = time_calls(lambda: ts.ts_sparse_conv(xc, wc, km, oc), 30)
        ts.ts_profile_enable(True)
        for _ in range(20):
            ts.ts_sparse_conv(xc, wc, km, oc)
        pk = {k: round(v[1] * 1e3 / v[0], 2) for k, v in ts.ts_profile_read().items()}
        ts.ts_profile_enable(False)
        main_k = max((k for k in pk if not k.startswith("k_pack") and not k.startswith("k_pad")), key=lambda k: pk[k])
        b = 2 if f16 else 4
        fb = fused_conv_bytes(n_in, n_out, m, c_in, c_out, K_ ** 3, b)
        flops = 2.0 * m * c_in * c_out
        peak_tf = MFMA_F16_PEAK_TFLOPS if f16 else F32_PEAK_TFLOPS
        row = {"N_in": int(n_in), "N_out": int(n_out), "M": int(m), "C_in": c_in, "C_out": c_out, "K": K_, "stride": s_,
               "transposed": bool(transposed), "dtype": "f16" if f16 else "f32",
               "kmap_build_us": round(build_us, 1), "layer_us": round(layer_us, 2), "kernels_us": pk,
               "layer_kernel": main_k, "algorithmic_bytes": int(fb),
               "layer_kernel_GBs": round(fb / pk[main_k] * 1e-3, 1),
               "layer_kernel_frac_hbm": round(fb / pk[main_k] * 1e-3 / HBM_PEAK_GBS, 4),
               "layer_kernel_TFLOPs": round(flops / pk[main_k] * 1e-6, 2),
               "layer_kernel_frac_matrix_peak": round(flops / pk[main_k] * 1e-6 / peak_tf, 5),
               "matrix_peak_TFLOPs": peak_tf}
        if s_ == 1:
            slots = 1 << int(np.ceil(np.log2(max(2 * n_in, 1024))))
            row["kmap_frac_hbm"] = round(kmap_bytes(n_in, m, K_ ** 3, slots) / build_us * 1e-3 / HBM_PEAK_GBS, 4)
        km.free()
        if not args.no_cpu_baseline:
            th = oracle.default_threads()
            c0 = time.perf_counter()
            q = oracle.out_coords(coords_c, K_, s_)
            oracle.kmap(coords_c, q, K_, s_)
            c1 = time.perf_counter()
            if transposed:
                oracle.conv_transposed(coords_c, xh, wh, K_, s_, coarse_coords=q, threads=th)
            else:
                oracle.conv(coords_c, xh, wh, K_, s_, out_coords_=q, threads=th)
            c2 = time.perf_counter()
            row["oracle_map_ms_1_thread"] = round((c1 - c0) * 1e3, 1)
            row["oracle_layer_ms"] = round((c2 - c1) * 1e3, 1)
            row["oracle_threads"] = th
        return row

    if not args.no_configs:
        cfg = {}
        cfg["config1_uniform_grid_fp32_C32"] = config_row(uniform_grid_coords(0), 3, 1, False, 32, 32, np.float32, 100)
        cfg["config2_box_surfaces_9_boxes_C64"] = config_row(box_surface_coords(1, n_boxes=9), 3, 1, False, 64, 64, np.float16, 200)
        cfg["config2b_box_surfaces_40_boxes_C64"] = config_row(box_surface_coords(1, n_boxes=40), 3, 1, False, 64, 64, np.float16, 200)
        cfg["config4_down_K2s2_64to128"] = config_row(coords_h, 2, 2, False, 64, 128, np.float16, 400, gain=8.0)
        cfg["config4_up_K2s2_transposed_128to64"] = config_row(coords_h, 2, 2, True, 128, 64, np.float16, 402, gain=8.0)
        breakdown["configs"] = cfg

    # ---- CPU baseline: the oracle as it stands, on this machine's host cores (whole config-3 layer)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.default_threads()
        best = float("inf")
        for _ in range(3):
            c0 = time.perf_counter()
            oracle.kmap(coords_h, coords_h, K, 1)
            oracle.conv(coords_h, x_h, w_h, K, 1, threads=threads)
            best = min(best, time.perf_counter() - c0)
        c0 = time.perf_counter()
        oracle.kmap(coords_h, coords_h, K, 1)
        oracle.conv(coords_h, x_h, w_h, K, 1, threads=1)
        one_thread_ms = (time.perf_counter() - c0) * 1e3
        cpu = {"value": round(best * 1e3, 1), "unit": "ms", "cores": threads, "kind": "oracle",
               "value_1_thread": round(one_thread_ms, 1),
               "sample": f"whole config-3 layer (N={N}, C={C}): oracle map search on 1 thread + Eq.1 sum on "
                         f"{threads} threads, best of 3"}

    fb = fused_conv_bytes(N, N, M, C, C, K3, 2)
    achieved = fb / dom_us * 1e-3   # GB/s
    workload = f"config3_C{C}"
    traffic, traffic_tag = read_traffic(dom_name, workload)
    result = {
        "metric": "sparse_conv_layer_latency_ms (kernel-map build + one 3x3x3 submanifold layer, ~150k voxels)",
        "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_waiting": round(ms_per_step_waiting, 4),
        "pre_warm_steps": PRE_WARM_STEPS,
        "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "config 3: simulated 64-beam LiDAR, 5 sweeps, 0.05 m voxels", "N": int(N),
                   "M": int(M), "C_in": C, "C_out": C, "kernel": 3, "stride": 1,
                   "map_sizes": [int(s) for s in sizes]},
        "roofline": {"kernel": dom_name, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source_tag": traffic_tag, "source_tag": source_tag(),
                     "avg_us": round(dom_us, 2), "algorithmic_bytes": int(fb),
                     "mfma_tflops": round(2.0 * M * C * C / dom_us * 1e-6, 1),
                     "mfma_frac": round(2.0 * M * C * C / dom_us * 1e-6 / MFMA_F16_PEAK_TFLOPS, 4)},
        "cpu_baseline": cpu,
        "breakdown": breakdown,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
