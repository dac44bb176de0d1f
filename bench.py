#!/usr/bin/env python3
"""Benchmark of the quantized GNN layer path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM: pack the adjacency into bit planes, build its
zero-tile map, quantize and pack the weights, quantize and pack the features,
then run every layer (aggregate -> requantize -> update -> ReLU + requantize;
the last layer emits fp32).  The workload is the 5-layer GIN of the benchmark
description (65,536 nodes in 64 subgraphs of 1024, hidden 64, s = t = 8).

Prints ONE JSON line.  `value` counts executed bit-operations (2 per 1-bit
multiply-accumulate, only on tiles the zero-tile map keeps) per second of
step time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X vector-ALU ceiling for AND + popcount-accumulate: 256 CUs x 64 lanes per
# clock x 2.4 GHz 32-bit lane operations per second; two lane operations (v_and,
# v_bcnt) cover 32 one-bit multiply-accumulates = 64 bit-operations.
VALU_LANE_OPS = 256 * 64 * 2.4e9
PEAK_BITOPS = VALU_LANE_OPS / 2 * 64          # 1.258e15 bit-op/s

# HBM bytes per launch of the dominant kernel (read + write), from the rocprofv3
# FETCH_SIZE / WRITE_SIZE runs summarized under profiles/ (counters cannot be read
# from inside this process); keyed by (config, bits).  None: not profiled.
TRAFFIC = {(4, 8): 32.4e6}    # profiles/layer_kernel_bench_config4_hbm_traffic.md


def workload_bitops(net, n_nodes, tile_kbits):
    """Executed bit-operations of one forward pass, per kernel family."""
    nnz = int(net.map.nnz_tiles.cpu()[0])
    agg = [2.0 * nnz * 16 * tile_kbits * d * net.s for d, _ in net.dims]
    upd = [2.0 * n_nodes * d * h * net.s * net.t for d, h in net.dims]
    return agg, upd, nnz


def cpu_baseline(w, ranges, total_bitops, sample_blocks=8):
    """The CPU oracle, as it stands, on the first `sample_blocks` subgraphs."""
    import numpy as np
    from oracle import qgnn
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    g = w.graph
    n = sample_blocks * g.block
    A = g.scipy_csr()[:n, :n]
    X = w.X[:n]
    xr = (float(w.X.min()), float(w.X.max()))
    wr = [(float(W.min()), float(W.max())) for W in w.W]
    rqs = [((0, qgnn.inv_scale(0.0, float(r.agg_hi), w.s)),
            None if r.out_hi is None else (0, qgnn.inv_scale(0.0, float(r.out_hi), w.s)))
           for r in ranges]
    best = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        trace, _ = qgnn.forward(A, X, xr, w.W, wr, w.s, w.t, w.model == "gin", rqs=rqs)
        z = trace[-1]["Z"]
        best = min(best, time.perf_counter() - t0)
    frac = n / g.n_nodes
    return {"value": total_bitops * frac / best / 1e12, "unit": "Tbit-op/s",
            "cores": int(threads), "kind": "oracle",
            "sample": f"{sample_blocks} of {g.n_blocks} subgraphs, all layers, best of 3 "
                      f"({best * 1e3:.1f} ms); numpy/scipy integer products",
            "ms": best * 1e3}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload (4 or 5)")
    ap.add_argument("--bits", type=int, default=8)
    ap.add_argument("--tile-kbits", type=int, default=128)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 1 GiB device-to-device copy 5 times (reference point for "
                         "the FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path "
              "(subgraph batches would be sharded with no collective); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2111_09547_amd as q
    from paper_2111_09547_amd.model import QuantGNN, fused_layer_applies
    from workloads import make_workload

    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": src.numel() * 4, "copies": 5}))
        return
    w = make_workload(args.config, bits=args.bits)
    g = w.graph
    A_src = torch.from_numpy(g.dense_compact() if w.storage == "compact" else g.dense()).cuda()
    block_rows = g.block if w.storage == "compact" else 0
    Ws = [torch.from_numpy(W).cuda() for W in w.W]
    X = torch.from_numpy(w.X).cuda()
    xr = (float(w.X.min()), float(w.X.max()))
    self_term = w.model == "gin"
    net = QuantGNN(A_src, Ws, w.s, w.t, self_term, tile_kbits=args.tile_kbits,
                   block_rows=block_rows)
    ranges = net.calibrate(X, xr)          # user-set requantization ranges, outside the timing
    out = torch.empty((g.n_nodes, net.dims[-1][1]), dtype=torch.float32, device="cuda")

    def step():
        net.pack_static(X, xr)
        net.forward(X, xr, ranges, out=out, x_packed=True)

    def layers_only():
        net.forward(X, xr, ranges, out=out)

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    # The step as one HIP graph: the same launches, recorded once, so that the host's
    # per-launch cost (Python + ctypes, ~25 us each) does not limit a step of ~20 launches.
    graph_step = net.capture(X, xr, ranges, out, with_static=True)
    graph_layers = net.capture(X, xr, ranges, out)
    for _ in range(args.warmup):
        graph_step.replay()
    ms_step = timed(graph_step.replay, args.steps)
    # the same steps once more, each between its own pair of events: the median beside the mean
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        graph_step.replay()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    ms_step_median = per_step[len(per_step) // 2]
    # features-to-output only (adjacency, map and weights cached, as the paper does)
    ms_layers = timed(graph_layers.replay, args.steps)
    # the same, launched eagerly from Python
    for _ in range(3):
        step()
    ms_step_eager = timed(step, min(args.steps, 50))

    # the same steps again with HIP events around every kernel launch
    q.qgtc_prof_enable(True)
    q.qgtc_prof_reset()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    kinds = {"pack": q.KERNEL_PACK, "tile_map": q.KERNEL_TILE_MAP, "aggregate": q.KERNEL_AGGREGATE,
             "update": q.KERNEL_UPDATE, "sums": q.KERNEL_SUMS, "layer": q.KERNEL_LAYER}
    prof = {k: q.qgtc_prof_read(v) for k, v in kinds.items()}
    q.qgtc_prof_enable(False)
    q.qgtc_prof_reset()

    # the same forward pass as separate aggregation and update kernels (what the fused
    # layer kernel replaces)
    q.qgtc_set_option(q.OPT_LAYER_PATH, q.LAYER_TWO_KERNELS)
    planes = QuantGNN(A_src, Ws, w.s, w.t, self_term, tile_kbits=args.tile_kbits,
                      block_rows=block_rows, weights_as_bytes=False)
    for _ in range(3):
        planes.forward(X, xr, ranges, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        planes.forward(X, xr, ranges, out=out)
    torch.cuda.synchronize()
    ms_two_kernels = (time.perf_counter() - t0) * 1e3 / 20
    q.qgtc_set_option(q.OPT_LAYER_PATH, q.LAYER_FUSED)
    del planes

    # attainable AND + popcount rate, measured: the aggregation's inner block on registers
    # only, three waves per SIMD as the kernels run (12 workgroups of 1 wave per CU)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    probe_iters, probe_wgs = 500, 256 * 12
    q.qgtc_probe_popcount(probe_wgs, 1, probe_iters, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        q.qgtc_probe_popcount(probe_wgs, 1, probe_iters, sink)
    e1.record()
    torch.cuda.synchronize()
    measured_peak = 3 * probe_wgs * probe_iters * 4 * 128 * 64 * 64.0 / (e0.elapsed_time(e1) * 1e-3)

    # the zero-tile statistic at the paper's 8 x 128 tile (its Figure 8)
    map8 = q.qgtc_build_tile_map(net.A, 8, 128)
    ratio_8x128 = int(map8.nnz_tiles.cpu()[0]) / float(map8.c.n_tile_rows * map8.c.n_tile_cols)
    del map8

    agg_ops, upd_ops, nnz = workload_bitops(net, g.n_nodes, args.tile_kbits)
    total_ops = sum(agg_ops) + sum(upd_ops)
    # the dominant kernel: the fused layer kernel where it applies, else the aggregation
    fused = prof["layer"][1] > 0
    dom_ms, dom_n = prof["layer"] if fused else prof["aggregate"]
    fused_layers = [fused_layer_applies(d, h, w.s, w.t) for d, h in net.dims]
    dom_ops = sum(o for o, f in zip(agg_ops, fused_layers) if f == fused)
    agg_rate = dom_ops * args.steps / (dom_ms * 1e-3)               # bit-op/s over all launches
    n_layers = len(net.dims)
    dense_macs = sum(2.0 * g.n_nodes * g.block * d + 2.0 * g.n_nodes * d * h for d, h in net.dims)
    # every entry of the (block-diagonal) products counted, zero tiles included, times the bit widths
    nominal_ops = sum(2.0 * g.n_nodes * g.block * d * w.s + 2.0 * g.n_nodes * d * h * w.s * w.t
                      for d, h in net.dims)

    rec = {
        "metric": "quantized GNN layer bit-ops/s (TOPS-equiv) + ms/layer, vs VALU/HBM roofline",
        "value": total_ops / (ms_step * 1e-3) / 1e12,
        "unit": "Tbit-op/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": f"config {w.cfg}: {w.name}", "nodes": g.n_nodes,
                   "subgraphs": g.n_blocks, "layers": n_layers, "s_bits": w.s, "t_bits": w.t,
                   "dims": net.dims, "tile": [16, args.tile_kbits],
                   "nonzero_tiles": nnz,
                   "nonzero_tile_ratio": nnz / float(net.map.c.n_tile_rows * net.map.c.n_tile_cols),
                   "nonzero_tile_ratio_8x128": ratio_8x128,
                   "step": "pack A + tile map + pack W + pack X + all layers"},
        "ms_per_step_median": ms_step_median,
        "ms_per_step_eager": ms_step_eager,
        "launch": "one HIP graph per step (the same kernel launches, recorded once)",
        "ms_per_layer": ms_layers / n_layers,
        "ms_layers_only": ms_layers,
        "tops_equiv_dense": dense_macs / (ms_layers * 1e-3) / 1e12,
        "nominal_tbitops": nominal_ops / (ms_layers * 1e-3) / 1e12,
        "ms_layers_two_kernels": ms_two_kernels,
        "roofline": {"bound": "alu", "kernel": "layer_kernel" if fused else "aggregate_kernel",
                     "achieved": agg_rate / 1e12, "peak": PEAK_BITOPS / 1e12,
                     "unit": "Tbit-op/s", "frac": agg_rate / PEAK_BITOPS,
                     "avg_launch_ms": dom_ms / max(dom_n, 1), "launches": dom_n,
                     "counted": "executed AND+popcount bit-ops of the aggregation only; the update "
                                "inside the same kernel runs on the matrix cores and is not counted",
                     "measured_peak": measured_peak / 1e12,
                     "frac_of_measured_peak": agg_rate / measured_peak,
                     "traffic": TRAFFIC.get((w.cfg, w.s))},
        "kernels": {k: {"ms_per_step": v[0] / args.steps, "launches_per_step": v[1] / args.steps}
                    for k, v in prof.items()},
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(w, ranges, total_ops)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
