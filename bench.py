#!/usr/bin/env python3
"""Benchmark of the quantized GNN layer path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM: pack the adjacency into bit planes, build its
zero-tile map, quantize and pack the weights, quantize and pack the features,
then run every layer (aggregate -> requantize -> update -> ReLU + requantize;
the last layer emits fp32).  The workload of the headline line is the 5-layer GIN
of the benchmark description (config 4: 65,536 nodes in 64 subgraphs of 1024,
hidden 64, s = t = 8); `other_configs` carries the bit-width sweep of config 3 and
the zero-tile config 5 at s = t in {1, 2, 4, 8}.

Prints ONE JSON line.  `value` counts executed bit-operations (2 per 1-bit
multiply-accumulate, only on tiles the zero-tile map keeps; the update at its
nominal 2 N D H s t although it runs as int8 multiply-accumulates) per second of step
time; `value_popcount_executed` counts the aggregation's AND + popcount work alone.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X vector-ALU ceiling for AND + popcount-accumulate: 256 CUs x 64 lanes per
# clock x 2.4 GHz 32-bit lane operations per second; two lane operations (v_and,
# v_bcnt) cover 32 one-bit multiply-accumulates = 64 bit-operations.
VALU_LANE_OPS = 256 * 64 * 2.4e9
PEAK_BITOPS = VALU_LANE_OPS / 2 * 64          # 1.258e15 bit-op/s
METRIC = "quantized GNN layer bit-ops/s (TOPS-equiv) + ms/layer, vs VALU/HBM roofline"


def make_net(cfg, bits, tile_kbits, w=None):
    """Workload (made here unless given: the same graph and features serve every bit width),
    its tensors on the device and the layer stack, calibrated."""
    import dataclasses
    import torch
    from paper_2111_09547_amd.model import QuantGNN
    from workloads import make_workload
    if w is None:
        w = make_workload(cfg, bits=bits)
    elif w.s != bits:
        w = dataclasses.replace(w, s=bits, t=bits)
    g = w.graph
    compact = w.storage == "compact"
    A_src = torch.from_numpy(g.dense_compact() if compact else g.dense()).cuda()
    Ws = [torch.from_numpy(W).cuda() for W in w.W]
    X = torch.from_numpy(w.X).cuda()
    xr = (float(w.X.min()), float(w.X.max()))
    net = QuantGNN(A_src, Ws, w.s, w.t, w.model == "gin", tile_kbits=tile_kbits,
                   block_rows=g.block if compact else 0)
    ranges = net.calibrate(X, xr)          # user-set requantization ranges, outside the timing
    out = torch.empty((g.n_nodes, net.dims[-1][1]), dtype=torch.float32, device="cuda")
    return w, net, A_src, Ws, X, xr, ranges, out


def workload_bitops(net, n_nodes):
    """Bit-operations of one forward pass, per layer: the aggregation over the tiles the
    zero-tile map keeps, the update (nominal), the number of kept tiles, and the
    aggregation over the words the kernels really visit - the same as the first list unless
    they jump over the zero words inside kept tiles (then: 32 bits per (row, word) pair of A
    that holds a bit)."""
    import paper_2111_09547_amd as q
    nnz = int(net.map.nnz_tiles.cpu()[0])
    kb = net.map.c.tile_kbits
    agg = [2.0 * nnz * 16 * kb * d * net.s for d, _ in net.dims]
    upd = [2.0 * n_nodes * d * h * net.s * net.t for d, h in net.dims]
    jumping = (net.tuning is not None and net.tuning.zero_words == q.ZERO_WORDS_SKIP and net.s >= 3
               and net.plan is not None)
    visited = [2.0 * net.plan["nnz_row_words"] * 32 * d * net.s for d, _ in net.dims] if jumping else list(agg)
    return agg, upd, nnz, visited


def timed(fn, n):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / n


def timed_in_flight(graphs, n):
    """n graph replays in all, dealt round-robin to one stream per graph: ms per replay."""
    import torch
    streams = [torch.cuda.Stream() for _ in graphs]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        with torch.cuda.stream(streams[i % len(graphs)]):
            graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / n


def kernel_events(fn, steps):
    """Runs fn `steps` times with the library's HIP events around every kernel launch
    (recorded on the launch stream): {kind: (total ms, launches)}."""
    import torch
    import paper_2111_09547_amd as q
    kinds = {"pack": q.KERNEL_PACK, "tile_map": q.KERNEL_TILE_MAP, "aggregate": q.KERNEL_AGGREGATE,
             "update": q.KERNEL_UPDATE, "sums": q.KERNEL_SUMS, "layer": q.KERNEL_LAYER}
    q.qgtc_prof_enable(True)
    q.qgtc_prof_reset()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    prof = {k: q.qgtc_prof_read(v) for k, v in kinds.items()}
    q.qgtc_prof_enable(False)
    q.qgtc_prof_reset()
    return prof


def dominant_kernel(net, w, prof, steps, agg_ops):
    """The kernel that carries the aggregation: the fused layer kernel where it applies,
    else the aggregation kernel.  Returns (name, achieved bit-op/s, avg launch ms, launches)."""
    from paper_2111_09547_amd.model import fused_layer_applies
    fused = prof["layer"][1] > 0
    dom_ms, dom_n = prof["layer"] if fused else prof["aggregate"]
    fused_layers = [fused_layer_applies(d, h, w.s, w.t) for d, h in net.dims]
    dom_ops = sum(o for o, f in zip(agg_ops, fused_layers) if f == fused)
    rate = dom_ops * steps / (dom_ms * 1e-3) if dom_ms > 0 else 0.0
    return ("layer_kernel" if fused else "aggregate_kernel"), rate, dom_ms / max(dom_n, 1), dom_n


def ratio_8x128(net):
    """The zero-tile statistic at the paper's 8 x 128 tile (its Figure 8)."""
    import paper_2111_09547_amd as q
    m = q.qgtc_build_tile_map(net.A, 8, 128)
    return int(m.nnz_tiles.cpu()[0]) / float(m.c.n_tile_rows * m.c.n_tile_cols)


def side_config(cfg, bits, steps, warmup, w=None):
    """One entry of other_configs: forward pass (pack X + all layers) as one HIP graph."""
    import torch
    w, net, A_src, Ws, X, xr, ranges, out = make_net(cfg, bits, "auto", w)
    g = w.graph
    graph = net.capture(X, xr, ranges, out, streams=net.auto_runs())
    for _ in range(warmup):
        graph.replay()
    ms = timed(graph.replay, steps)
    del graph
    prof = kernel_events(lambda: net.forward(X, xr, ranges, out=out), steps)
    agg_ops, upd_ops, nnz, visited = workload_bitops(net, g.n_nodes)
    name, rate, avg_ms, launches = dominant_kernel(net, w, prof, steps, visited)
    rec = {"config": cfg, "s_bits": w.s, "t_bits": w.t, "nodes": g.n_nodes, "dims": net.dims,
           "ms_forward": ms, "ms_per_layer": ms / len(net.dims),
           "tbitops_kept_tiles": sum(agg_ops) / (ms * 1e-3) / 1e12,
           "tbitops_popcount_executed": sum(visited) / (ms * 1e-3) / 1e12,
           "tbitops_update_nominal": sum(upd_ops) / (ms * 1e-3) / 1e12,
           "zero_word_jumping": visited != agg_ops,
           "visited_share_of_kept_tiles": sum(visited) / max(sum(agg_ops), 1.0),
           "tile": [16, net.map.c.tile_kbits], "nonzero_tiles": nnz,
           "nonzero_tile_ratio_8x128": ratio_8x128(net),
           "dominant_kernel": name, "avg_launch_ms": avg_ms, "launches": launches,
           "frac": rate / PEAK_BITOPS}
    del net, A_src, X, out
    torch.cuda.empty_cache()
    return rec


# ---------------------------------------------------------------- HBM traffic (rocprofv3)
def traffic_child(cfg, bits, tile_kbits="auto"):
    """What the counter runs execute: a device-to-device copy of known size (the reference
    the counters are scaled by), then a few forward passes."""
    import torch
    w, net, A_src, Ws, X, xr, ranges, out = make_net(cfg, bits, tile_kbits)
    src = torch.ones(1 << 26, dtype=torch.int32, device="cuda")      # 256 MiB
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    for _ in range(4):
        net.forward(X, xr, ranges, out=out)
    torch.cuda.synchronize()
    print(json.dumps({"copy_kib": src.numel() * 4 // 1024}))


def measure_traffic(cfg, bits, kernel_substr="layer_kernel", timeout=150, tile_kbits="auto"):
    """HBM bytes per launch of the dominant kernel (read + written), from two rocprofv3
    counter runs of this script (FETCH_SIZE, then WRITE_SIZE, KiB-like units per dispatch),
    each scaled by what the same counter reads for a plain copy of known size.  None when
    the profiler is not there or a run fails."""
    rocprof = "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(rocprof):
        return None, "rocprofv3 not found"
    total, notes = 0.0, []
    for counter, copy_dir in (("FETCH_SIZE", "read"), ("WRITE_SIZE", "written")):
        with tempfile.TemporaryDirectory(dir="/tmp") as tmp:
            cmd = [rocprof, "--pmc", counter, "--kernel-trace", "--output-format", "csv", "-d", tmp, "--",
                   sys.executable, os.path.abspath(__file__), "--traffic-child", "--config", str(cfg),
                   "--bits", str(bits), "--tile-kbits", str(tile_kbits)]
            env = dict(os.environ, TMPDIR="/tmp")
            try:
                proc = subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                                      text=True, timeout=timeout)
            except (subprocess.TimeoutExpired, OSError) as e:
                return None, f"{counter} run: {type(e).__name__}"
            files = glob.glob(os.path.join(tmp, "**", "*counter_collection.csv"), recursive=True)
            if proc.returncode != 0 or not files:
                return None, f"{counter} run failed (rc {proc.returncode})"
            copy_kib = None
            for line in proc.stdout.splitlines():
                if line.startswith("{") and "copy_kib" in line:
                    copy_kib = json.loads(line)["copy_kib"]
            import csv
            copy_vals, kern_vals = [], []
            with open(files[0]) as f:
                for row in csv.DictReader(f):
                    if row["Counter_Name"] != counter:
                        continue
                    name, val = row["Kernel_Name"], float(row["Counter_Value"])
                    if "copyBuffer" in name and int(row["Grid_Size"]) > 4096:
                        copy_vals.append(val)
                    elif kernel_substr in name:
                        kern_vals.append(val)
            if not copy_vals or not kern_vals or not copy_kib:
                return None, f"{counter}: kernels not found in the counter file"
            ref = sorted(copy_vals)[len(copy_vals) // 2]
            factor = copy_kib / ref                      # KiB per counter unit
            mean = sum(kern_vals) / len(kern_vals)
            total += mean * factor * 1024.0
            notes.append(f"{counter} x {factor:.3f} KiB ({len(kern_vals)} launches)")
    return total, "; ".join(notes)


# ---------------------------------------------------------------- the oracle on the host
def cpu_baseline(w, ranges, total_bitops, sample_blocks=8):
    """The CPU oracle, as it stands, on the first `sample_blocks` subgraphs, in its two
    forms: sparse adjacency (scipy CSR product, one thread) and dense 0/1 blocks (float64
    BLAS product, the BLAS pool's threads)."""
    import numpy as np
    from oracle import qgnn
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas_threads = os.cpu_count() or 1
    g = w.graph
    n = sample_blocks * g.block
    xr = (float(w.X.min()), float(w.X.max()))
    wr = [(float(W.min()), float(W.max())) for W in w.W]
    rqs = [((0, qgnn.inv_scale(0.0, float(r.agg_hi), w.s)),
            None if r.out_hi is None else (0, qgnn.inv_scale(0.0, float(r.out_hi), w.s)))
           for r in ranges]
    gin = w.model == "gin"
    frac = n / g.n_nodes

    A = g.scipy_csr()[:n, :n]
    best_csr = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        qgnn.forward(A, w.X[:n], xr, w.W, wr, w.s, w.t, gin, rqs=rqs)
        best_csr = min(best_csr, time.perf_counter() - t0)

    blocks = [A[b * g.block:(b + 1) * g.block, b * g.block:(b + 1) * g.block].toarray().astype(np.uint8)
              for b in range(sample_blocks)]
    best_dense = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        for b, Ab in enumerate(blocks):                 # subgraphs are independent graphs
            qgnn.forward(Ab, w.X[b * g.block:(b + 1) * g.block], xr, w.W, wr, w.s, w.t, gin, rqs=rqs)
        best_dense = min(best_dense, time.perf_counter() - t0)

    variants = [
        {"form": "sparse adjacency: scipy CSR integer product (single-threaded) + float64 BLAS update",
         "ms": best_csr * 1e3, "value": total_bitops * frac / best_csr / 1e12, "cores": 1},
        {"form": "dense 0/1 blocks: float64 BLAS products (exact below 2^53)",
         "ms": best_dense * 1e3, "value": total_bitops * frac / best_dense / 1e12, "cores": int(blas_threads)},
    ]
    best = max(variants, key=lambda v: v["value"])
    return {"value": best["value"], "unit": "Tbit-op/s", "cores": best["cores"], "kind": "oracle",
            "sample": f"{sample_blocks} of {g.n_blocks} subgraphs, all layers, best of 3, faster of the oracle's "
                      f"two input forms ({best['form']})",
            "ms": best["ms"], "variants": variants}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload of the headline line (3, 4 or 5)")
    ap.add_argument("--bits", type=int, default=8)
    ap.add_argument("--tile-kbits", default="auto",
                    help="width of the zero-tile map's tiles: 32, 64, 128 or auto (the library's selector, "
                         "decided once per adjacency)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--no-traffic", action="store_true", help="skip the two rocprofv3 counter runs")
    ap.add_argument("--runs", type=int, default=-1,
                    help="independent runs of subgraphs (streams) per forward pass; default: what the "
                         "library's selector says (QuantGNN.auto_runs)")
    ap.add_argument("--no-in-flight", action="store_true",
                    help="skip the throughput runs with two and three batches in flight")
    ap.add_argument("--traffic-child", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 1 GiB device-to-device copy 5 times (reference point for "
                         "the FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.tile_kbits != "auto":
        args.tile_kbits = int(args.tile_kbits)
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path "
              "(subgraph batches would be sharded with no collective); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    # The counter runs are child processes of their own (rocprofv3 around this script); they
    # come first, before this process touches the GPU.
    traffic, traffic_note = (None, "skipped")
    dom_guess = "layer_kernel" if args.bits <= 8 else "aggregate_kernel"
    if not (args.no_traffic or args.traffic_child or args.copy_calibration):
        traffic, traffic_note = measure_traffic(args.config, args.bits, dom_guess, tile_kbits=args.tile_kbits)

    import torch
    import paper_2111_09547_amd as q
    from paper_2111_09547_amd.model import QuantGNN

    torch.cuda.set_device(0)
    if args.traffic_child:
        traffic_child(args.config, args.bits, args.tile_kbits)
        return
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": src.numel() * 4, "copies": 5}))
        return

    w, net, A_src, Ws, X, xr, ranges, out = make_net(args.config, args.bits, args.tile_kbits)
    g = w.graph
    self_term = w.model == "gin"
    block_rows = g.block if w.storage == "compact" else 0

    def step():
        net.pack_static(X, xr)
        net.forward(X, xr, ranges, out=out, x_packed=True)

    # The step as one HIP graph: the same launches, recorded once, so that the host's
    # per-launch cost (Python + ctypes, ~25 us each) does not limit a step of ~20 launches.
    n_runs = net.auto_runs() if args.runs < 0 else args.runs
    graph_step = net.capture(X, xr, ranges, out, with_static=True, streams=n_runs)
    graph_layers = net.capture(X, xr, ranges, out, streams=n_runs)
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
    if n_runs > 1:
        g1 = net.capture(X, xr, ranges, out)
        ms_layers_one_run = timed(g1.replay, args.steps)
        del g1
    else:
        ms_layers_one_run = ms_layers
    # the same, launched eagerly from Python
    for _ in range(3):
        step()
    ms_step_eager = timed(step, min(args.steps, 50))

    # Throughput with several independent batches in flight: every batch has its own buffers
    # and its own graph (the same step), replayed round-robin on one stream per batch, so the
    # drain of one batch's launches overlaps the start of another's.  The headline fields stay
    # one batch at a time.
    in_flight = []
    if not args.no_in_flight:
        more = [make_net(args.config, args.bits, net.map.c.tile_kbits, w) for _ in range(2)]
        g_steps = [graph_step] + [m[1].capture(m[4], m[5], m[6], m[7], with_static=True, streams=n_runs) for m in more]
        g_layers = [graph_layers] + [m[1].capture(m[4], m[5], m[6], m[7], streams=n_runs) for m in more]
        for k in (2, 3):
            timed_in_flight(g_steps[:k], 2 * k)
            in_flight.append({"batches": k, "ms_per_step": timed_in_flight(g_steps[:k], args.steps),
                              "ms_layers_only": timed_in_flight(g_layers[:k], args.steps)})
        for m in more:
            assert torch.equal(m[7], out)               # every batch computed the same output
        del g_steps, g_layers, more

    # the same steps again with HIP events around every kernel launch
    prof = kernel_events(step, args.steps)

    # the same forward pass as separate aggregation and update kernels (what the fused
    # layer kernel replaces)
    planes = QuantGNN(A_src, Ws, w.s, w.t, self_term, tile_kbits=net.map.c.tile_kbits,
                      block_rows=block_rows, weights_as_bytes=False,
                      tuning=q.Tuning(layer_path=q.LAYER_TWO_KERNELS))
    for _ in range(3):
        planes.forward(X, xr, ranges, out=out)
    ms_two_kernels = timed(lambda: planes.forward(X, xr, ranges, out=out), 20)
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

    agg_ops, upd_ops, nnz, visited = workload_bitops(net, g.n_nodes)
    total_ops = sum(agg_ops) + sum(upd_ops)
    dom_name, agg_rate, dom_avg_ms, dom_n = dominant_kernel(net, w, prof, args.steps, visited)
    # the same launches with every word of the kept tiles visited (the form whose work is the
    # tile-level count: bound by the vector ALUs)
    visit_all = None
    if visited != agg_ops:
        keep = net.tuning
        net.tuning = q.Tuning(update_path=keep.update_path, agg_xcd_run=keep.agg_xcd_run, layer_path=keep.layer_path,
                              layer_ksplit=keep.layer_ksplit, zero_words=q.ZERO_WORDS_VISIT,
                              even_progress=keep.even_progress)
        for _ in range(3):
            step()
        prof_v = kernel_events(step, args.steps)
        g_v = net.capture(X, xr, ranges, out, streams=n_runs)
        ms_layers_v = timed(g_v.replay, args.steps)
        del g_v
        net.tuning = keep
        _, rate_v, avg_v, _ = dominant_kernel(net, w, prof_v, args.steps, agg_ops)
        visit_all = {"frac": rate_v / PEAK_BITOPS, "avg_launch_ms": avg_v, "ms_layers_only": ms_layers_v}
    n_layers = len(net.dims)
    dense_macs = sum(2.0 * g.n_nodes * g.block * d + 2.0 * g.n_nodes * d * h for d, h in net.dims)
    # every entry of the (block-diagonal) products counted, zero tiles included, times the bit widths
    nominal_ops = sum(2.0 * g.n_nodes * g.block * d * w.s + 2.0 * g.n_nodes * d * h * w.s * w.t
                      for d, h in net.dims)
    tile_kbits = net.map.c.tile_kbits

    if dom_name != dom_guess:
        traffic, traffic_note = None, f"counter runs looked for {dom_guess}, the step ran {dom_name}"

    rec = {
        "metric": METRIC,
        "value": total_ops / (ms_step * 1e-3) / 1e12,
        "unit": "Tbit-op/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": f"config {w.cfg}: {w.name}", "nodes": g.n_nodes,
                   "subgraphs": g.n_blocks, "layers": n_layers, "s_bits": w.s, "t_bits": w.t,
                   "dims": net.dims, "tile": [16, tile_kbits],
                   "nonzero_tiles": nnz,
                   "nonzero_tile_ratio": nnz / float(net.map.c.n_tile_rows * net.map.c.n_tile_cols),
                   "nonzero_tile_ratio_8x128": ratio_8x128(net),
                   "step": "pack A + tile map + pack W + pack X + all layers"},
        "value_counts": "aggregation: AND + popcount bit-ops of the tiles the zero-tile map keeps (where the kernels "
                        "also jump over the zero words inside kept tiles, value_popcount_executed counts only "
                        "the words they visit); update: nominal 2 N D H s t (it executes as int8 "
                        "multiply-accumulates on the matrix cores)",
        "value_popcount_kept_tiles": sum(agg_ops) / (ms_step * 1e-3) / 1e12,
        "value_popcount_executed": sum(visited) / (ms_step * 1e-3) / 1e12,
        "zero_word_jumping": visited != agg_ops,
        "visited_share_of_kept_tiles": sum(visited) / max(sum(agg_ops), 1.0),
        "value_update_nominal": sum(upd_ops) / (ms_step * 1e-3) / 1e12,
        "ms_per_step_median": ms_step_median,
        "ms_per_step_eager": ms_step_eager,
        "launch": "one HIP graph per step (the same kernel launches, recorded once); the layers of a batch "
                  f"run as {n_runs} independent run(s) of subgraphs on as many streams inside the graph",
        "ms_layers_only_one_run": ms_layers_one_run,
        "ms_per_layer": ms_layers / n_layers,
        "ms_layers_only": ms_layers,
        "tops_equiv_dense": dense_macs / (ms_layers * 1e-3) / 1e12,
        "nominal_tbitops": nominal_ops / (ms_layers * 1e-3) / 1e12,
        "ms_layers_two_kernels": ms_two_kernels,
        "batches_in_flight": [dict(r, value=total_ops / (r["ms_per_step"] * 1e-3) / 1e12,
                                   aggregation_frac_of_peak=sum(visited) / (r["ms_layers_only"] * 1e-3) / PEAK_BITOPS)
                              for r in in_flight],
        "roofline": {"bound": "alu", "kernel": dom_name,
                     "achieved": agg_rate / 1e12, "peak": PEAK_BITOPS / 1e12,
                     "unit": "Tbit-op/s", "frac": agg_rate / PEAK_BITOPS,
                     "avg_launch_ms": dom_avg_ms, "launches": dom_n,
                     "counted": "executed (visited) AND+popcount bit-ops of the aggregation only; the update "
                                "inside the same kernel runs on the matrix cores and is not counted; launch "
                                "durations are taken with the launches one after the other on one stream",
                     "frac_in_step": sum(visited) / (ms_layers * 1e-3) / PEAK_BITOPS,
                     # the work of the kept tiles (what a kernel without zero-word jumping executes, and
                     # what `frac` counted before that existed) over the same launch time: above 1 when
                     # the jumping form skips more than the vector ALUs could have done
                     "frac_kept_tile_work": agg_rate / PEAK_BITOPS * (sum(agg_ops) / sum(visited)),
                     "visit_all_form": visit_all,
                     "measured_peak": measured_peak / 1e12,
                     "frac_of_measured_peak": agg_rate / measured_peak,
                     "traffic": traffic, "traffic_source": traffic_note},
        "kernels": {k: {"ms_per_step": v[0] / args.steps, "launches_per_step": v[1] / args.steps}
                    for k, v in prof.items()},
    }
    del graph_step, graph_layers
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(w, ranges, total_ops)
    del net, A_src, X, out
    torch.cuda.empty_cache()
    if not args.no_other_configs:
        from workloads import make_workload
        others = []
        side_steps = max(10, min(args.steps, 30))
        for cfg, sweep in ((5, (1, 2, 4, 8)), (3, (1, 2, 3, 4, 5, 6, 7, 8, 16, 32))):
            wl = make_workload(cfg, bits=sweep[0])
            for bits in sweep:
                others.append(side_config(cfg, bits, side_steps, 3, wl))
            del wl
        rec["other_configs"] = others
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
