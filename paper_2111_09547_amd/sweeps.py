"""Measurement sweeps beside bench.py (one GPU, synthetic inputs, HIP events):

  table3   the aggregation A(1 bit) x X(s bits) at the shapes of the paper's Table 3
           (N in {2048, 4096, 8192}, D in {32, 64}, s = 1..4), every tile non-zero,
           as full-precision-equivalent TFLOP/s = 2 N^2 D / t (the paper's unit)
  config3  one layer per bit width (s = t in 1..8, 16, 32) on the 8 x 1024 batch
  config5  the 2-layer GCN on the power-law graph for s = t in {1, 2, 4, 8}, with 128-, 64- and
           32-bit tiles, and in the update-first order A.(X.W)

  sizes    the 1-bit x 1-bit aggregation over N in {128 .. 32768} and D in {16 .. 1024}
           (the paper's adjacency-matrix-size study, Fig. 9), every tile non-zero
  reuse    the paper's tile-reuse study (Fig. 10): D = 1024, N in {1024 .. 8192}, X with 4,
           8 and 16 bits, A read once for all planes (one launch) against once per plane
           (s one-bit launches)
  transfer host -> device cost of a batch (Section 4.6): dense fp32 adjacency + fp32
           features in two copies against the low-bit compound buffer packed on the host
           and copied once (configs 4 and 5; pinned memory on both sides)
  gate     the stand-alone update Y.W as s*t one-bit products (AND + popcount, Algorithm 1's
           second loop) against the same product on the int8 matrix cores, s = t = 1..8, at
           the update shapes of configs 4 and 5, int32 and low-bit outputs: the measurement
           behind the selector's rule for the update (qgtc_plan_layer)
  streaming the HBM-bound kernels one at a time at the shapes of configs 4 and 5: packing the
           adjacency and the features, the zero-tile map and statistics, the update on the
           matrix cores from planes and from bytes; achieved TB/s of algorithmic bytes
  tiles    cost of an adjacency bit by tile width (16 x 32 / 64 / 128) on configs 4 and 5:
           the measurement behind the selector's tile-width rule

Run:  python -m paper_2111_09547_amd.sweeps [table3|config3|config5|sizes|reuse|transfer|gate|streaming|tiles ...]
Prints one JSON line per measurement and a markdown table per sweep."""
from __future__ import annotations

import json
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2111_09547_amd as q                         # noqa: E402
from paper_2111_09547_amd.model import QuantGNN          # noqa: E402

PEAK_BITOPS = 256 * 64 * 2.4e9 / 2 * 64                  # vector-ALU AND + popcount ceiling, bit-op/s


def timeit(fn, n=20, warm=3, reps=5):
    """Median over `reps` groups of n calls, in microseconds per call."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) / n * 1e3)
    return sorted(ts)[len(ts) // 2]


def _planned(ab, d, s_bits, mode=None):
    """An int32-output epilogue with the tuning the selector gives for this adjacency (a user
    would plan once per adjacency: these sweeps use dense random matrices, where visiting
    every word of a tile beats jumping over the few zero ones)."""
    st = q.tile_stats_numbers(q.qgtc_tile_stats(ab))
    plan = q.qgtc_plan_layer(ab.rows, d, d, min(s_bits, 8), 8, n_tile_rows=st["n_tile_rows"], a_cols=ab.cols,
                             nnz_tiles=st["nnz_tiles"], nnz_row_words=st["nnz_row_words"])
    return q.Epilogue(mode=q.OUT_I32 if mode is None else mode, tuning=q.Tuning(zero_words=plan["zero_words"]))


def table3():
    rows = []
    gen = torch.Generator(device="cuda").manual_seed(3)
    for d in (32, 64):
        for n in (2048, 4096, 8192):
            a = (torch.rand((n, n), device="cuda", generator=gen) < 0.5).to(torch.uint8)
            ab = q.qgtc_pack_bits(a, 1, q.LEFT)
            tmap = q.qgtc_build_tile_map(ab, 16, 128)
            assert int(tmap.nnz_tiles.cpu()[0]) == (n // 16) * (n // 128)
            rec = {"sweep": "table3", "N": n, "D": d}
            for s in (1, 2, 3, 4):
                x = torch.randint(0, 2 ** s, (n, d), dtype=torch.int32, device="cuda", generator=gen)
                xb = q.qgtc_pack_bits(x, s, q.RIGHT)
                ep = _planned(ab, d, s)
                out = q.qgtc_aggregate(ab, tmap, xb, ep)
                t = timeit(lambda: q.qgtc_aggregate(ab, tmap, xb, ep, out=out))
                rec[f"us_{s}bit"] = round(t, 2)
                rec[f"tflops_equiv_{s}bit"] = round(2.0 * n * n * d / t / 1e6, 1)
                rec[f"frac_valu_{s}bit"] = round(2.0 * n * n * d * s / (t * 1e-6) / PEAK_BITOPS, 3)
            print(json.dumps(rec), flush=True)
            rows.append(rec)
    print("\n| N | D | 1-bit | 2-bit | 3-bit | 4-bit |  (TFLOP/s-equivalent = 2 N^2 D / t; in brackets: "
          "fraction of the vector-ALU popcount ceiling)")
    print("|---|---|---|---|---|---|")
    for r in rows:
        cells = " | ".join(f"{r[f'tflops_equiv_{s}bit']} ({r[f'frac_valu_{s}bit']})" for s in (1, 2, 3, 4))
        print(f"| {r['N']} | {r['D']} | {cells} |")


def _layer_bitops(net, n_nodes, kb):
    nnz = int(net.map.nnz_tiles.cpu()[0])
    agg = sum(2.0 * nnz * 16 * kb * d * net.s for d, _ in net.dims)
    upd = sum(2.0 * n_nodes * d * h * net.s * net.t for d, h in net.dims)
    return agg, upd


def _model_sweep(cfg, bit_list, kb=128, update_first=False):
    from workloads import make_workload
    rows = []
    for bits in bit_list:
        w = make_workload(cfg, bits=bits)
        g = w.graph
        compact = w.storage == "compact"
        a_src = torch.from_numpy(g.dense_compact() if compact else g.dense()).cuda()
        ws = [torch.from_numpy(W).cuda() for W in w.W]
        x = torch.from_numpy(w.X).cuda()
        xr = (float(w.X.min()), float(w.X.max()))
        net = QuantGNN(a_src, ws, w.s, w.t, w.model == "gin", tile_kbits=kb,
                       block_rows=g.block if compact else 0, update_first=update_first)
        ranges = net.calibrate(x, xr)
        out = torch.empty((g.n_nodes, net.dims[-1][1]), dtype=torch.float32, device="cuda")
        graph = net.capture(x, xr, ranges, out)      # one graph launch per pass: no per-kernel host cost
        t = timeit(graph.replay, n=10, warm=30)      # the first case also wakes the clocks up
        del graph
        agg, upd = _layer_bitops(net, g.n_nodes, kb)
        if update_first:                 # the aggregation then runs on the H output columns
            nnz = int(net.map.nnz_tiles.cpu()[0])
            agg = sum(2.0 * nnz * 16 * kb * h * net.s for _, h in net.dims)
        rec = {"sweep": f"config{cfg}", "order": "update first" if update_first else "aggregate first",
               "bits": bits, "layers": len(net.dims), "us_forward": round(t, 1),
               "us_per_layer": round(t / len(net.dims), 1),
               "tbitops_executed": round((agg + upd) / t / 1e6, 1),
               "agg_frac_valu": round(agg / (t * 1e-6) / PEAK_BITOPS, 3),
               "tile_kbits": kb, "nonzero_tiles": int(net.map.nnz_tiles.cpu()[0])}
        print(json.dumps(rec), flush=True)
        rows.append(rec)
        del net, a_src, x
        torch.cuda.empty_cache()
    print(f"\nconfig {cfg}, {rows[0]['order']}, tiles of 16 x {kb}:")
    print(f"\n| s = t | forward (pack X + {rows[0]['layers']} layer(s)) us | Tbit-op/s of the kept tiles | "
          "kept-tile aggregation bit-ops / forward time over the vector-ALU ceiling (from 3 bits on the kernels "
          "jump over zero words inside kept tiles and visit only part of them) |")
    print("|---|---|---|---|")
    for r in rows:
        print(f"| {r['bits']} | {r['us_forward']} | {r['tbitops_executed']} | {r['agg_frac_valu']} |")


def config3():
    _model_sweep(3, (1, 2, 3, 4, 5, 6, 7, 8, 16, 32))


def config5():
    for kb in (128, 64, 32):
        _model_sweep(5, (1, 2, 4, 8), kb=kb)
    _model_sweep(5, (1, 2, 4, 8), kb=128, update_first=True)


def _random_bits(rows, cols, nbits, layout, gen):
    """Packed operand of uniformly random bits (no dense source: N = 32768 would need 1 GiB)."""
    b = q.alloc_bits(rows, cols, nbits, layout)
    b.words.copy_(torch.randint(-2 ** 31, 2 ** 31 - 1, b.words.shape, dtype=torch.int64, device="cuda",
                                generator=gen).to(torch.int32))
    if layout == q.LEFT and cols % 32:              # padding bits of the last word stay zero
        raise ValueError("columns must fill whole words")
    return b


def sizes():
    gen = torch.Generator(device="cuda").manual_seed(9)
    ns = (128, 256, 512, 1024, 2048, 4096, 8192, 16384, 32768)
    ds = (16, 32, 64, 128, 256, 512, 1024)
    table = {}
    for n in ns:
        ab = _random_bits(n, n, 1, q.LEFT, gen)
        tmap = q.qgtc_build_tile_map(ab, 16, 128)
        for d in ds:
            xb = _random_bits(n, d, 1, q.RIGHT, gen)
            ep = _planned(ab, d, 1)
            out = q.qgtc_aggregate(ab, tmap, xb, ep)
            t = timeit(lambda: q.qgtc_aggregate(ab, tmap, xb, ep, out=out), n=10 if n >= 8192 else 20)
            rec = {"sweep": "sizes", "N": n, "D": d, "us": round(t, 2),
                   "tflops_equiv": round(2.0 * n * n * d / t / 1e6, 1),
                   "frac_valu": round(2.0 * n * n * d / (t * 1e-6) / PEAK_BITOPS, 3)}
            print(json.dumps(rec), flush=True)
            table[(n, d)] = rec
            del xb, out
        del ab, tmap
        torch.cuda.empty_cache()
    print("\n1-bit x 1-bit aggregation, TFLOP/s-equivalent = 2 N^2 D / t (fraction of the vector-ALU ceiling):")
    print("\n| N \\ D | " + " | ".join(str(d) for d in ds) + " |")
    print("|---|" + "---|" * len(ds))
    for n in ns:
        print(f"| {n} | " + " | ".join(f"{table[(n, d)]['tflops_equiv']} ({table[(n, d)]['frac_valu']})" for d in ds) + " |")


def reuse():
    gen = torch.Generator(device="cuda").manual_seed(10)
    d = 1024
    rows = []
    for n in (1024, 2048, 4096, 8192):
        ab = _random_bits(n, n, 1, q.LEFT, gen)
        tmap = q.qgtc_build_tile_map(ab, 16, 128)
        ep = _planned(ab, d, 8)
        x1 = _random_bits(n, d, 1, q.RIGHT, gen)
        out = q.qgtc_aggregate(ab, tmap, x1, ep)
        t1 = timeit(lambda: q.qgtc_aggregate(ab, tmap, x1, ep, out=out), n=10)
        rec = {"sweep": "reuse", "N": n, "D": d, "us_1bit": round(t1, 1)}
        for s_bits in (4, 8, 16):
            xs = _random_bits(n, d, s_bits, q.RIGHT, gen)
            ts = timeit(lambda: q.qgtc_aggregate(ab, tmap, xs, ep, out=out), n=10)
            rec[f"us_{s_bits}bit_one_launch"] = round(ts, 1)
            rec[f"us_{s_bits}bit_plane_by_plane"] = round(s_bits * t1, 1)
            rec[f"tflops_equiv_{s_bits}bit"] = round(2.0 * n * n * d / ts / 1e6, 1)
            del xs
        print(json.dumps(rec), flush=True)
        rows.append(rec)
        del ab, tmap, x1, out
        torch.cuda.empty_cache()
    print("\nA read once for all planes (one launch) against once per plane (s launches of the 1-bit kernel), us:")
    print("\n| N | 4 bit: one launch / per plane | 8 bit | 16 bit |")
    print("|---|---|---|---|")
    for r in rows:
        print(f"| {r['N']} | " + " | ".join(f"{r[f'us_{b}bit_one_launch']} / {r[f'us_{b}bit_plane_by_plane']}"
                                             for b in (4, 8, 16)) + " |")


def transfer():
    import time
    from workloads import make_workload
    from .packing import SubgraphPacket
    rows = []
    for cfg in (4, 5):
        w = make_workload(cfg)
        g = w.graph
        a_u8 = torch.from_numpy(g.dense_compact())
        x = torch.from_numpy(w.X)
        xr = (float(w.X.min()), float(w.X.max()))
        a_f32 = a_u8.to(torch.float32).pin_memory()
        x_pin = x.pin_memory()
        da, dx = torch.empty_like(a_f32, device="cuda"), torch.empty_like(x_pin, device="cuda")

        def dense():
            da.copy_(a_f32, non_blocking=True)
            dx.copy_(x_pin, non_blocking=True)
        t_dense = timeit(dense, n=3, warm=1, reps=3)
        pk = SubgraphPacket(g.n_nodes, g.block, x.shape[1], w.s, block_rows=g.block)
        t_pack = float("inf")
        for _ in range(3):
            t0 = time.perf_counter()
            pk.pack(a_u8, x, xr, threads=16)
            t_pack = min(t_pack, (time.perf_counter() - t0) * 1e6)
        t_low = timeit(pk.upload, n=3, warm=1, reps=3)
        dense_bytes = a_f32.numel() * 4 + x_pin.numel() * 4
        rec = {"sweep": "transfer", "config": cfg, "dense_fp32_MiB": round(dense_bytes / 2 ** 20, 1),
               "dense_us": round(t_dense, 1), "dense_GBps": round(dense_bytes / t_dense / 1e3, 1),
               "packed_MiB": round(pk.nbytes / 2 ** 20, 1), "packed_copy_us": round(t_low, 1),
               "packed_GBps": round(pk.nbytes / t_low / 1e3, 1), "host_pack_us_16_threads": round(t_pack, 1)}
        print(json.dumps(rec), flush=True)
        rows.append(rec)
        del a_f32, x_pin, da, dx, pk
        torch.cuda.empty_cache()
    print("\n| config | dense fp32 A + X, two copies | packed A + X, one copy | host packing (16 threads) |")
    print("|---|---|---|---|")
    for r in rows:
        print(f"| {r['config']} | {r['dense_fp32_MiB']} MiB, {r['dense_us']} us ({r['dense_GBps']} GB/s) | "
              f"{r['packed_MiB']} MiB, {r['packed_copy_us']} us ({r['packed_GBps']} GB/s) | "
              f"{r['host_pack_us_16_threads']} us |")


def _kernel_us(fn, kind, n=10, warm=3):
    """Mean GPU time per launch, from the library's events around each launch."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    q.qgtc_prof_enable(True)
    q.qgtc_prof_reset()
    for _ in range(n):
        fn()
    torch.cuda.synchronize()
    ms, launches = q.qgtc_prof_read(kind)
    q.qgtc_prof_enable(False)
    q.qgtc_prof_reset()
    return ms * 1e3 / max(launches, 1)


GATE_SHAPES = ((65536, 64, 64), (65536, 128, 64), (262144, 512, 16))


def gate():
    """Each case: 3 warm-up and 10 timed launches of one kernel, in the order printed."""
    gen = torch.Generator(device="cuda").manual_seed(12)
    rows = []
    for (n, d, h) in GATE_SHAPES:
        for s in range(1, 9):
            yq = torch.randint(0, 2 ** s, (n, d), device="cuda", dtype=torch.int32, generator=gen)
            wq = torch.randint(0, 2 ** s, (d, h), device="cuda", dtype=torch.int32, generator=gen)
            yb = q.qgtc_pack_bits(yq, s, q.LEFT, out=q.alloc_bits(n, d, s, q.LEFT, ld_words=-(-d // 32)))
            wb = q.qgtc_pack_bits(wq, s, q.RIGHT)
            out_i = torch.empty((n, h), dtype=torch.int32, device="cuda")
            out_b = q.alloc_bits(n, h, s, q.RIGHT)
            rec = {"sweep": "gate", "N": n, "D": d, "H": h, "bits": s}
            for path, name in ((q.UPDATE_POPCOUNT, "popcount"), (q.UPDATE_MATRIX_CORES, "mfma")):
                tn = q.Tuning(update_path=path)
                ep_i = q.Epilogue(mode=q.OUT_I32, tuning=tn)
                ep_b = q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=s, rq_lo=0, rq_inv_scale=1e-3, tuning=tn)
                t_i = _kernel_us(lambda: q.qgtc_update(yb, wb, ep_i, out=out_i), q.KERNEL_UPDATE)
                t_b = _kernel_us(lambda: q.qgtc_update(yb, wb, ep_b, out=out_b), q.KERNEL_UPDATE)
                rec[f"us_{name}_int32"] = round(t_i, 1)
                rec[f"us_{name}_bits"] = round(t_b, 1)
                # bytes: the planes of Y once, W, and the output
                rec[f"gbps_{name}_int32"] = round((n * d * s / 8 + d * h * s / 8 + n * h * 4) / t_i / 1e3, 1)
                rec[f"gbps_{name}_bits"] = round((n * d * s / 8 + d * h * s / 8 + n * h * s / 8) / t_b / 1e3, 1)
            print(json.dumps(rec), flush=True)
            rows.append(rec)
            del yq, yb, out_i, out_b
        torch.cuda.empty_cache()
    print("\nupdate Y.W, s = t, popcount kernel against int8 matrix cores; us per launch (achieved GB/s of "
          "algorithmic bytes):")
    print("\n| N x D -> H | bits | popcount, int32 out | matrix cores, int32 out | popcount, low-bit out | "
          "matrix cores, low-bit out |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['N']} x {r['D']} -> {r['H']} | {r['bits']} | "
              f"{r['us_popcount_int32']} ({r['gbps_popcount_int32']}) | {r['us_mfma_int32']} ({r['gbps_mfma_int32']}) | "
              f"{r['us_popcount_bits']} ({r['gbps_popcount_bits']}) | {r['us_mfma_bits']} ({r['gbps_mfma_bits']}) |")


def streaming():
    """Each kernel alone on the device (in a forward pass the packing of A and of X overlap on
    two streams and share the bandwidth)."""
    gen = torch.Generator(device="cuda").manual_seed(14)
    rows = []

    def case(name, fn, nbytes, kind):
        t = _kernel_us(fn, kind, n=10, warm=3)
        rec = {"sweep": "streaming", "kernel": name, "us": round(t, 1), "MiB": round(nbytes / 2 ** 20, 1),
               "TBps": round(nbytes / t / 1e6, 2), "frac_of_8TBps": round(nbytes / t / 8e6, 2)}
        print(json.dumps(rec), flush=True)
        rows.append(rec)

    for (cfg, n, blk, d, h) in ((4, 65536, 1024, 128, 64), (5, 262144, 2048, 512, 16)):
        a8 = (torch.rand((n, blk), device="cuda", generator=gen) < 0.006).to(torch.uint8)
        ab = q.alloc_bits(n, blk, 1, q.LEFT, blk)
        case(f"config {cfg}: pack A, uint8 {n} x {blk} -> 1 bit", lambda: q.qgtc_pack_bits(a8, 1, q.LEFT, out=ab),
             n * blk * (1 + 1 / 8), q.KERNEL_PACK)
        del a8
        for kb in (128, 32):
            m = q.qgtc_build_tile_map(ab, 16, kb)
            case(f"config {cfg}: zero-tile map 16 x {kb} (list, total and run length, degrees)",
                 lambda: q.qgtc_build_tile_map(ab, 16, kb, out=m), n * blk / 8, q.KERNEL_TILE_MAP)
        cnt = q.qgtc_tile_stats(ab)
        case(f"config {cfg}: tile statistics at three widths", lambda: q.qgtc_tile_stats(ab, out=cnt), n * blk / 8,
             q.KERNEL_TILE_MAP)
        x = torch.randn((n, d), device="cuda", generator=gen)
        xr = (float(x.min()), float(x.max()))
        for s in (8, 4, 1):
            xb = q.alloc_bits(n, d, s, q.RIGHT)
            case(f"config {cfg}: pack X, fp32 {n} x {d} -> {s} planes", lambda: q.qgtc_pack_bits(x, s, q.RIGHT, quant=xr, out=xb),
                 n * d * (4 + s / 8), q.KERNEL_PACK)
        xl = q.alloc_bits(n, d, 8, q.LEFT_BYTES)
        case(f"config {cfg}: pack X, fp32 {n} x {d} -> bytes", lambda: q.qgtc_pack_bits(x, 8, q.LEFT_BYTES, quant=xr, out=xl),
             n * d * 5, q.KERNEL_PACK)
        del x
        for s in (8, 7, 4):
            yq = torch.randint(0, 2 ** s, (n, d), device="cuda", dtype=torch.int32, generator=gen)
            wq = torch.randint(0, 2 ** s, (d, h), device="cuda", dtype=torch.int32, generator=gen)
            yb = q.qgtc_pack_bits(yq, s, q.LEFT, out=q.alloc_bits(n, d, s, q.LEFT, ld_words=-(-d // 32)))
            yl = q.qgtc_pack_bits(yq, s, q.LEFT_BYTES)
            wb = q.qgtc_pack_bits(wq, s, q.RIGHT)
            ob = q.alloc_bits(n, h, s, q.RIGHT)
            oi = torch.empty((n, h), dtype=torch.int32, device="cuda")
            ep_b = q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=s, rq_lo=0, rq_inv_scale=1e-3)
            case(f"config {cfg}: update {n} x {d} -> {h}, {s}-bit planes, int32 out",
                 lambda: q.qgtc_update(yb, wb, q.Epilogue(mode=q.OUT_I32), out=oi), n * d * s / 8 + n * h * 4, q.KERNEL_UPDATE)
            case(f"config {cfg}: update {n} x {d} -> {h}, {s}-bit planes, low-bit out",
                 lambda: q.qgtc_update(yb, wb, ep_b, out=ob), n * d * s / 8 + n * h * s / 8, q.KERNEL_UPDATE)
            case(f"config {cfg}: update {n} x {d} -> {h}, {s}-bit codes as bytes, low-bit out",
                 lambda: q.qgtc_update(yl, wb, ep_b, out=ob), n * d + n * h * s / 8, q.KERNEL_UPDATE)
            del yq, yb, yl, ob, oi
        del ab
        torch.cuda.empty_cache()
    print("\n| kernel (alone on the device) | us | algorithmic MiB | TB/s | fraction of 8 TB/s |")
    print("|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['kernel']} | {r['us']} | {r['MiB']} | {r['TBps']} | {r['frac_of_8TBps']} |")


def tiles():
    """One fused layer (8 bits, first layer's shape) per tile width: time per visited adjacency bit."""
    from workloads import make_workload
    rows = []
    for cfg in (4, 5):
        w = make_workload(cfg)
        g = w.graph
        a_src = torch.from_numpy(g.dense_compact()).cuda()
        ws = [torch.from_numpy(W).cuda() for W in w.W]
        x = torch.from_numpy(w.X).cuda()
        xr = (float(w.X.min()), float(w.X.max()))
        base = None
        for kb in (128, 64, 32):
            net = QuantGNN(a_src, ws, w.s, w.t, w.model == "gin", tile_kbits=kb, block_rows=g.block)
            ranges = net.calibrate(x, xr)
            out = torch.empty((g.n_nodes, net.dims[-1][1]), dtype=torch.float32, device="cuda")
            t = _kernel_us(lambda: net.forward(x, xr, ranges, out=out), q.KERNEL_LAYER, n=5, warm=2) * len(net.dims)
            nnz = int(net.map.nnz_tiles.cpu()[0])
            per_bit = t / (nnz * 16.0 * kb)
            base = base or per_bit
            rec = {"sweep": "tiles", "config": cfg, "tile_kbits": kb, "nonzero_tiles": nnz,
                   "us_layers": round(t, 1), "ps_per_adjacency_bit": round(per_bit * 1e6, 3),
                   "cost_relative_to_128": round(per_bit / base, 2)}
            print(json.dumps(rec), flush=True)
            rows.append(rec)
            del net, out
        del a_src, x
        torch.cuda.empty_cache()
    print("\n| config | tile | non-zero tiles | all layers us | cost per visited adjacency bit, relative to 16 x 128 |")
    print("|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['config']} | 16 x {r['tile_kbits']} | {r['nonzero_tiles']} | {r['us_layers']} | {r['cost_relative_to_128']} |")


def zero_words():
    """The aggregation with every word of the kept tiles visited against zero-word jumping,
    over the share of (row, word) pairs that hold a bit: the measurement behind the
    selector's 70 % rule.  N = 16384 nodes in 16 diagonal blocks of 1024, D = 64, int32 out."""
    gen = torch.Generator(device="cuda").manual_seed(16)
    n, blk, d = 16384, 1024, 64
    rows = []
    for p_edge in (0.002, 0.008, 0.02, 0.04, 0.07, 0.12, 0.3):
        a = (torch.rand((n, blk), device="cuda", generator=gen) < p_edge).to(torch.uint8)
        ab = q.qgtc_pack_bits(a, 1, q.LEFT, block_rows=blk)
        tmap = q.qgtc_build_tile_map(ab, 16, 128)
        st = q.tile_stats_numbers(q.qgtc_tile_stats(ab))
        share = st["nnz_row_words"] / (16.0 * st["nnz_tiles"][2] * 4)
        for s_bits in (3, 4, 8):
            x = torch.randint(0, 2 ** s_bits, (n, d), dtype=torch.int32, device="cuda", generator=gen)
            xb = q.qgtc_pack_bits(x, s_bits, q.RIGHT)
            out = torch.empty((n, d), dtype=torch.int32, device="cuda")
            t = {}
            for name, zw in (("visit", q.ZERO_WORDS_VISIT), ("jump", q.ZERO_WORDS_SKIP)):
                ep = q.Epilogue(mode=q.OUT_I32, tuning=q.Tuning(zero_words=zw))
                t[name] = _kernel_us(lambda: q.qgtc_aggregate(ab, tmap, xb, ep, out=out), q.KERNEL_AGGREGATE, n=10, warm=3)
            plan = q.qgtc_plan_layer(n, d, d, s_bits, 8, n_tile_rows=st["n_tile_rows"], a_cols=blk,
                                     nnz_tiles=st["nnz_tiles"], nnz_row_words=st["nnz_row_words"])
            rec = {"sweep": "zero_words", "p_edge": p_edge, "pairs_present": round(share, 3), "bits": s_bits,
                   "us_visit_all": round(t["visit"], 1), "us_jump": round(t["jump"], 1),
                   "selector": "jump" if plan["zero_words"] == q.ZERO_WORDS_SKIP else "visit all"}
            print(json.dumps(rec), flush=True)
            rows.append(rec)
            del x, xb, out
        del a, ab, tmap
        torch.cuda.empty_cache()
    print("\n| edge probability | (row, word) pairs present in kept tiles | bits | visit all us | jump us | selector |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['p_edge']} | {r['pairs_present']} | {r['bits']} | {r['us_visit_all']} | {r['us_jump']} | {r['selector']} |")


def main():
    torch.cuda.set_device(0)
    which = sys.argv[1:] or ["table3", "config3", "config5", "sizes", "reuse", "transfer", "gate", "streaming", "tiles", "zero_words"]
    for name in which:
        {"table3": table3, "config3": config3, "config5": config5, "sizes": sizes, "reuse": reuse,
         "transfer": transfer, "gate": gate, "streaming": streaming, "tiles": tiles,
         "zero_words": zero_words}[name]()


if __name__ == "__main__":
    main()
