"""GPU parity of whole models (configs 4 and 5) against the CPU oracle:
layer by layer with the oracle fed the same integers ("teacher forced") and end
to end, at reduced and at full size."""
import numpy as np
import pytest
import torch

from oracle import qgnn
from workloads import make_workload

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2111_09547_amd")
from paper_2111_09547_amd.model import QuantGNN, LayerRanges  # noqa: E402
from gpu_util import dev, as_u32, pack_adjacency, assert_fp32_close  # noqa: E402


def run_model(w, tile_kbits=128):
    """Runs the HIP path with ranges calibrated by the HIP path itself and
    checks every layer against the oracle fed the same ranges."""
    g = w.graph
    Ws = [dev(W) for W in w.W]
    self_term = w.model == "gin"
    if w.storage == "dense":
        net = QuantGNN(dev(g.dense()), Ws, w.s, w.t, self_term, tile_kbits=tile_kbits)
    else:
        net = QuantGNN(dev(g.dense_compact()), Ws, w.s, w.t, self_term, tile_kbits=tile_kbits,
                       block_rows=g.block)
    X = dev(w.X)
    xr = (float(w.X.min()), float(w.X.max()))
    ranges = net.calibrate(X, xr)

    # the oracle, given the same user-set ranges
    A = g.scipy_csr()
    wr = [(float(W.min()), float(W.max())) for W in w.W]
    rqs = []
    for r in ranges:
        agg = (0, qgnn.inv_scale(0.0, float(r.agg_hi), w.s))
        out = None if r.out_hi is None else (0, qgnn.inv_scale(0.0, float(r.out_hi), w.s))
        rqs.append((agg, out))
    trace, _ = qgnn.forward(A, w.X, xr, w.W, wr, w.s, w.t, self_term, rqs=rqs)
    # the calibration the HIP path made equals what the oracle would calibrate
    for r, tr in zip(ranges, trace):
        assert r.agg_hi == max(1, int(qgnn.as_signed(tr["Y"]).max()))

    # end to end: last int32 accumulators and the fp32 output
    z = net.forward(X, xr, ranges, want_int=True)
    assert (as_u32(z) == trace[-1]["Z"]).all()
    out = net.forward(X, xr, ranges)
    torch.cuda.synchronize()

    # the oracle's fp32 output for the same user-set ranges
    ref, _, _ = qgnn.forward_dequantized(A, w.X, xr, w.W, wr, w.s, w.t, self_term, rqs=rqs)
    assert_fp32_close(out.cpu().numpy(), ref, f"config {w.cfg} s={w.s} end to end")

    # independent runs of subgraphs on several streams give the same bytes
    if w.storage == "compact":
        nb = w.graph.n_blocks
        assert net.auto_runs() in (1, 2)                           # the selector's own choice
        for k in ("auto", 2, 3, [nb - nb // 4, nb // 4], [1, nb - 1]):     # equal and uneven runs
            if isinstance(k, list) and min(k) < 1:
                continue
            again = net.forward(X, xr, ranges, streams=k)
            torch.cuda.synchronize()
            assert torch.equal(again, out), k
            zk = net.forward(X, xr, ranges, want_int=True, streams=k)
            torch.cuda.synchronize()
            assert (as_u32(zk) == trace[-1]["Z"]).all(), k

    # the same pass recorded as a HIP graph: every replay, with eager work of the program
    # in between, gives the eager result again
    buf = torch.empty_like(out)
    for k in ((1, 2) if w.storage == "compact" else (1,)):
        graph = net.capture(X, xr, ranges, buf, streams=k, with_static=True)
        for rep in range(3):
            buf.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(buf, out), (k, rep)
            eager = net.forward(X, xr, ranges)          # eager launches between the replays
            torch.cuda.synchronize()
            assert torch.equal(eager, out), (k, rep)
        del graph

    # layer by layer, teacher forced: feed the oracle's integers to each HIP layer
    for l, tr in enumerate(trace):
        xb = q.qgtc_pack_bits(dev(tr["Xq"].view(np.int32)), w.s, q.RIGHT)
        ep = q.Epilogue(mode=q.OUT_I32, self_term=self_term)
        y32 = q.qgtc_aggregate(net.A, net.map, xb, ep)
        assert (as_u32(y32) == tr["Y"]).all(), l
        zz = q.qgtc_layer(net.A, net.map, xb, net.W[l], net._agg_ep(ranges[l].agg_hi),
                          q.Epilogue(mode=q.OUT_I32))
        assert (as_u32(zz) == tr["Z"]).all(), l
    return net, ranges


@pytest.mark.parametrize("cfg,bits,nb", [(5, 8, 4), (5, 4, 4), (4, 8, 2), (5, 8, None), (5, 4, None), (5, 2, None),
                                         (5, 1, None), (4, 8, None)])
def test_update_first_order(cfg, bits, nb):
    """A.(X.W) per layer (qgtc_update, then qgtc_aggregate): calibrated ranges, the last
    int32 accumulators and the scale-only fp32 output against the oracle run in the same
    order with the same ranges."""
    w = make_workload(cfg, bits=bits, n_blocks=nb)
    g = w.graph
    self_term = w.model == "gin"
    net = QuantGNN(dev(g.dense_compact()), [dev(W) for W in w.W], w.s, w.t, self_term,
                   block_rows=g.block, update_first=True)
    X = dev(w.X)
    xr = (float(w.X.min()), float(w.X.max()))
    wr = [(float(W.min()), float(W.max())) for W in w.W]
    ranges = net.calibrate(X, xr)
    rqs = [((0, qgnn.inv_scale(0.0, float(r.agg_hi), w.s)),
            None if r.out_hi is None else (0, qgnn.inv_scale(0.0, float(r.out_hi), w.s))) for r in ranges]
    ref, trace, _ = qgnn.forward_dequantized(g.scipy_csr(), w.X, xr, w.W, wr, w.s, w.t, self_term, rqs=rqs,
                                             update_first=True)
    for r, tr in zip(ranges, trace):
        assert r.agg_hi == max(1, int(qgnn.as_signed(tr["Y"]).max()))
    z = net.forward(X, xr, ranges, want_int=True)
    assert (as_u32(z) == trace[-1]["Z"]).all()
    out = net.forward(X, xr, ranges).cpu().numpy()
    assert_fp32_close(out, ref, f"config {cfg} s={bits} update first")


@pytest.mark.parametrize("nb", [2, None])
def test_config4_gin_five_layers(nb):
    w = make_workload(4, n_blocks=nb)
    run_model(w)


def test_selector_runs_on_the_bench_configurations():
    """The full-size batches as bench.py issues them: config 4 on 128-bit tiles as one run
    (with zero-word jumping four of its five launches are exactly one round of the wave
    slots) and as two runs when every word is visited (1.33 rounds); config 5 (long launches,
    hubs first) as one run on 64-bit tiles (32-bit tiles at 2 bits, where every word of a kept
    tile is visited and the width with the fewest kept bits wins)."""
    from paper_2111_09547_amd.model import QuantGNN, choose_tile_kbits
    for cfg, want, kb in ((4, 1, 128), (5, 1, 64)):
        w = make_workload(cfg)
        g = w.graph
        net = QuantGNN(dev(g.dense_compact()), [dev(W) for W in w.W], w.s, w.t, w.model == "gin",
                       block_rows=g.block, tile_kbits="auto")
        assert net.auto_runs() == want, cfg
        assert net.tile_kbits == kb, cfg
        if cfg == 5:
            assert choose_tile_kbits(net.A, 512, 16, 2, 2) == 32
        else:
            visit = QuantGNN(net.A, [dev(W) for W in w.W], w.s, w.t, True, block_rows=g.block, tile_kbits="auto",
                             tuning=q.Tuning(zero_words=q.ZERO_WORDS_VISIT))
            assert visit.tuning.zero_words == q.ZERO_WORDS_VISIT and visit.auto_runs() == 2
            del visit
        del net
        torch.cuda.empty_cache()


@pytest.mark.parametrize("bits,nb,kb", [(1, 4, 128), (2, 4, 64), (4, 4, 32), (8, 4, 128), (8, None, 128), (4, None, 32),
                                        (8, None, "auto"),
                                        (1, None, 128), (2, None, 128), (2, None, 32), (1, None, 32)])
def test_config5_gcn_two_layers(bits, nb, kb):
    w = make_workload(5, bits=bits, n_blocks=nb)
    run_model(w, tile_kbits=kb)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 6, 7, 8, 16, 32])
def test_config3_full_size_bit_sweep(bits):
    w = make_workload(3, bits=bits)
    A = w.graph.scipy_csr()
    xr = (float(w.X.min()), float(w.X.max()))
    wr = (float(w.W[0].min()), float(w.W[0].max()))
    Xq = qgnn.quantize(w.X, xr[0], xr[1], w.s)
    Wq = qgnn.quantize(w.W[0], wr[0], wr[1], w.t)
    Y, Yq, Z, (rq_lo, rq_inv) = qgnn.layer(A, Xq, Wq, w.s)
    Ab = pack_adjacency(w.graph, "dense")
    m = q.qgtc_build_tile_map(Ab)
    Xb = q.qgtc_pack_bits(dev(w.X), w.s, q.RIGHT, quant=xr)
    Wb = q.qgtc_pack_bits(dev(w.W[0]), w.t, q.RIGHT, quant=wr)
    agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=w.s, rq_lo=rq_lo, rq_inv_scale=float(rq_inv))
    got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32))
    assert (as_u32(got) == Z).all()
    # the tile map keeps exactly the diagonal blocks (8 blocks of 1024: 8 of 64 tile columns)
    assert int(m.nnz_tiles.cpu()[0]) == 512 * 8


@pytest.mark.parametrize("cfg,nb,last_bn", [(4, 2, False), (4, 4, True), (5, 4, False)])
def test_batchnorm_folded_into_the_layers(cfg, nb, last_bn):
    """A batch normalization after every hidden layer (Section 4.5), folded into the layer
    kernel's output epilogue: the last accumulators, bit for bit, and the fp32 output
    against the oracle given the same ranges and its own fold of the same parameters."""
    from paper_2111_09547_amd.model import BatchNorm
    w = make_workload(cfg, n_blocks=nb)
    g = w.graph
    self_term = w.model == "gin"
    rng = np.random.default_rng([31, cfg, nb])
    n_layers = len(w.W)
    params = []
    for l, W in enumerate(w.W):
        h = W.shape[1]
        if l == n_layers - 1 and not last_bn:
            params.append(None)
            continue
        params.append(dict(gamma=rng.uniform(0.5, 1.5, size=h), beta=rng.uniform(-0.3, 0.6, size=h),
                           mean=rng.uniform(-0.2, 0.4, size=h) * (l + 1) * 0.05,
                           var=rng.uniform(0.5, 2.0, size=h) * 0.02, eps=1e-5))
    bns = [None if p is None else BatchNorm(**p) for p in params]
    net = QuantGNN(dev(g.dense_compact()), [dev(W) for W in w.W], w.s, w.t, self_term,
                   block_rows=g.block, batchnorm=bns)
    X = dev(w.X)
    xr = (float(w.X.min()), float(w.X.max()))
    wr = [(float(W.min()), float(W.max())) for W in w.W]
    ranges = net.calibrate(X, xr)

    # the oracle's side: the same user-set ranges and the same batch-normalization parameters;
    # it folds them itself, with the real value of one accumulator unit of each layer
    rqs = [((0, qgnn.inv_scale(0.0, float(r.agg_hi), w.s)),
            None if r.out_hi is None else (0, qgnn.inv_scale(0.0, float(r.out_hi), w.s))) for r in ranges]
    ref, trace, _ = qgnn.forward_dequantized(g.scipy_csr(), w.X, xr, w.W, wr, w.s, w.t, self_term, rqs=rqs,
                                             batchnorms=params)
    for l, (r, tr) in enumerate(zip(ranges, trace)):
        assert r.agg_hi == max(1, int(qgnn.as_signed(tr["Y"]).max())), l
        if l < n_layers - 1:                      # the range the HIP path calibrated is the oracle's
            ca, cb = tr["affine"]
            assert float(qgnn.calibrate_requant_affine(tr["Z"], ca, cb, w.s)[1]) == float(rqs[l][1][1]), l
            assert tr["Xq_next"].max() == 2 ** w.s - 1

    z = net.forward(X, xr, ranges, want_int=True)
    assert (as_u32(z) == trace[-1]["Z"]).all()
    out = net.forward(X, xr, ranges).cpu().numpy()
    assert_fp32_close(out, ref, f"config {cfg} with batch normalization")
    # the recorded pass gives the same bytes
    buf = torch.empty_like(net.forward(X, xr, ranges))
    graph = net.capture(X, xr, ranges, buf, with_static=True)
    for _ in range(2):
        buf.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(buf.cpu().numpy(), out)


@pytest.mark.parametrize("cfg,nb", [(4, 2), (5, 4)])
def test_host_packed_batch_in_one_transfer(cfg, nb):
    """Section 4.6: adjacency and features packed on the host into one pinned buffer and
    copied once give the words the device packing gives, and the same model output."""
    from paper_2111_09547_amd.packing import SubgraphPacket
    from gpu_util import words_np
    w = make_workload(cfg, n_blocks=nb)
    g = w.graph
    self_term = w.model == "gin"
    a_host = torch.from_numpy(g.dense_compact())
    x_host = torch.from_numpy(w.X)
    xr = (float(w.X.min()), float(w.X.max()))
    pk = SubgraphPacket(g.n_nodes, g.block, w.X.shape[1], w.s, block_rows=g.block)
    pk.pack(a_host, x_host, xr)
    a_bits, x_bits = pk.upload()
    ref_a = q.qgtc_pack_bits(a_host.cuda(), 1, q.LEFT, block_rows=g.block)
    ref_x = q.qgtc_pack_bits(x_host.cuda(), w.s, q.RIGHT, quant=xr)
    torch.cuda.synchronize()
    assert (words_np(a_bits) == words_np(ref_a)).all()
    assert (words_np(x_bits) == words_np(ref_x)).all()

    Ws = [dev(W) for W in w.W]
    ref_net = QuantGNN(dev(g.dense_compact()), Ws, w.s, w.t, self_term, block_rows=g.block)
    ranges = ref_net.calibrate(dev(w.X), xr)
    want = ref_net.forward(dev(w.X), xr, ranges)
    net = QuantGNN(a_bits, Ws, w.s, w.t, self_term, block_rows=g.block)      # the packed adjacency as it is
    got = net.forward(None, xr, ranges, x_bits=x_bits)
    torch.cuda.synchronize()
    assert torch.equal(got, want)


def test_tile_width_is_chosen_from_the_zero_tile_maps():
    """tile_kbits="auto": dense subgraphs keep 128-bit tiles; so do the first eight subgraphs of
    the power-law graph (its hubs) at 8 bits, where the kernels jump over zero words and a
    tile's own cost counts, while at 2 bits, where every word of a kept tile is visited, the
    gaps inside the subgraphs make 32-bit tiles the least work; the output does not depend on
    the choice."""
    from paper_2111_09547_amd.model import choose_tile_kbits
    for cfg, nb, want in ((4, 2, 128), (5, 8, 128)):
        w = make_workload(cfg, n_blocks=nb)
        g = w.graph
        Ws = [dev(W) for W in w.W]
        auto = QuantGNN(dev(g.dense_compact()), Ws, w.s, w.t, w.model == "gin", tile_kbits="auto",
                        block_rows=g.block)
        assert auto.tile_kbits == want == choose_tile_kbits(auto.A)
        if cfg == 5:
            assert choose_tile_kbits(auto.A, s=2, t=2) == 32
        assert auto.map.c.tile_kbits == want
        ref = QuantGNN(dev(g.dense_compact()), Ws, w.s, w.t, w.model == "gin", tile_kbits=128,
                       block_rows=g.block)
        X = dev(w.X)
        xr = (float(w.X.min()), float(w.X.max()))
        ranges = ref.calibrate(X, xr)
        assert torch.equal(auto.forward(X, xr, ranges), ref.forward(X, xr, ranges))
