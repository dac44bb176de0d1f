"""qgtc_layer_static (the layer for callers that cannot allocate device memory: its
workspace is a static device array of the library) against qgtc_layer with a
caller-supplied workspace, through the C ABI, on two calls in a row, the second
with a smaller input: bit-exact integers and packed words, identical fp32 bits.
Both layer paths use the array: the fused kernel keeps the re-ordered weights in
it, the two-kernel path the packed planes of Y and their row sums."""
import numpy as np
import pytest
import torch

from oracle import qgnn

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2111_09547_amd")
from gpu_util import dev, as_u32, pack_adjacency  # noqa: E402


def _case(rng, n, d, h, s, t):
    A = (rng.random((n, n)) < 0.05).astype(np.uint8)
    Xq = rng.integers(0, 2 ** min(s, 31), size=(n, d)).astype(np.uint32)
    Wq = rng.integers(0, 2 ** min(t, 31), size=(d, h)).astype(np.uint32)
    return A, Xq, Wq


def _check_case(n, d, h, s, t, seed):
    rng = np.random.default_rng([77, seed, n, d, h, s, t])
    A, Xq, Wq = _case(rng, n, d, h, s, t)
    Y = qgnn.aggregate(A, Xq)
    rq_inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Y).max())), s)
    Z = qgnn.update(qgnn.requantize(Y, 0, rq_inv, s), Wq)

    Ab = pack_adjacency(A)
    m = q.qgtc_build_tile_map(Ab, 16, 128)
    Xb = q.qgtc_pack_bits(dev(Xq.view(np.int32)), s, q.RIGHT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=s, rq_lo=0, rq_inv_scale=float(rq_inv))
    rl = dev(rng.integers(1, 30, size=n).astype(np.int32))
    cs = q.qgtc_col_sums(Wb)
    out_bits = min(s, 6)
    z_inv = float(qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Z).max())), out_bits))
    eps = [q.Epilogue(mode=q.OUT_I32),
           q.Epilogue(mode=q.OUT_F32, cc=1.7e-3, rs=-0.031, l0a=0.4, l0b=-0.9, ck=-6.4, cs=0.0125,
                      row_i=None, row_l=rl, col_i=cs),
           q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=out_bits, rq_lo=3, rq_inv_scale=z_inv)]
    for ep in eps:
        if ep.mode == q.OUT_BITS:
            want, got = q.alloc_bits(n, h, out_bits, q.RIGHT), q.alloc_bits(n, h, out_bits, q.RIGHT)
            want.words.fill_(-1)
            got.words.fill_(-1)
        else:
            dt = torch.int32 if ep.mode == q.OUT_I32 else torch.float32
            want = torch.full((n, h), -7, dtype=dt, device="cuda")
            got = torch.full((n, h), -7, dtype=dt, device="cuda")
        q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, ep, out=want)
        q.qgtc_layer_static(Ab, m, Xb, Wb, agg_ep, ep, out=got)
        torch.cuda.synchronize()
        if ep.mode == q.OUT_BITS:
            assert torch.equal(got.words, want.words), (n, d, h, s, t, "bits")
        else:
            # fp32: the two calls run the same kernels on the same integers - same bits
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (n, d, h, s, t, ep.mode)
        if ep.mode == q.OUT_I32:
            assert (as_u32(got) == Z).all()          # and the oracle's integers


@pytest.mark.parametrize("bits", [8, 16])
def test_layer_static_matches_layer_on_two_calls_in_a_row(bits):
    """8 bits: the fused kernel (scratch = weights in operand order); 16 bits: aggregate +
    update (scratch = packed planes of Y and row sums).  The second call is smaller, so it
    finds the first call's contents in the array."""
    _check_case(530, 200, 72, bits, bits, 0)
    _check_case(130, 40, 16, bits, bits, 1)


def test_layer_static_rejects_what_does_not_fit():
    """Beyond the static array's size the call fails before anything is launched."""
    n, d = 70000, 2048                                   # 16-bit planes of Y: 70000 * 64 * 16 * 4 B > 16 MiB
    assert q.lib().qgtc_layer_workspace_bytes(n, d, 16, 16) > q.LAYER_STATIC_MAX_BYTES
    Ab = q.alloc_bits(n, 128, 1, q.LEFT, block_rows=128)
    Xb = q.alloc_bits(n, d, 16, q.RIGHT)
    Wb = q.alloc_bits(d, 16, 16, q.RIGHT)
    agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=16, rq_lo=0, rq_inv_scale=1.0)
    out = torch.empty((n, 16), dtype=torch.int32, device="cuda")
    with pytest.raises(q.QgtcError) as e:
        q.qgtc_layer_static(Ab, None, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32), out=out)
    assert e.value.status == 6                           # QGTC_ERR_WORKSPACE
