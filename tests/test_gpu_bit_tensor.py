"""The paper's PyTorch-level names (Section 5) against the oracle: to_bit / to_val round
trip and Eq. (2), bitMM2Int and bitMM2Bit for a binary and for a multi-bit left operand."""
import numpy as np
import pytest
import torch

from oracle import qgnn, bitplane as bp

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2111_09547_amd")
from paper_2111_09547_amd.bit_tensor import to_bit, to_val, bitMM2Int, bitMM2Bit  # noqa: E402
from gpu_util import dev, as_u32, words_np  # noqa: E402


@pytest.mark.parametrize("bits", [1, 3, 8, 13])
def test_to_bit_and_back(bits):
    rng = np.random.default_rng([71, bits])
    v = rng.integers(0, 2 ** bits, size=(77, 45)).astype(np.int32)
    for side in ("left", "right"):
        assert (to_val(to_bit(dev(v), bits, side=side)).cpu().numpy() == v).all()
    x = rng.normal(size=(60, 33)).astype(np.float32)
    got = to_val(to_bit(dev(x), bits)).cpu().numpy()                 # min-max by default
    assert (got.view(np.uint32) == qgnn.quantize(x, float(x.min()), float(x.max()), bits)).all()
    got = to_val(to_bit(dev(x), bits, quant=(-1.0, 2.5))).cpu().numpy()
    assert (got.view(np.uint32) == qgnn.quantize(x, -1.0, 2.5, bits)).all()


@pytest.mark.parametrize("sa,sb", [(1, 4), (1, 8), (3, 5), (8, 8), (2, 11)])
def test_bit_products(sa, sb):
    rng = np.random.default_rng([72, sa, sb])
    m, k, n = 150, 96, 40
    L = rng.integers(0, 2 ** sa, size=(m, k)).astype(np.uint32)
    R = rng.integers(0, 2 ** sb, size=(k, n)).astype(np.uint32)
    Lb = to_bit(dev(L.view(np.int32)), sa, side="left")
    Rb = to_bit(dev(R.view(np.int32)), sb, side="right")
    C = qgnn.matmul_mod32(L, R)
    assert (as_u32(bitMM2Int(Lb, Rb)) == C).all()
    bit_c = 5
    inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(C).max())), bit_c)
    want = qgnn.requantize(C, 0, inv, bit_c)
    layout = bp.LEFT if sa == 1 else bp.RIGHT        # next left operand after an aggregation, next X after an update
    for got in (bitMM2Bit(Lb, Rb, bit_c, inv_scale=float(inv)), bitMM2Bit(Lb, Rb, bit_c)):
        assert got.nbits == bit_c
        assert (words_np(got) == bp.pack(want, bit_c, layout)).all()
        assert (to_val(got).cpu().numpy().view(np.uint32) == want).all()
