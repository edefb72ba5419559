"""Parity of the binary convolution with max-pooling (and the optional ReLU) in its epilogue (block order
BinConv -> Pool, sec. 3.2) with the CPU oracle: max_pool of the oracle's block output.  The pooled value is
one of the convolution outputs, so the tolerance is the convolution's (1e-5 relative, 1e-6 absolute); it
must also equal, bit for bit, the maximum over the GPU's own unpooled output."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import workloads as wl
from paper_1603_05279_amd import xnor
from tests.helpers import to_dev

pytestmark = pytest.mark.gpu

# n, c, h, w, k_out, kh, kw, stride, pad, pool, pstride, relu, give_K
CASES = [
    (3, 40, 27, 27, 70, 5, 5, (1, 1), (2, 2), (3, 3), (2, 2), False, False),     # AlexNet conv2 geometry
    (4, 64, 13, 13, 256, 3, 3, (1, 1), (1, 1), (3, 3), (2, 2), False, True),     # AlexNet conv5 geometry
    (2, 33, 14, 14, 300, 3, 3, (1, 1), (1, 1), (2, 2), (2, 2), True, False),     # two filter tiles, ReLU
    (2, 16, 9, 20, 31, 3, 3, (1, 1), (0, 0), (2, 3), (1, 2), False, True),       # 7 x 18 output, non-square window
    (1, 8, 31, 31, 5, 3, 3, (2, 2), (1, 1), (3, 3), (3, 3), True, False),        # strided convolution, 16 x 16 output
    (5, 100, 7, 7, 200, 3, 3, (1, 1), (1, 1), (7, 7), (1, 1), False, False),     # global pooling
    (2, 20, 6, 64, 40, 1, 1, (1, 1), (0, 0), (2, 2), (2, 2), False, True),       # 64-wide rows: 3 rows per 192-pixel tile
    (1, 3, 5, 5, 2, 3, 3, (1, 1), (1, 1), (1, 1), (1, 1), False, False),         # 1 x 1 window: the convolution itself
]


def run(x, W, stride, pad, pool, pstride, relu, give_K):
    n, c, h, w = x.shape
    k, _, kh, kw = W.shape
    desc = xnor.make_desc(n, c, h, w, k, kh, kw, stride, pad)
    ho, wo = xnor.output_hw(desc)
    hpo, wpo = (ho - pool[0]) // pstride[0] + 1, (wo - pool[1]) // pstride[1] + 1
    pw = xnor.PackedWeights(to_dev(W))
    bufs = xnor.ConvBuffers(desc)
    xnor.xnor_binactiv(to_dev(x), None, None, bufs.xbits, bufs.A, bufs.K, desc)
    out_pool = torch.full((n, k, hpo, wpo), float("nan"), dtype=torch.float32, device="cuda")
    xnor.xnor_conv2d_pool(bufs.xbits, pw.wmfma, bufs.K if give_K else None, None if give_K else bufs.A, pw.alpha,
                          out_pool, desc, pool, pstride, relu)
    xnor.xnor_conv2d(bufs.xbits, pw.wbits, pw.wmfma, bufs.K, None, pw.alpha, bufs.out, None, desc, xnor.XNOR_ALGO_MFMA_F4)
    torch.cuda.synchronize()
    return out_pool.cpu().numpy(), bufs.out.cpu().numpy()


@pytest.mark.parametrize("case", CASES)
def test_conv_pool_matches_oracle(case):
    n, c, h, w, k, kh, kw, stride, pad, pool, pstride, relu, give_K = case
    print("case", case, flush=True)
    x, W = wl.random_conv_case(300 + c + k, n, c, h, w, k, kh, kw, with_zeros=True)
    got, unpooled = run(x, W, stride, pad, pool, pstride, relu, give_K)
    ref = xo.max_pool(xo.binary_conv2d(x, W, stride, pad)["out"], pool, pstride, (0, 0), relu)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-6)
    if give_K:       # same K values as the unpooled launch: the pooled value is exactly one of its outputs
        assert np.array_equal(got, xo.max_pool(unpooled, pool, pstride, (0, 0), relu))


def test_errors():
    desc = xnor.make_desc(1, 8, 9, 9, 8, 3, 3, (1, 1), (1, 1))
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt, device="cuda")
    args = (z(1, 9, 9, 1, dt=torch.int32), z(xnor.wmfma_bytes(8, 8, 3, 3), dt=torch.uint8), z(1, 9, 9), None, z(8))
    for pool, pstride, status in [((10, 3), (1, 1), -2), ((3, 3), (0, 1), -2)]:
        with pytest.raises(xnor.XnorError) as e:
            xnor.xnor_conv2d_pool(*args, z(1, 8, 1, 1), desc, pool, pstride)
        assert e.value.status == status
    with pytest.raises(xnor.XnorError) as e:        # K and A both missing
        xnor.xnor_conv2d_pool(args[0], args[1], None, None, args[4], z(1, 8, 4, 4), desc, (3, 3), (2, 2))
    assert e.value.status == -1
    wide = xnor.make_desc(1, 8, 3, 300, 8, 1, 1)    # one output row is wider than the largest tile
    with pytest.raises(xnor.XnorError) as e:
        xnor.xnor_conv2d_pool(z(1, 3, 300, 1, dt=torch.int32), z(xnor.wmfma_bytes(8, 8, 1, 1), dt=torch.uint8),
                              z(1, 3, 300), None, z(8), z(1, 8, 2, 150), wide, (2, 2), (1, 2))
    assert e.value.status == -3


def test_full_size_alexnet_conv2_pool():
    layer = wl.config_layers("alexnet_conv2")[0]
    d = wl.conv_inputs(layer, wl.config_seed("alexnet_conv2"))
    pad = (layer.pad, layer.pad)
    got, unpooled = run(d["x"], d["w"], (1, 1), pad, (3, 3), (2, 2), False, True)
    ref = xo.max_pool(xo.binary_conv2d(d["x"], d["w"], (1, 1), pad)["out"], (3, 3), (2, 2))
    np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-6)
    assert np.array_equal(got, xo.max_pool(unpooled, (3, 3), (2, 2)))
