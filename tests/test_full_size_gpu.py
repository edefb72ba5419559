"""Parity at benchmark sizes for the entry points built on top of the plain block: the fused chain of config 3
(xnor_conv2d_binactiv) checked block by block against the oracle, the binary gradient at the full batch of a
config-3 layer, the k-bit and Binary-Weight-Network convolutions on one ResNet-18 stage, and the pooled epilogue
on a 13 x 13 layer at full batch.  The oracle needs a few seconds per case on the GPU machine's host cores."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import workloads as wl
from paper_1603_05279_amd import xnor
from tests import test_bingrad_gpu as bg
from tests import test_bwn_gpu as bwn
from tests import test_conv_pool_gpu as cp
from tests import test_kbit_gpu as kb
from tests.helpers import RTOL, ATOL, pack_signs_channels_last, to_dev

pytestmark = pytest.mark.gpu


def test_config3_fused_chain_block_by_block_against_the_oracle():
    """conv3 -> conv4 -> conv5 of config 3 at batch 128 through the fused entry point: no float tensor is needed
    between the blocks, but each block is also asked for its float output y so that the oracle can be fed
    exactly what the next block consumed (teacher forcing: a last-bit difference in y may flip a sign).
    Per block: y against the oracle's block output on the same input; the emitted sign words against the
    oracle's BatchNorm + sign of the library's own y, bit for bit; A_next against the oracle's; the last block's
    integer map bit for bit."""
    layers = wl.config_layers("alexnet_conv345")
    data = [wl.conv_inputs(l, wl.config_seed("alexnet_conv345", i)) for i, l in enumerate(layers)]
    descs = [xnor.make_desc(l.n, l.c, l.h, l.w, l.k_out, l.kh, l.kw, l.stride, l.pad) for l in layers]
    pws = [xnor.PackedWeights(to_dev(d["w"])) for d in data]
    bns = [(to_dev(d["bn_scale"]), to_dev(d["bn_shift"])) for d in data]
    bufs = [xnor.ConvBuffers(d, with_dot=True) for d in descs]
    xnor.xnor_binactiv(to_dev(data[0]["x"]), bns[0][0], bns[0][1], bufs[0].xbits, bufs[0].A, None, descs[0])
    for i in range(2):
        ws = torch.empty((max(16, xnor.conv2d_binactiv_workspace_bytes(descs[i])),), dtype=torch.uint8, device="cuda")
        bufs[i].out.fill_(float("nan"))
        xnor.xnor_conv2d_binactiv(bufs[i].xbits, pws[i].wbits, pws[i].wmfma, None, bufs[i].A, pws[i].alpha,
                                  bns[i + 1][0], bns[i + 1][1], bufs[i + 1].xbits, bufs[i + 1].A, bufs[i].out, ws,
                                  descs[i], xnor.XNOR_ALGO_AUTO)
    xnor.xnor_conv2d(bufs[2].xbits, pws[2].wbits, pws[2].wmfma, None, bufs[2].A, pws[2].alpha, bufs[2].out,
                     bufs[2].dot, descs[2], xnor.XNOR_ALGO_AUTO)
    torch.cuda.synchronize()
    x_in = data[0]["x"]
    for i, layer in enumerate(layers):
        print("block", i, layer.name, flush=True)
        d = data[i]
        r = xo.binary_conv2d(x_in, d["w"], (1, 1), (1, 1), d["bn_scale"], d["bn_shift"])
        y = bufs[i].out.cpu().numpy()
        assert np.array_equal(bufs[i].xbits.cpu().numpy().view(np.uint32), pack_signs_channels_last(xo.sign(r["y"])))
        np.testing.assert_allclose(bufs[i].A.cpu().numpy(), xo.A_map(r["y"]), rtol=RTOL, atol=ATOL)
        np.testing.assert_allclose(y, r["out"], rtol=RTOL, atol=ATOL)
        if i == 2:
            assert np.array_equal(bufs[2].dot.cpu().numpy(), r["dot"])
        x_in = y          # the next block's input is what the library produced


def test_binary_gradient_full_batch_of_alexnet_conv3():
    layer = wl.config_layers("alexnet_conv345")[0]
    d = wl.conv_inputs(layer, wl.config_seed("alexnet_conv345"))
    x, W = d["x"], d["w"]
    pad = (layer.pad, layer.pad)
    rng = np.random.default_rng(78)
    g = rng.standard_normal((layer.n, layer.k_out, layer.h_out, layer.w_out)).astype(np.float32)
    fwd = xo.binary_conv2d(x, W, (1, 1), pad)
    K, alpha = fwd["K"].astype(np.float32), fwd["alpha"].astype(np.float32)
    r = bg.run(g, W, K, alpha, (layer.h, layer.w), pad, "auto")
    bg.check(r, g, W, K, alpha, (layer.h, layer.w), pad)


@pytest.mark.parametrize("bits", [(2, 2), (4, 4)])
def test_kbit_on_resnet18_256x14_full_batch(bits):
    """256 filters over 256 channels: the tilings that hold every filter in one workgroup."""
    layer = wl.config_layers("resnet18")[2]
    ka, kw_bits = bits
    rng = np.random.default_rng(500 + ka)
    x = rng.uniform(-1.1, 1.1, (layer.n, layer.c, layer.h, layer.w)).astype(np.float32)
    W = rng.uniform(-1, 1, (layer.k_out, layer.c, layer.kh, layer.kw)).astype(np.float32)
    out, num, xq = kb.run(x, W, (1, 1), (1, 1), ka, kw_bits)
    r = xo.kbit_conv2d(x, W, ka, kw_bits, (1, 1), (1, 1))
    assert np.array_equal(xq, kb.levels_image(xo.qk_levels(x, ka)))
    assert np.array_equal(num.astype(np.int64), r["num"])
    np.testing.assert_allclose(out, r["out"], rtol=1e-6, atol=0)


def test_bwn_on_resnet18_256x14_full_batch():
    layer = wl.config_layers("resnet18")[2]
    d = wl.conv_inputs(layer, wl.config_seed("resnet18", 2))
    out, alpha, _ = bwn.run(d["x"], d["w"], (1, 1), (1, 1))
    bwn.check(out, alpha, d["x"], d["w"], (1, 1), (1, 1))


def test_conv_pool_on_alexnet_conv5_full_batch():
    """13 x 13 outputs, 3 x 3 / 2 pooling: the geometry where pooling in the epilogue is the faster chain."""
    layer = wl.config_layers("alexnet_conv345")[2]
    d = wl.conv_inputs(layer, wl.config_seed("alexnet_conv345", 2))
    pad = (layer.pad, layer.pad)
    got, unpooled = cp.run(d["x"], d["w"], (1, 1), pad, (3, 3), (2, 2), True, True)
    ref = xo.max_pool(xo.binary_conv2d(d["x"], d["w"], (1, 1), pad)["out"], (3, 3), (2, 2), (0, 0), True)
    np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-6)
    assert np.array_equal(got, xo.max_pool(unpooled, (3, 3), (2, 2), (0, 0), True))
