"""Parity at the full benchmark sizes, in the launch configuration bench.py times (library's own
choice of inner loop and tiling), element by element against the oracle: the oracle finishes each
layer in about a second on the GPU machine's host cores."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import workloads as wl
from paper_1603_05279_amd import xnor
from tests.helpers import RTOL, ATOL, assert_block_matches_oracle, gpu_conv_block, to_dev

pytestmark = pytest.mark.gpu


def _run(layer, d, algo="auto"):
    s, p = (layer.stride,) * 2, (layer.pad,) * 2
    print("layer", layer.name, algo, flush=True)
    g = gpu_conv_block(d["x"], d["w"], s, p, d["bn_scale"], d["bn_shift"], algo=algo)
    assert_block_matches_oracle(g, d["x"], d["w"], s, p, d["bn_scale"], d["bn_shift"])
    return g


def test_alexnet_conv2_full_all_loops():
    layer = wl.config_layers("alexnet_conv2")[0]
    d = wl.conv_inputs(layer, wl.config_seed("alexnet_conv2"))
    for algo in ("auto", "mfma_i8", "popcount"):
        _run(layer, d, algo)


def test_alexnet_conv345_chain_full():
    """Block i+1 consumes block i's float output.  Each block is checked against the oracle fed the
    same input (the GPU's previous output), because one last-bit difference upstream may
    legitimately flip a sign downstream; the free-running oracle chain is compared as well."""
    layers = wl.config_layers("alexnet_conv345")
    x_gpu = None
    x_free = None
    for i, layer in enumerate(layers):
        d = wl.conv_inputs(layer, wl.config_seed("alexnet_conv345", i))
        if x_gpu is not None:
            d["x"] = x_gpu
        g = _run(layer, d)
        x_gpu = g["out"]
        # free-running oracle chain
        xin = d["x"] if x_free is None else x_free
        if x_free is None:
            xin = wl.conv_inputs(layer, wl.config_seed("alexnet_conv345", i))["x"]
        r = xo.binary_conv2d(xin, d["w"], (1, 1), (1, 1), d["bn_scale"], d["bn_shift"])
        x_free = r["out"]
        diff = int(np.count_nonzero(r["dot"] != g["dot"]))
        print(f"free-running chain, block {i}: {diff} of {g['dot'].size} dot entries differ", flush=True)
        # one flipped input sign changes a 3x3 neighbourhood in every filter: allow a few dozen flips
        assert diff <= 32 * 9 * layer.k_out


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_resnet18_stage_full(idx):
    layer = wl.config_layers("resnet18")[idx]
    d = wl.conv_inputs(layer, wl.config_seed("resnet18", idx))
    _run(layer, d)


@pytest.mark.parametrize("algo", ["auto", "popcount"])
def test_fc_full(algo):
    layer = wl.config_layers("fc")[0]
    d = wl.linear_inputs(layer, wl.config_seed("fc"))
    b, f, o = layer.batch, layer.in_features, layer.out_features
    r = xo.binary_linear(d["x"], d["w"])
    xd, wd = to_dev(d["x"]).reshape(b, f, 1, 1), to_dev(d["w"]).reshape(o, f, 1, 1)
    pw = xnor.PackedWeights(wd)
    desc = xnor.make_desc(b, f, 1, 1, o, 1, 1)
    bufs = xnor.ConvBuffers(desc, with_dot=True)
    xnor.xnor_binactiv(xd, None, None, bufs.xbits, bufs.A, bufs.K, desc)
    out = torch.full((b, o), float("nan"), device="cuda")
    dot = torch.zeros((b, o), dtype=torch.int32, device="cuda")
    xnor.xnor_linear(bufs.xbits, pw.wbits, pw.wmfma, bufs.K, pw.alpha, out, dot, b, f, o, xnor.ALGOS[algo])
    torch.cuda.synchronize()
    assert np.array_equal(dot.cpu().numpy(), r["dot"])
    np.testing.assert_allclose(pw.alpha.cpu().numpy(), r["alpha"], rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(bufs.K.cpu().numpy().reshape(b), r["K"], rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(out.cpu().numpy(), r["out"], rtol=RTOL, atol=ATOL)
