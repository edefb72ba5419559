"""The library is asynchronous on the caller's stream, allocates nothing and keeps no state between
calls, so a block can be issued on a side stream or captured into a HIP graph; every replay must
reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import workloads as wl
from paper_1603_05279_amd import xnor
from tests.helpers import to_dev

pytestmark = pytest.mark.gpu


def _setup(seed=3):
    layer = wl.ConvLayer("g", 6, 96, 13, 13, 64, 3, 3, 1, 1, 0.05, True)
    d = wl.conv_inputs(layer, seed)
    desc = xnor.make_desc(layer.n, layer.c, layer.h, layer.w, layer.k_out, 3, 3, 1, 1)
    x = to_dev(d["x"])
    sc, sf = to_dev(d["bn_scale"]), to_dev(d["bn_shift"])
    pw = xnor.PackedWeights(to_dev(d["w"]))
    bufs = xnor.ConvBuffers(desc, with_dot=True)
    ref = xo.binary_conv2d(d["x"], d["w"], (1, 1), (1, 1), d["bn_scale"], d["bn_shift"])
    return x, sc, sf, pw, bufs, ref


def test_block_on_a_side_stream_matches_oracle():
    x, sc, sf, pw, bufs, ref = _setup()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        xnor.binary_conv_block(x, sc, sf, pw, bufs, xnor.XNOR_ALGO_AUTO)     # picks up the current (side) stream
    side.synchronize()
    assert np.array_equal(bufs.dot.cpu().numpy(), ref["dot"])
    np.testing.assert_allclose(bufs.out.cpu().numpy(), ref["out"], rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("algo", ["mfma_f4", "mfma_i8", "popcount"])
def test_graph_replays_reproduce_eager_results(algo):
    x, sc, sf, pw, bufs, ref = _setup(5)
    a = xnor.ALGOS[algo]
    xnor.binary_conv_block(x, sc, sf, pw, bufs, a)                     # eager, also warms one-time setup
    torch.cuda.synchronize()
    eager_out, eager_dot = bufs.out.clone(), bufs.dot.clone()
    assert np.array_equal(eager_dot.cpu().numpy(), ref["dot"])
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        xnor.binary_conv_block(x, sc, sf, pw, bufs, a)
    torch.cuda.synchronize()
    for replay in range(4):
        bufs.out.fill_(float("nan"))
        bufs.dot.fill_(-1)
        bufs.xbits.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(bufs.out, eager_out), replay
        assert torch.equal(bufs.dot, eager_dot), replay
        xnor.binary_conv_block(x, sc, sf, pw, bufs, a)                 # eager work between replays
        torch.cuda.synchronize()


def test_full_size_sampled_properties():
    """Properties that hold at any size, on the alexnet_conv2 shape: parity of every dot entry with
    the number of valid terms, the bound |dot| <= n_valid, antisymmetry under input negation."""
    layer = wl.config_layers("alexnet_conv2")[0].with_batch(16)
    d = wl.conv_inputs(layer, 77)
    desc = xnor.make_desc(layer.n, layer.c, layer.h, layer.w, layer.k_out, 5, 5, 1, 2)
    pw = xnor.PackedWeights(to_dev(d["w"]))
    bufs = xnor.ConvBuffers(desc, with_dot=True)
    x = to_dev(d["x"])
    xnor.binary_conv_block(x, None, None, pw, bufs)
    torch.cuda.synchronize()
    dot = bufs.dot.cpu().numpy().astype(np.int64)
    idx = np.arange(27)
    valid = np.minimum(idx + 2, 26) - np.maximum(idx - 2, 0) + 1          # in-bounds taps per axis
    n_valid = 96 * valid[:, None] * valid[None, :]
    assert np.all((dot - n_valid) % 2 == 0)
    assert np.all(np.abs(dot) <= n_valid)
    out_pos = bufs.out.clone()
    xnor.binary_conv_block(-x, None, None, pw, bufs)                      # N(0,1) draws contain no zeros
    torch.cuda.synchronize()
    assert np.array_equal(bufs.dot.cpu().numpy().astype(np.int64), -dot)
    assert torch.equal(bufs.out, -out_pos)
