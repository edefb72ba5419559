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


def test_graph_replays_of_the_widened_entry_points():
    """Binary-gradient (clears its per-image maxima with a kernel, merges them with atomics), k-bit, Binary-Weight-
    Network and pooled-epilogue sequences captured in one graph: every replay reproduces the eager results bit for
    bit, with stale buffer contents and eager launches between the replays."""
    rng = np.random.default_rng(12)
    n, c, h, w, k = 4, 48, 13, 13, 72
    desc = xnor.make_desc(n, c, h, w, k, 3, 3, 1, 1)
    dev = "cuda"
    x = to_dev(rng.standard_normal((n, c, h, w)).astype(np.float32))
    wt = to_dev((rng.standard_normal((k, c, 3, 3)) * 0.05).astype(np.float32))
    g_out = to_dev(rng.standard_normal((n, k, h, w)).astype(np.float32))
    pw = xnor.PackedWeights(wt)
    bufs = xnor.ConvBuffers(desc)
    xnor.xnor_binactiv(x, None, None, bufs.xbits, bufs.A, bufs.K, desc)
    kw32, cw32 = xnor.words_per_pixel(k), xnor.words_per_pixel(c)
    u8 = lambda nbytes: torch.empty((nbytes,), dtype=torch.uint8, device=dev)
    f32 = lambda *s: torch.full(s, float("nan"), dtype=torch.float32, device=dev)
    i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=dev)
    # prepared once, outside the graph (per layer)
    wtbits, wtmfma, ones = i32(c, 9, kw32), u8(xnor.wmfma_bytes(c, k, 3, 3)), f32(c)
    xnor.xnor_bingrad_pack_weights(wt, wtbits, ones, wtmfma, k, c, 3, 3)
    wimg, alpha_b = u8(xnor.bwn_wimg_bytes(k, c, 3, 3)), f32(k)
    xnor.xnor_bwn_pack_weights(wt, alpha_b, wimg, k, c, 3, 3)
    wq2, scale2 = u8(xnor.kbit_wimg_bytes(k, c, 3, 3)), f32(k)
    xnor.xnor_kbit_pack_weights(torch.tanh(wt * 10), scale2, wq2, 2, 2, k, c, 3, 3)
    xs = torch.tanh(x)
    out = {"gbits": i32(n, h, w, kw32), "gmax": f32(n), "plane": f32(n, h, w), "gin": f32(n, c, h, w),
           "parts": u8(xnor.bwn_parts_bytes(n, c, h, w)), "bwn": f32(n, k, h, w),
           "xq": u8(xnor.kbit_input_bytes(n, c, h, w)), "kb": f32(n, k, h, w),
           "pool": f32(n, k, 6, 6)}

    def sequence():
        xnor.xnor_bingrad_binarize(g_out, bufs.K, pw.alpha, out["gbits"], out["gmax"], desc)
        xnor.xnor_bingrad_conv2d(out["gbits"], wtbits, wtmfma, out["gmax"], ones, out["plane"], out["gin"], None, desc)
        xnor.xnor_bwn_split(x, out["parts"], n, c, h, w)
        xnor.xnor_bwn_conv2d(out["parts"], wimg, alpha_b, out["bwn"], desc)
        xnor.xnor_kbit_pack_input(xs, out["xq"], 2, n, c, h, w)
        xnor.xnor_kbit_conv2d(out["xq"], wq2, scale2, out["kb"], None, desc, 2, 2)
        xnor.xnor_conv2d_pool(bufs.xbits, pw.wmfma, bufs.K, None, pw.alpha, out["pool"], desc, (3, 3), (2, 2))

    checked = ("gbits", "gmax", "gin", "bwn", "kb", "pool")
    sequence()
    torch.cuda.synchronize()
    eager = {name: out[name].clone() for name in checked}
    assert not any(torch.isnan(eager[name]).any() for name in ("gmax", "gin", "bwn", "kb", "pool"))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        sequence()
    torch.cuda.synchronize()
    for replay in range(4):
        for name in ("gmax", "plane", "gin", "bwn", "kb", "pool"):
            out[name].fill_(777.0)                    # stale contents, e.g. a maximum larger than any |gd|
        out["gbits"].fill_(-1)
        out["xq"].fill_(255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in checked:
            assert torch.equal(out[name], eager[name]), (name, replay)
        sequence()                                    # eager work between replays
        torch.cuda.synchronize()


def test_microbenchmark_kinds_run_and_report_plausible_counts():
    """Every xnor_ubench kind launches; the changing-operand matrix loop reports its own core-clock and wall-clock
    counts (a clock between 0.5 and 3 GHz, at least 32 cycles per matrix instruction and wave)."""
    buf = torch.zeros(8 << 20, dtype=torch.uint8, device="cuda")
    for kind, iters, nbytes in (("mfma_f4", 50, None), ("mfma_i8", 50, None), ("popcount", 20, None), ("fill", 0, 4 << 20),
                                ("fill_nt", 0, 4 << 20), ("read", 0, 4 << 20), ("copy", 0, 8 << 20), ("l2_read", 4, 4 << 20)):
        xnor.ubench(kind, 512, iters, buf, nbytes)
    torch.cuda.synchronize()
    buf.zero_()
    iters = 200
    xnor.ubench("mfma_f4_data", 256, iters, buf)
    torch.cuda.synchronize()
    clocks, ticks = (int(v) for v in buf[:16].view(torch.int64).cpu())
    assert ticks > 0 and clocks > 0
    ghz = clocks / (ticks * 10.0)
    assert 0.5 < ghz < 3.0, ghz
    assert clocks >= 32 * 8 * iters, clocks
