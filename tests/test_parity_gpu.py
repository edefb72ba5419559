"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import workloads as wl
from paper_1603_05279_amd import xnor
from tests.helpers import RTOL, ATOL, assert_block_matches_oracle, gpu_conv_block, pack_signs_channels_last, to_dev

pytestmark = pytest.mark.gpu

ALGOS = ["popcount", "mfma_i8", "mfma_f4"]

# n, c, h, w, k_out, kh, kw, stride, pad — several tiles, ragged tails, odd channel counts
SMALL = [
    (1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0)),          # smallest problem
    (1, 3, 5, 7, 2, 3, 3, (1, 1), (1, 1)),
    (2, 31, 9, 8, 5, 3, 2, (1, 1), (1, 0)),
    (3, 32, 11, 13, 33, 3, 3, (2, 2), (1, 1)),
    (2, 33, 6, 6, 7, 1, 1, (1, 1), (0, 0)),
    (5, 64, 14, 14, 64, 3, 3, (1, 1), (1, 1)),
    (3, 96, 27, 27, 40, 5, 5, (1, 1), (2, 2)),      # > 1 pixel tile per image, 3 words
    (9, 100, 7, 7, 70, 3, 3, (1, 1), (1, 1)),       # tile spans several images, channel tail
    (2, 40, 12, 10, 9, 4, 2, (2, 1), (1, 1)),       # even filter, mixed stride
    (2, 256, 13, 13, 96, 3, 3, (1, 1), (1, 1)),     # several channel chunks in LDS
    (1, 8, 40, 3, 4, 5, 3, (1, 1), (2, 1)),         # tall thin image
]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("case", SMALL)
def test_small_cases_match_oracle(case, algo):
    n, c, h, w, k_out, kh, kw, stride, pad = case
    x, wt = wl.random_conv_case(7 + c + h, n, c, h, w, k_out, kh, kw, with_zeros=True)
    print("case", case, algo, flush=True)
    g = gpu_conv_block(x, wt, stride, pad, algo=algo)
    assert_block_matches_oracle(g, x, wt, stride, pad)


@pytest.mark.parametrize("algo", ALGOS)
def test_config_tiny_full(algo):
    layer = wl.config_layers("tiny")[0]
    d = wl.conv_inputs(layer, wl.config_seed("tiny"))
    g = gpu_conv_block(d["x"], d["w"], (1, 1), (1, 1), algo=algo)
    assert_block_matches_oracle(g, d["x"], d["w"], (1, 1), (1, 1))


@pytest.mark.parametrize("algo", ALGOS)
def test_pixel_index_times_plane_size_beyond_32_bits(algo):
    """260 images of 64 x 64 output pixels: from image 257 on, (flattened pixel index) x (plane size) passes
    2^32, where a multiply-high division without its correction step names the wrong image."""
    n, c, hw, k_out = 260, 32, 64, 32
    x, wt = wl.random_conv_case(260, n, c, hw, hw, k_out, 3, 3)
    print("large pixel index", algo, flush=True)
    g = gpu_conv_block(x, wt, (1, 1), (1, 1), algo=algo)
    assert_block_matches_oracle(g, x, wt, (1, 1), (1, 1))
    g = gpu_conv_block(x, wt, (1, 1), (1, 1), algo=algo, fused=False)     # K from the stand-alone box filter
    assert_block_matches_oracle(g, x, wt, (1, 1), (1, 1))


def test_unfused_entry_points_give_identical_bits_and_K():
    x, wt = wl.random_conv_case(3, 2, 70, 9, 9, 6, 3, 3)
    a = gpu_conv_block(x, wt, (1, 1), (1, 1), fused=True)
    b = gpu_conv_block(x, wt, (1, 1), (1, 1), fused=False)
    for key in ("xbits", "A", "K", "dot", "out"):
        assert np.array_equal(a[key], b[key]), key


def test_streamed_binactiv_gives_identical_bits_A_and_K():
    """xnor_binactiv_streamed differs from xnor_binactiv in the cache policy of its loads only."""
    rng = np.random.default_rng(77)
    n, c, h, w = 3, 70, 19, 23
    x = to_dev(rng.standard_normal((n, c, h, w)).astype(np.float32))
    sc = to_dev((0.5 + rng.random(c)).astype(np.float32))
    sf = to_dev((0.1 * rng.standard_normal(c)).astype(np.float32))
    desc = xnor.make_desc(n, c, h, w, 8, 3, 3, 1, 1)
    a, b = xnor.ConvBuffers(desc), xnor.ConvBuffers(desc)
    xnor.xnor_binactiv(x, sc, sf, a.xbits, a.A, a.K, desc)
    xnor.xnor_binactiv_streamed(x, sc, sf, b.xbits, b.A, b.K, desc)
    torch.cuda.synchronize()
    assert torch.equal(a.xbits, b.xbits) and torch.equal(a.A, b.A) and torch.equal(a.K, b.K)
    _, s_ref, a_ref = xo.binactiv(x.cpu().numpy(), sc.cpu().numpy(), sf.cpu().numpy())
    assert np.array_equal(b.xbits.cpu().numpy().view(np.uint32), pack_signs_channels_last(s_ref))
    np.testing.assert_allclose(b.A.cpu().numpy(), a_ref, rtol=RTOL, atol=ATOL)


def test_batchnorm_block_matches_oracle_and_identity_fold():
    layer = wl.ConvLayer("bn_small", 4, 96, 13, 13, 48, 3, 3, 1, 1, 0.05, True)
    d = wl.conv_inputs(layer, 4242)
    g = gpu_conv_block(d["x"], d["w"], (1, 1), (1, 1), d["bn_scale"], d["bn_shift"])
    assert_block_matches_oracle(g, d["x"], d["w"], (1, 1), (1, 1), d["bn_scale"], d["bn_shift"])
    one, zero = np.ones(96, np.float32), np.zeros(96, np.float32)
    a = gpu_conv_block(d["x"], d["w"], (1, 1), (1, 1), one, zero)
    b = gpu_conv_block(d["x"], d["w"], (1, 1), (1, 1))
    for key in ("xbits", "A", "K", "dot", "out"):
        assert np.array_equal(a[key], b[key]), key


def test_popcount_without_prepared_weight_image():
    """wmfma = NULL: the vector-ALU loop falls back to the canonical wbits order."""
    x, wt = wl.random_conv_case(11, 2, 96, 9, 11, 40, 3, 3, with_zeros=True)
    r = xo.binary_conv2d(x, wt, (1, 1), (1, 1))
    desc = xnor.make_desc(2, 96, 9, 11, 40, 3, 3, 1, 1)
    pw = xnor.PackedWeights(to_dev(wt), with_mfma=False)
    bufs = xnor.ConvBuffers(desc, with_dot=True)
    xnor.xnor_binactiv(to_dev(x), None, None, bufs.xbits, bufs.A, bufs.K, desc)
    for algo in ("popcount", "auto"):
        bufs.dot.zero_()
        xnor.xnor_conv2d(bufs.xbits, pw.wbits, None, bufs.K, None, pw.alpha, bufs.out, bufs.dot, desc, xnor.ALGOS[algo])
        torch.cuda.synchronize()
        assert np.array_equal(bufs.dot.cpu().numpy(), r["dot"]), algo
        np.testing.assert_allclose(bufs.out.cpu().numpy(), r["out"], rtol=RTOL, atol=ATOL)


def test_runs_are_deterministic():
    x, wt = wl.random_conv_case(5, 3, 64, 10, 10, 64, 3, 3)
    a = gpu_conv_block(x, wt, (1, 1), (1, 1), algo="mfma_i8")
    b = gpu_conv_block(x, wt, (1, 1), (1, 1), algo="mfma_i8")
    for key in a:
        assert np.array_equal(a[key], b[key]), key


@pytest.mark.parametrize("algo", ALGOS)
def test_linear_matches_oracle(algo):
    rng = np.random.default_rng(99)
    b, f, o = 37, 1000, 130                         # ragged in every dimension
    x = rng.standard_normal((b, f)).astype(np.float32)
    w = (0.01 * rng.standard_normal((o, f))).astype(np.float32)
    r = xo.binary_linear(x, w)
    xd, wd = to_dev(x), to_dev(w.reshape(o, f, 1, 1))
    pw = xnor.PackedWeights(wd)
    desc = xnor.make_desc(b, f, 1, 1, o, 1, 1)
    bufs = xnor.ConvBuffers(desc, with_dot=True)
    xnor.xnor_binactiv(xd.reshape(b, f, 1, 1), None, None, bufs.xbits, bufs.A, bufs.K, desc)
    out = torch.full((b, o), float("nan"), device="cuda")
    dot = torch.zeros((b, o), dtype=torch.int32, device="cuda")
    xnor.xnor_linear(bufs.xbits, pw.wbits, pw.wmfma, bufs.K, pw.alpha, out, dot, b, f, o,
                     xnor.ALGOS[algo])
    torch.cuda.synchronize()
    assert np.array_equal(dot.cpu().numpy(), r["dot"])
    np.testing.assert_allclose(bufs.K.cpu().numpy().reshape(b), r["K"], rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(out.cpu().numpy(), r["out"], rtol=RTOL, atol=ATOL)


@pytest.mark.parametrize("algo", ["mfma_i8", "mfma_f4"])
@pytest.mark.parametrize("shape", [(37, 2048, 130), (70, 32 * 33, 200), (33, 4096 + 64, 33)])
def test_linear_with_waves_along_K_matches_oracle(shape, algo):
    """The 128 x 32 tiling whose two groups of four waves split the K loop (tile 15): even and odd step counts,
    ragged batch and filter counts, both operand encodings; the integer map is exact whatever the split."""
    rng = np.random.default_rng(150)
    b, f, o = shape
    x = rng.standard_normal((b, f)).astype(np.float32)
    w = (0.01 * rng.standard_normal((o, f))).astype(np.float32)
    r = xo.binary_linear(x, w)
    xd, wd = to_dev(x), to_dev(w.reshape(o, f, 1, 1))
    pw = xnor.PackedWeights(wd)
    desc = xnor.make_desc(b, f, 1, 1, o, 1, 1)
    bufs = xnor.ConvBuffers(desc, with_dot=True)
    xnor.xnor_binactiv(xd.reshape(b, f, 1, 1), None, None, bufs.xbits, bufs.A, bufs.K, desc)
    out = torch.full((b, o), float("nan"), device="cuda")
    dot = torch.zeros((b, o), dtype=torch.int32, device="cuda")
    xnor.set_tuning(15)
    try:
        xnor.xnor_linear(bufs.xbits, pw.wbits, pw.wmfma, bufs.K, pw.alpha, out, dot, b, f, o, xnor.ALGOS[algo])
        torch.cuda.synchronize()
    finally:
        xnor.set_tuning(0)
    assert np.array_equal(dot.cpu().numpy(), r["dot"])
    np.testing.assert_allclose(out.cpu().numpy(), r["out"], rtol=RTOL, atol=ATOL)


@pytest.mark.parametrize("algo", ["auto", "mfma_f4"])
def test_linear_with_few_rows_falls_back_to_the_four_wave_tiling(algo):
    """Five rows leave the activation region too small for the partial sums of the eight-wave tiling: asked for
    explicitly it is refused, the library's own choice takes the four-wave form and matches the oracle."""
    rng = np.random.default_rng(151)
    b, f, o = 5, 4096 + 64, 33
    x = rng.standard_normal((b, f)).astype(np.float32)
    w = (0.01 * rng.standard_normal((o, f))).astype(np.float32)
    r = xo.binary_linear(x, w)
    xd, wd = to_dev(x), to_dev(w.reshape(o, f, 1, 1))
    pw = xnor.PackedWeights(wd)
    desc = xnor.make_desc(b, f, 1, 1, o, 1, 1)
    bufs = xnor.ConvBuffers(desc, with_dot=True)
    xnor.xnor_binactiv(xd.reshape(b, f, 1, 1), None, None, bufs.xbits, bufs.A, bufs.K, desc)
    out = torch.full((b, o), float("nan"), device="cuda")
    dot = torch.zeros((b, o), dtype=torch.int32, device="cuda")
    xnor.set_tuning(15)
    try:
        with pytest.raises(xnor.XnorError) as e:
            xnor.xnor_linear(bufs.xbits, pw.wbits, pw.wmfma, bufs.K, pw.alpha, out, dot, b, f, o, xnor.XNOR_ALGO_MFMA_F4)
        assert e.value.status == -3
    finally:
        xnor.set_tuning(0)
    xnor.xnor_linear(bufs.xbits, pw.wbits, pw.wmfma, bufs.K, pw.alpha, out, dot, b, f, o, xnor.ALGOS[algo])
    torch.cuda.synchronize()
    assert np.array_equal(dot.cpu().numpy(), r["dot"])
    np.testing.assert_allclose(out.cpu().numpy(), r["out"], rtol=RTOL, atol=ATOL)


def test_auto_stays_exact_beyond_the_float_accumulator():
    """2^24 terms per dot product: the 4-bit path (float accumulator) is refused, the library's own choice must
    fall back to an exact integer path and still match the oracle bit for bit."""
    import torch
    from paper_1603_05279_amd import xnor
    c = 1 << 24
    rng = np.random.default_rng(24)
    x = rng.standard_normal((1, c, 1, 1)).astype(np.float32)
    w = x.reshape(1, c, 1, 1).copy()
    w[0, : c // 4] *= -1.0                                   # a quarter of the signs disagree: dot = c/2
    desc = xnor.make_desc(1, c, 1, 1, 1, 1, 1)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    pw = xnor.PackedWeights(wd)
    bufs = xnor.ConvBuffers(desc, with_dot=True)
    xnor.xnor_binactiv(xd, None, None, bufs.xbits, bufs.A, bufs.K, desc)
    with pytest.raises(xnor.XnorError) as e:
        xnor.xnor_conv2d(bufs.xbits, pw.wbits, pw.wmfma, bufs.K, None, pw.alpha, bufs.out, bufs.dot, desc,
                         xnor.XNOR_ALGO_MFMA_F4)
    assert e.value.status == -3
    xnor.xnor_conv2d(bufs.xbits, pw.wbits, pw.wmfma, bufs.K, None, pw.alpha, bufs.out, bufs.dot, desc, xnor.XNOR_ALGO_AUTO)
    torch.cuda.synchronize()
    assert bufs.dot.item() == c // 2
    ref = float(c // 2) * float(np.abs(x).astype(np.float64).mean()) ** 2
    np.testing.assert_allclose(bufs.out.item(), ref, rtol=1e-5)
