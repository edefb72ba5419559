"""Parity of the binary-gradient backward convolution (sec. 3.2, "Binary Gradient") with the CPU oracle,
through the C ABI: sign words and per-image maximum of the gradient bit-exact, the integer map
bit-exact, the scaled data gradient within 1e-5 relative / 1e-6 absolute."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import workloads as wl
from paper_1603_05279_amd import xnor
from tests.helpers import to_dev

pytestmark = pytest.mark.gpu

# forward layer: n, c, h, w, k_out, kh, kw, pad  (stride 1; strided layers below)
CASES = [
    (1, 1, 1, 1, 1, 1, 1, (0, 0)),
    (2, 3, 5, 7, 2, 3, 3, (1, 1)),
    (2, 33, 9, 8, 31, 3, 2, (1, 0)),
    (3, 40, 11, 13, 70, 3, 3, (0, 0)),           # unpadded forward: full padding backward
    (2, 17, 6, 6, 129, 1, 1, (0, 0)),
    (5, 64, 14, 14, 64, 3, 3, (1, 1)),
    (3, 96, 27, 27, 40, 5, 5, (2, 2)),
    (4, 100, 7, 7, 200, 3, 3, (1, 1)),
    (2, 260, 12, 10, 48, 4, 2, (1, 1)),
]


def pack_bits(sg):
    """[n][k][h][w] of +-1 -> uint32 [n][h][w][ceil(k/32)], bit j of word wd = filter wd*32+j is +1."""
    n, k, h, w = sg.shape
    kw_ = (k + 31) // 32
    bits = np.zeros((n, h, w, kw_ * 32), dtype=np.uint64)
    bits[..., :k] = np.transpose(sg > 0, (0, 2, 3, 1))
    return (bits.reshape(n, h, w, kw_, 32) << np.arange(32, dtype=np.uint64)).sum(axis=-1).astype(np.uint32)


def run(g, W, K, alpha, in_hw, pad, algo, with_dot=True, stride=(1, 1)):
    n, k, ho, wo = g.shape
    _, c, kh, kw = W.shape
    h, w = in_hw
    desc = xnor.make_desc(n, c, h, w, k, kh, kw, stride, pad)
    assert xnor.output_hw(desc) == (ho, wo)
    dev = "cuda"
    wtbits = torch.empty((c, kh * kw, xnor.words_per_pixel(k)), dtype=torch.int32, device=dev)
    wtmfma = torch.empty((xnor.wmfma_bytes(c, k, kh, kw),), dtype=torch.uint8, device=dev)
    ones = torch.zeros((c,), dtype=torch.float32, device=dev)
    gbits = torch.empty((n, ho, wo, xnor.words_per_pixel(k)), dtype=torch.int32, device=dev)
    gmax = torch.full((n,), 123.0, dtype=torch.float32, device=dev)       # stale contents must not survive
    plane = torch.empty((n, h, w), dtype=torch.float32, device=dev)
    gin = torch.full((n, c, h, w), float("nan"), dtype=torch.float32, device=dev)
    dot = torch.empty((n, c, h, w), dtype=torch.int32, device=dev) if with_dot else None
    xnor.xnor_bingrad_pack_weights(to_dev(W), wtbits, ones, wtmfma, k, c, kh, kw)
    xnor.xnor_bingrad_binarize(to_dev(g), None if K is None else to_dev(K), None if alpha is None else to_dev(alpha),
                               gbits, gmax, desc)
    xnor.xnor_bingrad_conv2d(gbits, wtbits, wtmfma, gmax, ones, plane, gin, dot, desc, xnor.ALGOS[algo])
    torch.cuda.synchronize()
    return {"gbits": gbits.cpu().numpy().view(np.uint32), "gmax": gmax.cpu().numpy(), "gin": gin.cpu().numpy(),
            "dot": None if dot is None else dot.cpu().numpy(), "ones": ones.cpu().numpy()}


def check(r, g, W, K, alpha, in_hw, pad, stride=(1, 1)):
    ref = xo.binary_grad_input(g, W, K, alpha, stride, pad, in_hw=in_hw)
    assert np.array_equal(r["gbits"], pack_bits(ref["sg"]))
    assert np.array_equal(r["gmax"], ref["gmax"])
    assert (r["ones"] == 1.0).all()
    if r["dot"] is not None:
        assert np.array_equal(r["dot"], ref["dot"])
    np.testing.assert_allclose(r["gin"], ref["gin"], rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("algo", ["popcount", "mfma_i8", "mfma_f4"])
@pytest.mark.parametrize("case", CASES)
def test_bingrad_matches_oracle(case, algo):
    n, c, h, w, k, kh, kw, pad = case
    print("case", case, algo, flush=True)
    x, W = wl.random_conv_case(71 + c + k, n, c, h, w, k, kh, kw, with_zeros=True)
    ho, wo = xo.out_hw(h, w, kh, kw, (1, 1), pad)
    rng = np.random.default_rng(5 + c)
    g = (rng.standard_normal((n, k, ho, wo)) * 1e-3).astype(np.float32)
    g[rng.random(g.shape) < 0.05] = 0.0
    g.flat[0] = -0.0
    fwd = xo.binary_conv2d(x, W, (1, 1), pad)
    K = fwd["K"].astype(np.float32)
    alpha = fwd["alpha"].astype(np.float32)
    r = run(g, W, K, alpha, (h, w), pad, algo)
    check(r, g, W, K, alpha, (h, w), pad)


# n, c, h, w, k_out, kh, kw, stride, pad: strided forward layers (the gradient is staged with zeros between pixels)
STRIDED = [
    (2, 3, 9, 9, 4, 3, 3, (2, 2), (1, 1)),
    (1, 40, 11, 14, 70, 3, 3, (2, 1), (0, 1)),          # uncovered input rows at the bottom: (11 - 3) % 2 = 0, (14 + 2 - 3) % 1 = 0
    (3, 33, 12, 13, 31, 4, 2, (2, 2), (1, 0)),          # (12 + 2 - 4) % 2 = 0, (13 - 2) % 2 = 1: one uncovered column
    (2, 64, 28, 28, 128, 3, 3, (2, 2), (1, 1)),         # ResNet down-sampling geometry
    (1, 20, 17, 9, 10, 5, 3, (3, 2), (2, 1)),
    (2, 96, 16, 16, 130, 1, 1, (2, 2), (0, 0)),         # strided 1x1 (projection shortcut)
]


@pytest.mark.parametrize("algo", ["mfma_i8", "mfma_f4", "auto"])
@pytest.mark.parametrize("case", STRIDED)
def test_bingrad_strided_layers(case, algo):
    n, c, h, w, k, kh, kw, stride, pad = case
    print("case", case, algo, flush=True)
    x, W = wl.random_conv_case(171 + c + k, n, c, h, w, k, kh, kw)
    ho, wo = xo.out_hw(h, w, kh, kw, stride, pad)
    g = np.random.default_rng(15 + c).standard_normal((n, k, ho, wo)).astype(np.float32)
    fwd = xo.binary_conv2d(x, W, stride, pad)
    K, alpha = fwd["K"].astype(np.float32), fwd["alpha"].astype(np.float32)
    r = run(g, W, K, alpha, (h, w), pad, algo, stride=stride)
    check(r, g, W, K, alpha, (h, w), pad, stride=stride)


def test_without_K_and_alpha_the_gradient_itself_is_binarised():
    rng = np.random.default_rng(8)
    g = rng.standard_normal((2, 45, 6, 9)).astype(np.float32)
    W = rng.standard_normal((45, 20, 3, 3)).astype(np.float32)
    r = run(g, W, None, None, (6, 9), (1, 1), "mfma_f4")
    check(r, g, W, None, None, (6, 9), (1, 1))
    assert np.array_equal(r["gmax"], np.abs(g).reshape(2, -1).max(axis=1))


def test_all_zero_and_nan_gradients():
    g = np.zeros((2, 8, 4, 4), np.float32)
    g[1, 3, 2, 2] = np.nan                 # NaN: sign -1, ignored by the maximum
    g[1, 0, 0, 0] = -2.5
    W = np.random.default_rng(3).standard_normal((8, 5, 3, 3)).astype(np.float32)
    r = run(g, W, None, None, (4, 4), (1, 1), "mfma_f4")
    check(r, g, W, None, None, (4, 4), (1, 1))
    assert r["gmax"].tolist() == [0.0, 2.5]
    assert (r["gin"][0] == 0.0).all()


def test_errors():
    dev = "cuda"
    desc = xnor.make_desc(1, 8, 9, 9, 8, 3, 3, (2, 2), (1, 1))        # stride 2 on the vector-ALU path: not built
    t = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt, device=dev)
    import ctypes
    L = xnor.lib()
    st = L.xnor_bingrad_conv2d(t(1, 5, 5, 1, dt=torch.int32).data_ptr(), t(8, 9, 1, dt=torch.int32).data_ptr(), None,
                               t(1).data_ptr(), t(8).data_ptr(), t(1, 9, 9).data_ptr(), t(1, 8, 9, 9).data_ptr(), None,
                               ctypes.byref(desc), 1, None)
    assert st == -3
    desc = xnor.make_desc(1, 8, 9, 9, 8, 3, 3, (1, 1), (1, 1))
    assert L.xnor_bingrad_binarize(None, None, None, t(4, dt=torch.int32).data_ptr(), t(1).data_ptr(),
                                   ctypes.byref(desc), None) == -1
    assert L.xnor_bingrad_pack_weights(t(4).data_ptr(), t(4, dt=torch.int32).data_ptr(), t(4).data_ptr(), None,
                                       0, 8, 3, 3, None) == -2


def test_full_size_alexnet_conv3():
    layer = wl.config_layers("alexnet_conv345")[0]
    d = wl.conv_inputs(layer, wl.config_seed("alexnet_conv345"))
    x, W = d["x"][:16], d["w"]
    pad = (layer.pad, layer.pad)
    rng = np.random.default_rng(77)
    g = rng.standard_normal((16, layer.k_out, layer.h_out, layer.w_out)).astype(np.float32)
    fwd = xo.binary_conv2d(x, W, (1, 1), pad)
    K, alpha = fwd["K"].astype(np.float32), fwd["alpha"].astype(np.float32)
    r = run(g, W, K, alpha, (layer.h, layer.w), pad, "mfma_f4")
    check(r, g, W, K, alpha, (layer.h, layer.w), pad)
