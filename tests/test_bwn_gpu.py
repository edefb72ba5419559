"""Parity of the Binary-Weight-Network convolution (real activations, +-1 weights; sec. 3.1) with the CPU
oracle, through the C ABI.

The GPU sum is a float32 accumulation of exact terms (the activations are split into three bfloat16
numbers whose sum is the float, the weights are +-1), the oracle accumulates in float64.  They differ by
the rounding of the running float sums: at most about 2^-24 per addition relative to the partial sums,
which are of the size sqrt(terms) * rms(I) for the N(0,1) inputs used here.  Tolerance:
|out - ref| <= 1e-5 * |ref| + 1e-5 * alpha_k * sqrt(c*kh*kw) * rms(I)."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import workloads as wl
from paper_1603_05279_amd import xnor
from tests.helpers import to_dev

pytestmark = pytest.mark.gpu

# n, c, h, w, k_out, kh, kw, stride, pad
CASES = [
    (1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0)),
    (1, 3, 5, 7, 2, 3, 3, (1, 1), (1, 1)),
    (2, 15, 9, 8, 5, 3, 2, (1, 1), (1, 0)),          # one partial channel group
    (3, 16, 11, 13, 33, 3, 3, (2, 2), (1, 1)),
    (2, 17, 6, 6, 7, 1, 1, (1, 1), (0, 0)),          # 1x1
    (5, 64, 14, 14, 64, 3, 3, (1, 1), (1, 1)),
    (3, 96, 27, 27, 40, 5, 5, (1, 1), (2, 2)),       # several chunks of channel words in LDS
    (4, 100, 7, 7, 200, 3, 3, (1, 1), (1, 1)),       # tile spans images, two filter tiles
    (2, 40, 12, 10, 300, 4, 2, (2, 1), (1, 1)),
]


def run(x, w, stride, pad):
    n, c, h, wd = x.shape
    k, _, kh, kw = w.shape
    desc = xnor.make_desc(n, c, h, wd, k, kh, kw, stride, pad)
    ho, wo = xnor.output_hw(desc)
    parts = torch.empty((xnor.bwn_parts_bytes(n, c, h, wd),), dtype=torch.uint8, device="cuda")
    wimg = torch.empty((xnor.bwn_wimg_bytes(k, c, kh, kw),), dtype=torch.uint8, device="cuda")
    alpha = torch.empty((k,), dtype=torch.float32, device="cuda")
    out = torch.full((n, k, ho, wo), float("nan"), dtype=torch.float32, device="cuda")
    xnor.xnor_bwn_pack_weights(to_dev(w), alpha, wimg, k, c, kh, kw)
    xnor.xnor_bwn_split(to_dev(x), parts, n, c, h, wd)
    xnor.xnor_bwn_conv2d(parts, wimg, alpha, out, desc)
    torch.cuda.synchronize()
    return out.cpu().numpy(), alpha.cpu().numpy(), parts.cpu().numpy()


def check(out, alpha, x, w, stride, pad):
    r = xo.bwn_conv2d(x, w, stride, pad)
    np.testing.assert_allclose(alpha, r["alpha"], rtol=1e-5, atol=1e-6)
    terms = w.shape[1] * w.shape[2] * w.shape[3]
    atol = 1e-5 * r["alpha"][None, :, None, None] * np.sqrt(terms) * max(float(np.sqrt(np.mean(x * x))), 1e-30)
    err = np.abs(out - r["out"])
    assert (err <= 1e-5 * np.abs(r["out"]) + atol).all(), float(err.max())


@pytest.mark.parametrize("case", CASES)
def test_bwn_matches_oracle(case):
    n, c, h, w, k, kh, kw, stride, pad = case
    x, wt = wl.random_conv_case(31 + c + h, n, c, h, w, k, kh, kw, with_zeros=True)
    print("case", case, flush=True)
    out, alpha, _ = run(x, wt, stride, pad)
    check(out, alpha, x, wt, stride, pad)


def test_split_is_exact():
    # hi + mid + lo == x bit for bit, also for tiny and large magnitudes; channel tail words are zero
    rng = np.random.default_rng(9)
    x = (rng.standard_normal((2, 19, 5, 4)) * np.exp(rng.uniform(-30, 30, (2, 19, 5, 4)))).astype(np.float32)
    x[0, 0, 0, 0] = 0.0
    x[0, 1, 0, 0] = -0.0
    _, _, parts = run(x, np.ones((1, 19, 1, 1), np.float32), (1, 1), (0, 0))
    p = parts.view(np.uint16).reshape(2, 5, 4, 2, 3, 16).astype(np.uint32)       # [n][h][w][group][part][channel]
    vals = (p << 16).view(np.float32).astype(np.float64)
    total = vals.sum(axis=4)                                                     # [n][h][w][group][16]
    total = total.reshape(2, 5, 4, 32)[..., :19]
    assert np.array_equal(total.astype(np.float32), np.transpose(x, (0, 2, 3, 1)))
    assert (p.reshape(2, 5, 4, 2, 3, 16)[:, :, :, 1, :, 3:] == 0).all()         # channels 19..31


def test_weights_of_the_form_alpha_B_give_the_float_convolution():
    # the estimate W ~ alpha*B is exact here, so BWN must equal a library float convolution
    rng = np.random.default_rng(4)
    B = (np.where(rng.standard_normal((48, 32, 3, 3)) >= 0, 1.0, -1.0) * 0.125).astype(np.float32)
    x = rng.standard_normal((3, 32, 12, 12)).astype(np.float32)
    out, alpha, _ = run(x, B, (1, 1), (1, 1))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(B).double(), None, 1, 1).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-5, atol=1e-5 * 0.125 * np.sqrt(288))


def test_full_size_alexnet_conv2():
    layer = wl.config_layers("alexnet_conv2")[0]
    d = wl.conv_inputs(layer, wl.config_seed("alexnet_conv2"))
    out, alpha, _ = run(d["x"], d["w"], (1, 1), (2, 2))
    check(out, alpha, d["x"], d["w"], (1, 1), (2, 2))
