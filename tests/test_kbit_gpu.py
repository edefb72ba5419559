"""Parity of the k-bit quantised convolution (sec. 3.2, "k-bit Quantization") with the CPU oracle, through the
C ABI: bit planes of the level indices and the integer numerator bit-exact, the quotient within 1e-6
relative (both sides divide the same integer in double and round once)."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import xnor
from tests.helpers import to_dev

pytestmark = pytest.mark.gpu

# n, c, h, w, k_out, kh, kw, stride, pad, ka, kw_bits
CASES = [
    (1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0), 1, 1),
    (2, 3, 5, 7, 2, 3, 3, (1, 1), (1, 1), 2, 1),
    (2, 33, 9, 8, 31, 3, 2, (1, 1), (1, 0), 2, 2),
    (3, 40, 11, 13, 70, 3, 3, (2, 2), (1, 1), 3, 1),
    (2, 17, 6, 6, 129, 1, 1, (1, 1), (0, 0), 4, 2),
    (5, 64, 14, 14, 64, 3, 3, (1, 1), (1, 1), 2, 2),
    (2, 96, 27, 27, 40, 5, 5, (1, 1), (2, 2), 1, 3),
    (1, 100, 7, 7, 20, 3, 3, (1, 1), (1, 1), 8, 8),
]


def run(x, W, stride, pad, ka, kb, algo):
    n, c, h, w = x.shape
    k, _, kh, kw = W.shape
    desc = xnor.make_desc(n, c, h, w, k, kh, kw, stride, pad)
    ho, wo = xnor.output_hw(desc)
    dev = "cuda"
    cw = xnor.words_per_pixel(c)
    xplanes = torch.empty((ka, n, h, w, cw), dtype=torch.int32, device=dev)
    wbits = torch.empty((kb * k, kh * kw, cw), dtype=torch.int32, device=dev)
    wmfma = torch.empty((xnor.wmfma_bytes(kb * k, c, kh, kw),), dtype=torch.uint8, device=dev)
    ones = torch.zeros((kb * k,), dtype=torch.float32, device=dev)
    ws = torch.empty((xnor.kbit_workspace_bytes(desc, ka, kb),), dtype=torch.uint8, device=dev)
    out = torch.full((n, k, ho, wo), float("nan"), dtype=torch.float32, device=dev)
    num = torch.empty((n, k, ho, wo), dtype=torch.int32, device=dev)
    xnor.xnor_kbit_pack_weights(to_dev(W), wbits, ones, wmfma, kb, k, c, kh, kw)
    xnor.xnor_kbit_pack_input(to_dev(x), xplanes, ka, n, c, h, w)
    xnor.xnor_kbit_conv2d(xplanes, wbits, wmfma, ones, ws, out, num, desc, ka, kb, xnor.ALGOS[algo])
    torch.cuda.synchronize()
    return out.cpu().numpy(), num.cpu().numpy(), xplanes.cpu().numpy().view(np.uint32)


def planes_of(a, k):
    """numerators a = 2u - L [n][c][h][w] -> packed bit planes [k][n][h][w][cw] of the level index u"""
    L = (1 << k) - 1
    u = (a + L) // 2
    n, c, h, w = a.shape
    cw = (c + 31) // 32
    out = np.zeros((k, n, h, w, cw), dtype=np.uint32)
    for p in range(k):
        bits = np.zeros((n, h, w, cw * 32), dtype=np.uint64)
        bits[..., :c] = np.transpose((u >> p) & 1, (0, 2, 3, 1))
        out[p] = (bits.reshape(n, h, w, cw, 32) << np.arange(32, dtype=np.uint64)).sum(axis=-1).astype(np.uint32)
    return out


@pytest.mark.parametrize("algo", ["popcount", "mfma_f4"])
@pytest.mark.parametrize("case", CASES)
def test_kbit_conv_matches_oracle(case, algo):
    n, c, h, w, k, kh, kw, stride, pad, ka, kb = case
    print("case", case, algo, flush=True)
    rng = np.random.default_rng(11 + c + k)
    x = rng.uniform(-1.2, 1.2, (n, c, h, w)).astype(np.float32)          # some values beyond [-1, 1]: clamped
    W = rng.uniform(-1, 1, (k, c, kh, kw)).astype(np.float32)
    x.flat[:3] = [0.0, -0.0, 1.0]
    out, num, xplanes = run(x, W, stride, pad, ka, kb, algo)
    r = xo.kbit_conv2d(x, W, ka, kb, stride, pad)
    assert np.array_equal(xplanes, planes_of(xo.qk_levels(x, ka), ka))
    assert np.array_equal(num.astype(np.int64), r["num"])
    np.testing.assert_allclose(out, r["out"], rtol=1e-6, atol=0)


def test_one_bit_each_is_the_binary_dot_map():
    rng = np.random.default_rng(2)
    x = rng.uniform(-1, 1, (2, 48, 9, 9)).astype(np.float32)
    W = rng.uniform(-1, 1, (24, 48, 3, 3)).astype(np.float32)
    out, num, _ = run(x, W, (1, 1), (1, 1), 1, 1, "mfma_f4")
    ref = xo.dot_map(xo.sign(x), xo.sign(W), (1, 1), (1, 1))
    assert np.array_equal(num, ref)
    assert np.array_equal(out, ref.astype(np.float32))


def test_level_ties_and_errors():
    # inputs exactly halfway between two levels round up, like the oracle; NaN counts as -1
    k = 2
    x = np.array([0.0, -2.0 / 3.0, 2.0 / 3.0, np.nan, -1.0, 1.0, 1.0 / 3.0, -1.0 / 3.0], np.float32).reshape(1, 8, 1, 1)
    W = np.ones((1, 8, 1, 1), np.float32)
    out, num, xplanes = run(x, W, (1, 1), (0, 0), k, 1, "popcount")
    assert np.array_equal(xplanes, planes_of(xo.qk_levels(x, k), k))
    assert num.item() == int(xo.qk_levels(x, k).sum())
    desc = xnor.make_desc(1, 8, 1, 1, 1, 1, 1)
    with pytest.raises(xnor.XnorError) as e:
        xnor.xnor_kbit_pack_input(to_dev(x), torch.empty(8, dtype=torch.int32, device="cuda"), 9, 1, 8, 1, 1)
    assert e.value.status == -2
    assert xnor.kbit_workspace_bytes(desc, 0, 1) == 0
