"""Parity of xnor_pool_binactiv (Pool -> next block's BatchNorm -> BinActiv in one pass over the float
tensor) with the CPU oracle, through the C ABI: sign words bit-exact (the pooled maximum is one of the
inputs, so both sides normalise and compare the same float32 value), A to the stated tolerance."""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import xnor
from tests.helpers import RTOL, ATOL, pack_signs_channels_last, to_dev

pytestmark = pytest.mark.gpu

# n, c, h, w, pool, stride, pad
CASES = [
    (1, 1, 1, 1, (1, 1), (1, 1), (0, 0)),          # degenerate: no pooling at all
    (2, 3, 5, 7, (2, 2), (2, 2), (0, 0)),
    (3, 33, 9, 11, (3, 2), (2, 1), (1, 1)),        # padding, mixed window and stride, channel tail
    (2, 96, 27, 27, (3, 3), (2, 2), (0, 0)),       # AlexNet pool after conv2 (small batch)
    (4, 70, 13, 13, (3, 3), (2, 2), (0, 0)),       # AlexNet pool after conv5
    (5, 64, 8, 8, (8, 8), (8, 8), (0, 0)),         # global pooling: one pixel per image
    (2, 40, 20, 6, (2, 3), (1, 3), (1, 0)),        # several 64-pixel tiles per image
]


def run(x, pool, stride, pad, bn, relu):
    n, c, h, w = x.shape
    ho, wo = (h + 2 * pad[0] - pool[0]) // stride[0] + 1, (w + 2 * pad[1] - pool[1]) // stride[1] + 1
    xb = torch.full((n, ho, wo, xnor.words_per_pixel(c)), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    A = torch.full((n, ho, wo), float("nan"), dtype=torch.float32, device="cuda")
    sc, sf = (to_dev(bn[0]), to_dev(bn[1])) if bn is not None else (None, None)
    xnor.xnor_pool_binactiv(to_dev(x), sc, sf, xb, A, n, c, h, w, pool, stride, pad, relu)
    torch.cuda.synchronize()
    return xb.cpu().numpy().view(np.uint32), A.cpu().numpy()


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("with_bn", [False, True])
@pytest.mark.parametrize("case", CASES)
def test_pool_binactiv_matches_oracle(case, with_bn, relu):
    n, c, h, w, pool, stride, pad = case
    rng = np.random.default_rng(5 + c + h)
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    x[rng.random(x.shape) < 0.05] = 0.0
    bn = ((rng.uniform(0.5, 1.5, c)).astype(np.float32), (0.3 * rng.standard_normal(c)).astype(np.float32)) \
        if with_bn else None
    print("case", case, with_bn, relu, flush=True)
    bits, A = run(x, pool, stride, pad, bn, relu)
    p = xo.max_pool(x, pool, stride, pad, relu)
    y, s, A_ref = xo.binactiv(p, *(bn if bn is not None else (None, None)))
    assert np.array_equal(bits, pack_signs_channels_last(s))
    np.testing.assert_allclose(A, A_ref, rtol=RTOL, atol=ATOL)


def test_identity_window_equals_plain_binactiv_and_nan_is_skipped():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 50, 9, 9)).astype(np.float32)
    bits, A = run(x, (1, 1), (1, 1), (0, 0), None, False)
    desc = xnor.make_desc(2, 50, 9, 9, 1, 1, 1)
    xb = torch.empty((2, 9, 9, 2), dtype=torch.int32, device="cuda")
    A2 = torch.empty((2, 9, 9), dtype=torch.float32, device="cuda")
    xnor.xnor_binactiv(to_dev(x), None, None, xb, A2, None, desc)
    torch.cuda.synchronize()
    assert np.array_equal(bits, xb.cpu().numpy().view(np.uint32))
    np.testing.assert_allclose(A, A2.cpu().numpy(), rtol=RTOL, atol=ATOL)   # other split of the channel sum
    x[0, 0, :3, :3] = np.nan
    x[0, 0, 1, 1] = -2.0                       # the only number of that window
    bits, A = run(x, (3, 3), (3, 3), (0, 0), None, False)
    p = xo.max_pool(x, (3, 3), (3, 3))
    assert p[0, 0, 0, 0] == -2.0
    y, s, A_ref = xo.binactiv(p)
    assert np.array_equal(bits, pack_signs_channels_last(s))
    np.testing.assert_allclose(A, A_ref, rtol=RTOL, atol=ATOL)


def test_full_size_alexnet_pool_after_conv2():
    # 64 x 256 x 27 x 27 -> 13 x 13 with the next block's BatchNorm: the shape between conv2 and conv3
    rng = np.random.default_rng(11)
    x = rng.standard_normal((64, 256, 27, 27)).astype(np.float32)
    bn = (rng.uniform(0.5, 1.5, 256).astype(np.float32), (0.1 * rng.standard_normal(256)).astype(np.float32))
    bits, A = run(x, (3, 3), (2, 2), (0, 0), bn, False)
    p = xo.max_pool(x, (3, 3), (2, 2))
    y, s, A_ref = xo.binactiv(p, *bn)
    assert np.array_equal(bits, pack_signs_channels_last(s))
    np.testing.assert_allclose(A, A_ref, rtol=RTOL, atol=ATOL)


def test_argument_errors():
    xb = torch.empty((1, 2, 2, 1), dtype=torch.int32, device="cuda")
    A = torch.empty((1, 2, 2), dtype=torch.float32, device="cuda")
    x = torch.zeros((1, 4, 5, 5), dtype=torch.float32, device="cuda")
    for kw, status in [(dict(pool=(6, 6)), -2), (dict(stride=(0, 1)), -2), (dict(pad=(2, 2)), -2)]:
        a = dict(pool=(3, 3), stride=(2, 2), pad=(0, 0))
        a.update(kw)
        with pytest.raises(xnor.XnorError) as e:
            xnor.xnor_pool_binactiv(x, None, None, xb, A, 1, 4, 5, 5, a["pool"], a["stride"], a["pad"])
        assert e.value.status == status, kw
