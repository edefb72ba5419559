"""xnor_conv2d_binactiv_noalloc (library-owned scratch, no workspace argument) against xnor_conv2d_binactiv
(caller workspace) through the C ABI: same sign words, same A_next, same y, bit for bit, on two calls in a
row, the second with a smaller input (the scratch keeps the first call's contents).  Both shapes have more than
one filter tile, so the partial |z| sums really travel through the scratch."""
import ctypes

import numpy as np
import pytest
import torch

from paper_1603_05279_amd import xnor
from tests.helpers import to_dev

pytestmark = pytest.mark.gpu


def both_entry_points(rng, n, c, h, w, k_out, kh, pad, bn):
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    wt = (0.05 * rng.standard_normal((k_out, c, kh, kh))).astype(np.float32)
    desc = xnor.make_desc(n, c, h, w, k_out, kh, kh, 1, pad)
    ho, wo = xnor.output_hw(desc)
    pw = xnor.PackedWeights(to_dev(wt))
    bufs = xnor.ConvBuffers(desc)
    sc = to_dev(rng.uniform(0.5, 1.5, k_out).astype(np.float32)) if bn else None
    sf = to_dev((0.1 * rng.standard_normal(k_out)).astype(np.float32)) if bn else None
    xnor.xnor_binactiv(to_dev(x), None, None, bufs.xbits, bufs.A, None, desc)
    ws_bytes = xnor.conv2d_binactiv_workspace_bytes(desc)
    assert 0 < ws_bytes <= xnor.NOALLOC_SCRATCH_BYTES
    res = []
    for noalloc in (False, True):
        xb = torch.full((n, ho, wo, xnor.words_per_pixel(k_out)), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        An = torch.full((n, ho, wo), float("nan"), dtype=torch.float32, device="cuda")
        out = torch.full((n, k_out, ho, wo), float("nan"), dtype=torch.float32, device="cuda")
        if noalloc:
            xnor.xnor_conv2d_binactiv_noalloc(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha, sc, sf, xb, An,
                                              out, desc, xnor.XNOR_ALGO_AUTO)
        else:
            ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
            xnor.xnor_conv2d_binactiv(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha, sc, sf, xb, An, out,
                                      ws, desc, xnor.XNOR_ALGO_AUTO)
        torch.cuda.synchronize()
        res.append((xb.cpu().numpy(), An.cpu().numpy(), out.cpu().numpy()))
    return res


def test_noalloc_entry_point_matches_the_workspace_one_twice_in_a_row():
    rng = np.random.default_rng(707)
    # first call: 384 filters over 3 x 13 x 13 pixels; second, smaller: 200 filters over 2 x 7 x 9 pixels
    for shape in [(3, 96, 13, 13, 384, 3, 1, True), (2, 40, 7, 9, 200, 3, 1, False)]:
        (xb0, an0, y0), (xb1, an1, y1) = both_entry_points(rng, *shape)
        assert not np.isnan(an0).any() and not np.isnan(y0).any()
        assert np.array_equal(xb0, xb1), "sign words differ"
        assert np.array_equal(an0.view(np.uint32), an1.view(np.uint32)), "A_next differs"
        assert np.array_equal(y0.view(np.uint32), y1.view(np.uint32)), "y differs"


def test_noalloc_entry_point_refuses_what_does_not_fit():
    L = xnor.lib()
    fake = ctypes.c_void_p(0x1000)
    # 128 filters over 256 x 64 x 64 pixels: 4 filter blocks x 1 Mi pixels x 4 bytes = 16 MiB of partial sums
    big = xnor.make_desc(256, 64, 64, 64, 128, 3, 3, 1, 1)
    assert xnor.conv2d_binactiv_workspace_bytes(big) > xnor.NOALLOC_SCRATCH_BYTES
    assert L.xnor_conv2d_binactiv_noalloc(fake, fake, fake, None, fake, fake, None, None, fake, fake, None,
                                          ctypes.byref(big), 0, None) == -3
