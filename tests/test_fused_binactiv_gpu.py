"""Parity of xnor_conv2d_binactiv (BinConv + the next block's BatchNorm and BinActiv in one kernel)
with the CPU oracle, through the C ABI.

The sign bits are decided by float32 values.  The convolution's float output y agrees with the
oracle's (formed in float64, rounded once) to float rounding only, so a bit whose z lies within
rounding distance of zero may legitimately differ between the two.  The tests therefore check
 (1) teacher-forced and bit-exact: the oracle's BatchNorm + sign applied to the library's own y
     (itself checked against the oracle to the stated tolerance) must give exactly the emitted bits;
 (2) free-running: against the oracle's own chain, bits may differ only where |z| is at rounding
     distance from zero.
"""
import numpy as np
import pytest
import torch

from oracle import xnor_oracle as xo
from paper_1603_05279_amd import workloads as wl
from paper_1603_05279_amd import xnor
from tests.helpers import RTOL, ATOL, pack_signs_channels_last, to_dev

pytestmark = pytest.mark.gpu

ALGOS = ["mfma_i8", "mfma_f4"]

# n, c, h, w, k_out, kh, kw, stride, pad
CASES = [
    (1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0)),          # smallest problem
    (2, 31, 9, 8, 5, 3, 2, (1, 1), (1, 0)),         # one partial filter block
    (3, 32, 11, 13, 33, 3, 3, (2, 2), (1, 1)),      # 33 filters: second word holds one bit
    (5, 64, 14, 14, 64, 3, 3, (1, 1), (1, 1)),      # exactly two words, no workspace needed
    (3, 96, 27, 27, 40, 5, 5, (1, 1), (2, 2)),      # several pixel tiles
    (9, 100, 7, 7, 70, 3, 3, (1, 1), (1, 1)),       # tile spans several images
    (2, 64, 13, 13, 200, 3, 3, (1, 1), (1, 1)),     # two filter tiles: partial sums through the workspace
    (2, 40, 10, 12, 300, 3, 3, (1, 1), (1, 1)),     # three filter tiles, ragged last one
    (2, 256, 13, 13, 96, 3, 3, (1, 1), (1, 1)),     # several channel chunks in LDS
]


def run_fused(x, w, stride, pad, bn_next, algo, with_out=True, tile=0):
    n, c, h, wd = x.shape
    k_out, _, kh, kw = w.shape
    desc = xnor.make_desc(n, c, h, wd, k_out, kh, kw, stride, pad)
    ho, wo = xnor.output_hw(desc)
    xd = to_dev(x)
    pw = xnor.PackedWeights(to_dev(w))
    bufs = xnor.ConvBuffers(desc)
    sc, sf = (to_dev(bn_next[0]), to_dev(bn_next[1])) if bn_next is not None else (None, None)
    cwn = xnor.words_per_pixel(k_out)
    xbits_next = torch.full((n, ho, wo, cwn), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    A_next = torch.full((n, ho, wo), float("nan"), dtype=torch.float32, device="cuda")
    out = torch.full((n, k_out, ho, wo), float("nan"), dtype=torch.float32, device="cuda") if with_out else None
    ws_bytes = xnor.conv2d_binactiv_workspace_bytes(desc)
    ws = torch.empty((max(ws_bytes, 16),), dtype=torch.uint8, device="cuda") if ws_bytes else None
    xnor.xnor_binactiv(xd, None, None, bufs.xbits, bufs.A, None, desc)
    xnor.set_tuning(tile)
    try:
        xnor.xnor_conv2d_binactiv(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha, sc, sf,
                                  xbits_next, A_next, out, ws, desc, xnor.ALGOS[algo])
        # the plain convolution on the same operands, for the bit-identity of y
        xnor.xnor_conv2d(bufs.xbits, pw.wbits, pw.wmfma, None, bufs.A, pw.alpha, bufs.out, None, desc,
                         xnor.ALGOS[algo])
    finally:
        xnor.set_tuning(0)
    torch.cuda.synchronize()
    return {"xbits_next": xbits_next.cpu().numpy().view(np.uint32), "A_next": A_next.cpu().numpy(),
            "out": out.cpu().numpy() if with_out else None, "out_plain": bufs.out.cpu().numpy()}


def check_against_oracle(g, x, w, stride, pad, bn_next):
    sc, sf = bn_next if bn_next is not None else (None, None)
    # (1) teacher-forced, bit-exact
    y_gpu = g["out_plain"]
    if g["out"] is not None:
        assert np.array_equal(g["out"].view(np.uint32), y_gpu.view(np.uint32)), "fused y differs from xnor_conv2d"
    z, s, A = xo.binactiv(y_gpu, sc, sf)
    assert np.array_equal(g["xbits_next"], pack_signs_channels_last(s)), "sign bits of the next block differ"
    np.testing.assert_allclose(g["A_next"], A, rtol=RTOL, atol=ATOL)
    # (2) free-running against the oracle's own chain
    r = xo.binary_conv2d(x, w, stride, pad)
    np.testing.assert_allclose(y_gpu, r["out"], rtol=RTOL, atol=ATOL)
    z_o, s_o, A_o = xo.binactiv(r["out"], sc, sf)
    np.testing.assert_allclose(g["A_next"], A_o, rtol=RTOL, atol=ATOL)
    diff = s != s_o
    if diff.any():
        scale = np.ones(w.shape[0], np.float32) if sc is None else np.abs(sc)
        bound = 4 * RTOL * np.abs(r["out"]) * scale[None, :, None, None] + 1e-30
        assert (np.abs(z_o)[diff] <= bound[diff]).all(), "a sign differs away from the rounding zone"
        assert diff.mean() < 1e-3


def bn_for(k_out, seed):
    rng = np.random.default_rng(seed)
    return (rng.uniform(0.5, 1.5, k_out).astype(np.float32), (0.05 * rng.standard_normal(k_out)).astype(np.float32))


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("with_bn", [False, True])
@pytest.mark.parametrize("case", CASES)
def test_fused_epilogue_matches_oracle(case, with_bn, algo):
    n, c, h, w, k_out, kh, kw, stride, pad = case
    x, wt = wl.random_conv_case(11 + c + h, n, c, h, w, k_out, kh, kw, with_zeros=True)
    bn = bn_for(k_out, 100 + k_out) if with_bn else None
    print("case", case, with_bn, algo, flush=True)
    g = run_fused(x, wt, stride, pad, bn, algo)
    check_against_oracle(g, x, wt, stride, pad, bn)


@pytest.mark.parametrize("tile", [1, 2, 4, 5, 11, 13, 14])
def test_every_fused_tiling_gives_the_same_bits(tile):
    x, wt = wl.random_conv_case(5, 3, 70, 15, 15, 300, 3, 3)
    bn = bn_for(300, 9)
    print("tile", tile, flush=True)
    g = run_fused(x, wt, (1, 1), (1, 1), bn, "mfma_f4", tile=tile)
    check_against_oracle(g, x, wt, (1, 1), (1, 1), bn)


def test_out_pointer_is_optional_and_results_repeat():
    x, wt = wl.random_conv_case(8, 2, 96, 13, 13, 130, 3, 3)
    bn = bn_for(130, 3)
    a = run_fused(x, wt, (1, 1), (1, 1), bn, "mfma_f4", with_out=True)
    b = run_fused(x, wt, (1, 1), (1, 1), bn, "mfma_f4", with_out=False)
    c = run_fused(x, wt, (1, 1), (1, 1), bn, "mfma_i8", with_out=False)
    for other in (b, c):
        assert np.array_equal(a["xbits_next"], other["xbits_next"])
        assert np.array_equal(a["A_next"].view(np.uint32), other["A_next"].view(np.uint32))


def test_matches_the_separate_binactiv_kernel():
    # xnor_binactiv on the float output must give the same bits; A agrees to rounding
    x, wt = wl.random_conv_case(21, 2, 64, 14, 14, 96, 3, 3)
    bn = bn_for(96, 5)
    g = run_fused(x, wt, (1, 1), (1, 1), bn, "mfma_f4")
    y = to_dev(g["out"])
    n, k, ho, wo = y.shape
    d2 = xnor.make_desc(n, k, ho, wo, 8, 1, 1)
    xb = torch.empty((n, ho, wo, xnor.words_per_pixel(k)), dtype=torch.int32, device="cuda")
    A = torch.empty((n, ho, wo), dtype=torch.float32, device="cuda")
    xnor.xnor_binactiv(y, to_dev(bn[0]), to_dev(bn[1]), xb, A, None, d2)
    torch.cuda.synchronize()
    assert np.array_equal(xb.cpu().numpy().view(np.uint32), g["xbits_next"])
    np.testing.assert_allclose(A.cpu().numpy(), g["A_next"], rtol=RTOL, atol=ATOL)


def test_chain_alexnet_conv345_fused_equals_unfused():
    """conv3 -> conv4 -> conv5 at full size: the fused chain (no float tensor between the layers) feeds
    every layer the same bits as the layer-by-layer chain, so the integer maps are identical and the
    final float output agrees to rounding (A, hence K, is summed in a different order)."""
    layers = wl.config_layers("alexnet_conv345")
    seed = wl.config_seed("alexnet_conv345")
    data = [wl.conv_inputs(l, seed + i) for i, l in enumerate(layers)]
    x0 = to_dev(data[0]["x"])
    descs = [xnor.make_desc(l.n, l.c, l.h, l.w, l.k_out, l.kh, l.kw, (l.stride, l.stride), (l.pad, l.pad))
             for l in layers]
    pws = [xnor.PackedWeights(to_dev(d["w"])) for d in data]
    bns = [(to_dev(d["bn_scale"]), to_dev(d["bn_shift"])) if d.get("bn_scale") is not None else (None, None)
           for d in data]
    bufs = [xnor.ConvBuffers(d, with_dot=True) for d in descs]
    # layer by layer
    src = x0
    for i in range(3):
        xnor.xnor_binactiv(src, bns[i][0], bns[i][1], bufs[i].xbits, bufs[i].A, None, descs[i])
        xnor.xnor_conv2d(bufs[i].xbits, pws[i].wbits, pws[i].wmfma, None, bufs[i].A, pws[i].alpha, bufs[i].out,
                         bufs[i].dot, descs[i], xnor.XNOR_ALGO_MFMA_F4)
        src = bufs[i].out
    torch.cuda.synchronize()
    ref_bits = [b.xbits.clone() for b in bufs]
    ref_dot2, ref_out2 = bufs[2].dot.clone(), bufs[2].out.clone()
    # fused: one BinActiv at the head, then each convolution emits the next layer's operands
    fb = [xnor.ConvBuffers(d, with_dot=True) for d in descs]
    xnor.xnor_binactiv(x0, bns[0][0], bns[0][1], fb[0].xbits, fb[0].A, None, descs[0])
    for i in range(2):
        nb = xnor.conv2d_binactiv_workspace_bytes(descs[i])
        ws = torch.empty((max(nb, 16),), dtype=torch.uint8, device="cuda")
        xnor.xnor_conv2d_binactiv(fb[i].xbits, pws[i].wbits, pws[i].wmfma, None, fb[i].A, pws[i].alpha,
                                  bns[i + 1][0], bns[i + 1][1], fb[i + 1].xbits, fb[i + 1].A, None, ws,
                                  descs[i], xnor.XNOR_ALGO_MFMA_F4)
    xnor.xnor_conv2d(fb[2].xbits, pws[2].wbits, pws[2].wmfma, None, fb[2].A, pws[2].alpha, fb[2].out,
                     fb[2].dot, descs[2], xnor.XNOR_ALGO_MFMA_F4)
    torch.cuda.synchronize()
    for i in range(3):
        assert torch.equal(fb[i].xbits, ref_bits[i]), f"input bits of layer {i} differ"
        np.testing.assert_allclose(fb[i].A.cpu().numpy(), bufs[i].A.cpu().numpy(), rtol=RTOL, atol=ATOL)
    assert torch.equal(fb[2].dot, ref_dot2)
    np.testing.assert_allclose(fb[2].out.cpu().numpy(), ref_out2.cpu().numpy(), rtol=RTOL, atol=ATOL)


def test_argument_errors():
    x, wt = wl.random_conv_case(1, 1, 32, 5, 5, 96, 3, 3)
    desc = xnor.make_desc(1, 32, 5, 5, 96, 3, 3, (1, 1), (1, 1))
    pw = xnor.PackedWeights(to_dev(wt))
    bufs = xnor.ConvBuffers(desc)
    xb = torch.empty((1, 5, 5, 3), dtype=torch.int32, device="cuda")
    A = torch.empty((1, 5, 5), dtype=torch.float32, device="cuda")
    ws = torch.empty((xnor.conv2d_binactiv_workspace_bytes(desc),), dtype=torch.uint8, device="cuda")
    assert xnor.conv2d_binactiv_workspace_bytes(desc) == 3 * 25 * 4

    def call(**kw):
        a = dict(xbits=bufs.xbits, wbits=pw.wbits, wmfma=pw.wmfma, K=None, A=bufs.A, alpha=pw.alpha,
                 bn_scale_next=None, bn_shift_next=None, xbits_next=xb, A_next=A, out=None, workspace=ws,
                 desc=desc, algo=xnor.XNOR_ALGO_AUTO)
        a.update(kw)
        xnor.xnor_conv2d_binactiv(**a)

    for kw, status in [(dict(algo=xnor.XNOR_ALGO_POPCOUNT), -3), (dict(workspace=None), -1),
                       (dict(xbits_next=None), -1), (dict(A_next=None), -1), (dict(wmfma=None), -1),
                       (dict(bn_scale_next=pw.alpha), -1), (dict(K=None, A=None), -1)]:
        with pytest.raises(xnor.XnorError) as e:
            call(**kw)
        assert e.value.status == status, kw
    call()
    torch.cuda.synchronize()
