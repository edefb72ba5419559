"""Seeded random problem shapes through every inner loop and the fused epilogue, element by element
against the CPU oracle: ragged pixel and filter tails, channel counts around the word size, filters
larger than the unpadded image, strides, asymmetric padding amounts."""
import os

import numpy as np
import pytest

from paper_1603_05279_amd import workloads as wl
from tests.helpers import assert_block_matches_oracle, gpu_conv_block
from tests.test_fused_binactiv_gpu import bn_for, check_against_oracle, run_fused

pytestmark = pytest.mark.gpu


def random_shapes(seed, count):
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        n = int(rng.integers(1, 5))
        c = int(rng.choice([1, 2, 7, 31, 32, 33, 63, 64, 65, 96, 100, 129]))
        h, w = int(rng.integers(1, 21)), int(rng.integers(1, 21))
        k_out = int(rng.choice([1, 3, 31, 32, 33, 64, 70, 127, 128, 130, 200, 257]))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, kh)), int(rng.integers(0, kw))      # pad < kernel
        if kh > h + 2 * ph or kw > w + 2 * pw:
            continue
        shapes.append((n, c, h, w, k_out, kh, kw, (sh, sw), (ph, pw)))
    return shapes


# XNOR_TEST_SHAPES / XNOR_TEST_SEED widen the sweep for a soak run (defaults keep the suite short)
SHAPES = random_shapes(int(os.environ.get("XNOR_TEST_SEED", 20240611)), int(os.environ.get("XNOR_TEST_SHAPES", 40)))


@pytest.mark.parametrize("algo", ["popcount", "mfma_i8", "mfma_f4"])
def test_random_shapes_match_oracle(algo):
    for idx, (n, c, h, w, k_out, kh, kw, stride, pad) in enumerate(SHAPES):
        print("shape", idx, (n, c, h, w, k_out, kh, kw, stride, pad), algo, flush=True)
        x, wt = wl.random_conv_case(900 + idx, n, c, h, w, k_out, kh, kw, with_zeros=(idx % 3 == 0))
        g = gpu_conv_block(x, wt, stride, pad, algo=algo)
        assert_block_matches_oracle(g, x, wt, stride, pad)


@pytest.mark.parametrize("algo", ["mfma_i8", "mfma_f4"])
def test_random_shapes_fused_epilogue(algo):
    for idx, (n, c, h, w, k_out, kh, kw, stride, pad) in enumerate(SHAPES[::2]):
        print("shape", idx, (n, c, h, w, k_out, kh, kw, stride, pad), algo, flush=True)
        x, wt = wl.random_conv_case(1900 + idx, n, c, h, w, k_out, kh, kw, with_zeros=(idx % 3 == 0))
        bn = bn_for(k_out, 77 + idx) if idx % 2 else None
        g = run_fused(x, wt, stride, pad, bn, algo)
        check_against_oracle(g, x, wt, stride, pad, bn)


# ---- the widened entry points on the same seeded shapes -----------------------------------------------
def test_random_shapes_bwn():
    from tests.test_bwn_gpu import check as check_bwn, run as run_bwn
    for idx, (n, c, h, w, k_out, kh, kw, stride, pad) in enumerate(SHAPES[::2]):
        print("shape", idx, (n, c, h, w, k_out, kh, kw, stride, pad), "bwn", flush=True)
        x, wt = wl.random_conv_case(2900 + idx, n, c, h, w, k_out, kh, kw, with_zeros=(idx % 3 == 0))
        out, alpha, _ = run_bwn(x, wt, stride, pad)
        check_bwn(out, alpha, x, wt, stride, pad)


def test_random_shapes_binary_gradient():
    from oracle import xnor_oracle as xo
    from tests.test_bingrad_gpu import check as check_bg, run as run_bg
    done = 0
    for idx, (n, c, h, w, k_out, kh, kw, stride, pad) in enumerate(SHAPES):
        print("shape", idx, (n, c, h, w, k_out, kh, kw, stride, pad), "bingrad", flush=True)
        x, wt = wl.random_conv_case(3900 + idx, n, c, h, w, k_out, kh, kw)
        ho, wo = xo.out_hw(h, w, kh, kw, stride, pad)
        g = np.random.default_rng(idx).standard_normal((n, k_out, ho, wo)).astype(np.float32)
        fwd = xo.binary_conv2d(x, wt, stride, pad)
        K, alpha = fwd["K"].astype(np.float32), fwd["alpha"].astype(np.float32)
        # strided layers run on the matrix-core paths only
        algo = ("popcount", "mfma_i8", "mfma_f4")[idx % 3] if stride == (1, 1) else ("mfma_i8", "mfma_f4", "auto")[idx % 3]
        check_bg(run_bg(g, wt, K, alpha, (h, w), pad, algo, stride=stride), g, wt, K, alpha, (h, w), pad, stride=stride)
        done += 1
    assert done >= 20


def test_random_shapes_kbit():
    from oracle import xnor_oracle as xo
    from tests.test_kbit_gpu import levels_image, run as run_kbit
    rng = np.random.default_rng(77)
    for idx, (n, c, h, w, k_out, kh, kw, stride, pad) in enumerate(SHAPES[1::3]):
        ka, kb = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        print("shape", idx, (n, c, h, w, k_out, kh, kw, stride, pad), "kbit", ka, kb, flush=True)
        x = rng.uniform(-1.1, 1.1, (n, c, h, w)).astype(np.float32)
        wt = rng.uniform(-1, 1, (k_out, c, kh, kw)).astype(np.float32)
        out, num, xq = run_kbit(x, wt, stride, pad, ka, kb)
        r = xo.kbit_conv2d(x, wt, ka, kb, stride, pad)
        assert np.array_equal(xq, levels_image(xo.qk_levels(x, ka)))
        assert np.array_equal(num.astype(np.int64), r["num"])
        np.testing.assert_allclose(out, r["out"], rtol=1e-6, atol=0)


def test_random_shapes_conv_pool():
    from oracle import xnor_oracle as xo
    from tests.test_conv_pool_gpu import run as run_pool
    rng = np.random.default_rng(78)
    done = 0
    for idx, (n, c, h, w, k_out, kh, kw, stride, pad) in enumerate(SHAPES):
        ho, wo = xo.out_hw(h, w, kh, kw, stride, pad)
        pool = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        pstride = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
        if pool[0] > ho or pool[1] > wo:
            continue
        relu = bool(idx % 2)
        print("shape", idx, (n, c, h, w, k_out, kh, kw, stride, pad), "pool", pool, pstride, relu, flush=True)
        x, wt = wl.random_conv_case(4900 + idx, n, c, h, w, k_out, kh, kw, with_zeros=(idx % 3 == 0))
        got, unpooled = run_pool(x, wt, stride, pad, pool, pstride, relu, True)
        ref = xo.max_pool(xo.binary_conv2d(x, wt, stride, pad)["out"], pool, pstride, (0, 0), relu)
        np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-6)
        assert np.array_equal(got, xo.max_pool(unpooled, pool, pstride, (0, 0), relu))
        done += 1
    assert done >= 20
