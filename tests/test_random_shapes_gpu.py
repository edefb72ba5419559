"""Seeded random problem shapes through every inner loop and the fused epilogue, element by element
against the CPU oracle: ragged pixel and filter tails, channel counts around the word size, filters
larger than the unpadded image, strides, asymmetric padding amounts."""
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


SHAPES = random_shapes(20240611, 40)


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
