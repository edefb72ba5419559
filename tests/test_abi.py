"""The C-ABI library loads, exports every function include/xnor.h declares, and turns invalid
arguments into error codes before anything is launched (no GPU needed)."""
import ctypes
import glob
import os
import re
import subprocess

import pytest

from paper_1603_05279_amd import xnor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(xnor_[a-zA-Z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert set(xnor.EXPORTS) == set(names)
    L = xnor.lib()
    for name in names:
        assert getattr(L, name) is not None


def test_library_exports_nothing_but_the_c_abi():
    """Hidden visibility: the dynamic symbol table defines the declared xnor_* functions and no internal one."""
    out = subprocess.run(["nm", "-D", "--defined-only", xnor._LIB_PATH], capture_output=True, text=True, check=True)
    defined = {line.split()[-1] for line in out.stdout.splitlines() if line.split()[1:2] and line.split()[-2] in "TWtwV"}
    ours = {s for s in defined if "xnor" in s}
    assert ours == set(declared_functions()), ours ^ set(declared_functions())


def test_small_queries():
    assert [xnor.words_per_pixel(c) for c in (1, 31, 32, 33, 96, 9216)] == [1, 1, 1, 2, 3, 288]
    assert xnor.words_per_pixel(0) == 0
    # int8 image: one KiB per (32 filters, tap, word); 4-bit image: one KiB per two (tap, word) blocks;
    # each image ends with one all-zero KiB; then the scalar-path word image, 128 bytes per (block, tap, word)
    assert xnor.wmfma_bytes(256, 96, 5, 5) == (8 * 25 * 3 + 1) * 1024 + (8 * 38 + 1) * 1024 + 8 * 25 * 3 * 128
    assert xnor.wmfma_bytes(33, 1, 1, 1) == 3 * 1024 + 3 * 1024 + 2 * 128
    assert xnor.wmfma_bytes(0, 1, 1, 1) == 0
    assert xnor.output_hw(xnor.make_desc(64, 96, 27, 27, 256, 5, 5, 1, 2)) == (27, 27)
    assert xnor.output_hw(xnor.make_desc(1, 5, 7, 6, 2, 2, 2, 2, 1)) == (4, 4)
    assert xnor.status_string(0) == "ok"
    assert "NULL" in xnor.status_string(-1)


def test_pool_fusion_choice_follows_the_measured_rule():
    conv2 = xnor.make_desc(64, 96, 27, 27, 256, 5, 5, 1, 2)
    conv5 = xnor.make_desc(128, 384, 13, 13, 256, 3, 3, 1, 1)
    res14 = xnor.make_desc(256, 256, 14, 14, 256, 3, 3, 1, 1)
    res28 = xnor.make_desc(256, 128, 28, 28, 128, 3, 3, 1, 1)
    res56 = xnor.make_desc(256, 64, 56, 56, 64, 3, 3, 1, 1)
    assert xnor.pool_fusion_choice(conv5, (3, 3), (2, 2)) == 1
    assert xnor.pool_fusion_choice(res14, (2, 2), (2, 2)) == 1
    assert xnor.pool_fusion_choice(conv2, (3, 3), (2, 2)) == 0
    assert xnor.pool_fusion_choice(res28, (3, 3), (2, 2)) == 0
    assert xnor.pool_fusion_choice(res56, (4, 4), (2, 2)) == 0        # four rows of 56 pixels exceed the pooled tile
    with pytest.raises(xnor.XnorError):
        xnor.pool_fusion_choice(conv5, (14, 14), (1, 1))              # window larger than the output


def test_invalid_arguments_return_error_codes_without_launching():
    L = xnor.lib()
    good = xnor.make_desc(1, 64, 14, 14, 64, 3, 3, 1, 1)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    ERR_NULL, ERR_SHAPE, ERR_UNSUP, ERR_ALIGN = -1, -2, -3, -4
    assert L.xnor_binarize_pack(None, None, None, fake, 1, 1, 1, 1, None) == ERR_NULL
    assert L.xnor_binarize_pack(fake, None, None, fake, 0, 1, 1, 1, None) == ERR_SHAPE
    assert L.xnor_binarize_pack(odd, None, None, fake, 1, 1, 1, 1, None) == ERR_ALIGN
    assert L.xnor_binarize_pack(fake, fake, None, fake, 1, 1, 1, 1, None) == ERR_NULL   # scale without shift
    assert L.xnor_compute_K(fake, None, None, None, fake, ctypes.byref(good), None) == ERR_NULL
    assert L.xnor_compute_K(fake, None, None, fake, fake, None, None) == ERR_NULL
    assert L.xnor_pack_weights(fake, fake, None, None, 1, 1, 1, 1, None) == ERR_NULL
    assert L.xnor_pack_weights(fake, fake, fake, None, 1, -1, 1, 1, None) == ERR_SHAPE
    assert L.xnor_conv2d(fake, fake, None, fake, None, fake, None, None, ctypes.byref(good), 0, None) == ERR_NULL
    assert L.xnor_conv2d(fake, fake, None, None, None, fake, fake, None, ctypes.byref(good), 1, None) == ERR_NULL  # K or A
    assert L.xnor_conv2d(fake, fake, None, fake, None, fake, fake, None, ctypes.byref(good), 2, None) == ERR_NULL  # mfma needs wmfma
    assert L.xnor_conv2d(fake, fake, None, fake, None, fake, fake, None, ctypes.byref(good), 99, None) == ERR_UNSUP
    assert L.xnor_conv2d(fake, fake, None, None, fake, fake, odd, None, ctypes.byref(good), 1, None) == ERR_ALIGN
    big_filter = xnor.make_desc(1, 8, 3, 3, 4, 5, 5, 1, 0)
    assert L.xnor_conv2d(fake, fake, None, fake, None, fake, fake, None, ctypes.byref(big_filter), 1, None) == ERR_SHAPE
    zero_stride = xnor.make_desc(1, 8, 3, 3, 4, 3, 3, 0, 0)
    assert L.xnor_binactiv(fake, None, None, fake, fake, fake, ctypes.byref(zero_stride), None) == ERR_SHAPE
    assert L.xnor_binactiv_streamed(fake, None, None, fake, fake, fake, ctypes.byref(zero_stride), None) == ERR_SHAPE
    assert L.xnor_binactiv_streamed(None, None, None, fake, fake, fake, ctypes.byref(good), None) == ERR_NULL
    assert L.xnor_binactiv_streamed(fake, None, None, odd, fake, fake, ctypes.byref(good), None) == ERR_ALIGN
    assert L.xnor_binactiv_streamed(fake, fake, None, fake, fake, fake, ctypes.byref(good), None) == ERR_NULL   # scale without shift
    assert L.xnor_linear(fake, fake, None, fake, fake, fake, None, 0, 8, 8, 1, None) == ERR_SHAPE
    assert L.xnor_conv2d(fake, fake, None, fake, None, fake, fake, None, ctypes.byref(good), 3, None) == ERR_NULL
    # matrix-core kernels address a tile's results with 32-bit offsets: an image whose output exceeds
    # 2 GiB is refused by them before any launch (XNOR_ALGO_AUTO would take the popcount kernel)
    huge = xnor.make_desc(1, 32, 256, 256, 32768, 1, 1, 1, 0)
    assert L.xnor_conv2d(fake, fake, fake, fake, None, fake, fake, None, ctypes.byref(huge), 3, None) == ERR_UNSUP
    assert L.xnor_conv2d(fake, fake, fake, fake, None, fake, fake, None, ctypes.byref(huge), 2, None) == ERR_UNSUP
    # fused epilogue: matrix-core loops only, workspace required above 64 filters
    assert L.xnor_conv2d_binactiv(fake, fake, fake, fake, None, fake, None, None, fake, fake, None, fake,
                                  ctypes.byref(good), 1, None) == ERR_UNSUP
    wide = xnor.make_desc(1, 64, 14, 14, 96, 3, 3, 1, 1)
    assert L.xnor_conv2d_binactiv(fake, fake, fake, fake, None, fake, None, None, fake, fake, None, None,
                                  ctypes.byref(wide), 0, None) == ERR_NULL
    assert L.xnor_conv2d_binactiv_workspace_bytes(ctypes.byref(good)) == 0
    assert L.xnor_conv2d_binactiv_workspace_bytes(ctypes.byref(wide)) == 3 * 14 * 14 * 4
    assert L.xnor_set_tuning(99, 0) == ERR_UNSUP
    assert L.xnor_set_tuning(0, 0) == 0
    # microbenchmarks: buffer, sizes and kind are checked before the launch
    assert L.xnor_ubench(0, 256, 1, None, 64, None) == ERR_NULL
    assert L.xnor_ubench(0, 0, 1, fake, 64, None) == ERR_SHAPE
    assert L.xnor_ubench(3, 256, 0, fake, 48, None) == ERR_SHAPE            # fill: a multiple of 32 bytes
    assert L.xnor_ubench(6, 256, 1, fake, 8, None) == ERR_SHAPE             # changing operands: 16 bytes of counts
    assert L.xnor_ubench(7, 256, 1, fake, 65536 + 32, None) == ERR_SHAPE    # L2 stream: whole 64 KiB windows
    assert L.xnor_ubench(0, 256, 1, odd, 64, None) == ERR_ALIGN
    assert L.xnor_ubench(42, 256, 1, fake, 64, None) == ERR_UNSUP
    with pytest.raises(xnor.XnorError):
        xnor.output_hw(big_filter)
