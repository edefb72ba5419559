"""Thin ctypes binding of libxnor (include/xnor.h): same names, argument marshalling only.

Tensors are torch CUDA tensors used as plain device buffers; every step of the path runs in
the library's HIP kernels.  There is no fallback: a missing library raises at import of the
first call, a non-zero status raises XnorError.
"""
import ctypes
import os

import torch

# XNOR_LIBRARY selects another build of the library (development: comparing builds); default: the in-tree one
_LIB_PATH = os.environ.get("XNOR_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libxnor.so")

XNOR_ALGO_AUTO, XNOR_ALGO_POPCOUNT, XNOR_ALGO_MFMA_I8, XNOR_ALGO_MFMA_F4 = 0, 1, 2, 3
ALGOS = {"auto": XNOR_ALGO_AUTO, "popcount": XNOR_ALGO_POPCOUNT, "mfma_i8": XNOR_ALGO_MFMA_I8,
         "mfma_f4": XNOR_ALGO_MFMA_F4}

EXPORTS = ["xnor_words_per_pixel", "xnor_output_hw", "xnor_status_string", "xnor_wmfma_bytes",
           "xnor_set_tuning", "xnor_ubench",
           "xnor_binarize_pack", "xnor_compute_K", "xnor_binactiv", "xnor_binactiv_streamed", "xnor_pack_weights",
           "xnor_conv2d", "xnor_linear",
           "xnor_conv2d_binactiv_workspace_bytes", "xnor_conv2d_binactiv", "xnor_conv2d_binactiv_noalloc",
           "xnor_pool_binactiv",
           "xnor_bwn_parts_bytes", "xnor_bwn_wimg_bytes", "xnor_bwn_split", "xnor_bwn_pack_weights",
           "xnor_bwn_conv2d",
           "xnor_bingrad_pack_weights", "xnor_bingrad_binarize", "xnor_bingrad_conv2d",
           "xnor_conv2d_pool", "xnor_pool_fusion_choice",
           "xnor_kbit_input_bytes", "xnor_kbit_wimg_bytes", "xnor_kbit_pack_input", "xnor_kbit_pack_weights",
           "xnor_kbit_conv2d"]


class XnorError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__(f"{fn} failed: {status} ({status_string(status)})")


class ConvDesc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in
                ("n", "c", "h_in", "w_in", "k_out", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w")]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_1603_05279_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with paper_1603_05279_amd/build.py "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, ip = ctypes.c_void_p, ctypes.c_int
        L.xnor_words_per_pixel.argtypes = [ip]
        L.xnor_words_per_pixel.restype = ip
        L.xnor_output_hw.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(ip), ctypes.POINTER(ip)]
        L.xnor_output_hw.restype = ip
        L.xnor_status_string.argtypes = [ip]
        L.xnor_status_string.restype = ctypes.c_char_p
        L.xnor_wmfma_bytes.argtypes = [ip, ip, ip, ip]
        L.xnor_wmfma_bytes.restype = ctypes.c_size_t
        L.xnor_set_tuning.argtypes = [ip, ip]
        L.xnor_set_tuning.restype = ip
        L.xnor_ubench.argtypes = [ip, ip, ip, vp, ctypes.c_size_t, vp]
        L.xnor_ubench.restype = ip
        L.xnor_binarize_pack.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, vp]
        L.xnor_binarize_pack.restype = ip
        L.xnor_compute_K.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(ConvDesc), vp]
        L.xnor_compute_K.restype = ip
        L.xnor_binactiv.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.POINTER(ConvDesc), vp]
        L.xnor_binactiv.restype = ip
        L.xnor_binactiv_streamed.argtypes = L.xnor_binactiv.argtypes
        L.xnor_binactiv_streamed.restype = ip
        L.xnor_pack_weights.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, vp]
        L.xnor_pack_weights.restype = ip
        L.xnor_conv2d.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(ConvDesc), ip, vp]
        L.xnor_conv2d.restype = ip
        L.xnor_linear.argtypes = [vp, vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, vp]
        L.xnor_linear.restype = ip
        L.xnor_conv2d_binactiv_workspace_bytes.argtypes = [ctypes.POINTER(ConvDesc)]
        L.xnor_conv2d_binactiv_workspace_bytes.restype = ctypes.c_size_t
        L.xnor_conv2d_binactiv.argtypes = [vp] * 12 + [ctypes.POINTER(ConvDesc), ip, vp]
        L.xnor_conv2d_binactiv.restype = ip
        L.xnor_conv2d_binactiv_noalloc.argtypes = [vp] * 11 + [ctypes.POINTER(ConvDesc), ip, vp]
        L.xnor_conv2d_binactiv_noalloc.restype = ip
        L.xnor_pool_binactiv.argtypes = [vp] * 5 + [ip] * 11 + [vp]
        L.xnor_pool_binactiv.restype = ip
        L.xnor_bwn_parts_bytes.argtypes = [ip, ip, ip, ip]
        L.xnor_bwn_parts_bytes.restype = ctypes.c_size_t
        L.xnor_bwn_wimg_bytes.argtypes = [ip, ip, ip, ip]
        L.xnor_bwn_wimg_bytes.restype = ctypes.c_size_t
        L.xnor_bwn_split.argtypes = [vp, vp, ip, ip, ip, ip, vp]
        L.xnor_bwn_split.restype = ip
        L.xnor_bwn_pack_weights.argtypes = [vp, vp, vp, ip, ip, ip, ip, vp]
        L.xnor_bwn_pack_weights.restype = ip
        L.xnor_bwn_conv2d.argtypes = [vp, vp, vp, vp, ctypes.POINTER(ConvDesc), vp]
        L.xnor_bwn_conv2d.restype = ip
        L.xnor_bingrad_pack_weights.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, vp]
        L.xnor_bingrad_pack_weights.restype = ip
        L.xnor_bingrad_binarize.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(ConvDesc), vp]
        L.xnor_bingrad_binarize.restype = ip
        L.xnor_bingrad_conv2d.argtypes = [vp] * 8 + [ctypes.POINTER(ConvDesc), ip, vp]
        L.xnor_bingrad_conv2d.restype = ip
        L.xnor_conv2d_pool.argtypes = [vp] * 6 + [ctypes.POINTER(ConvDesc)] + [ip] * 5 + [vp]
        L.xnor_conv2d_pool.restype = ip
        L.xnor_pool_fusion_choice.argtypes = [ctypes.POINTER(ConvDesc), ip, ip, ip, ip]
        L.xnor_pool_fusion_choice.restype = ip
        L.xnor_kbit_input_bytes.argtypes = [ip, ip, ip, ip]
        L.xnor_kbit_input_bytes.restype = ctypes.c_size_t
        L.xnor_kbit_wimg_bytes.argtypes = [ip, ip, ip, ip]
        L.xnor_kbit_wimg_bytes.restype = ctypes.c_size_t
        L.xnor_kbit_pack_input.argtypes = [vp, vp, ip, ip, ip, ip, ip, vp]
        L.xnor_kbit_pack_input.restype = ip
        L.xnor_kbit_pack_weights.argtypes = [vp, vp, vp, ip, ip, ip, ip, ip, ip, vp]
        L.xnor_kbit_pack_weights.restype = ip
        L.xnor_kbit_conv2d.argtypes = [vp] * 5 + [ctypes.POINTER(ConvDesc), ip, ip, vp]
        L.xnor_kbit_conv2d.restype = ip
        _lib = L
    return _lib


UBENCH = {"mfma_f4": 0, "mfma_i8": 1, "popcount": 2, "fill": 3, "read": 4, "copy": 5, "mfma_f4_data": 6, "l2_read": 7, "fill_nt": 8}


def ubench(kind, workgroups, iters, buf, nbytes=None, stream=None):
    """One microbenchmark launch (include/xnor_ubench.h); buf is a torch uint8 device tensor."""
    nbytes = buf.numel() * buf.element_size() if nbytes is None else nbytes
    _check("xnor_ubench", lib().xnor_ubench(UBENCH[kind], int(workgroups), int(iters), ctypes.c_void_p(buf.data_ptr()),
                                            ctypes.c_size_t(nbytes), _stream(stream)))


def pool_fusion_choice(desc, pool, pstride):
    """1: pooling in the convolution's epilogue is the faster chain, 0: pooling on load in front of BinActiv."""
    r = lib().xnor_pool_fusion_choice(ctypes.byref(desc), int(pool[0]), int(pool[1]), int(pstride[0]), int(pstride[1]))
    if r < 0:
        raise XnorError("xnor_pool_fusion_choice", r)
    return r


def status_string(status):
    return lib().xnor_status_string(int(status)).decode()


def words_per_pixel(c):
    return lib().xnor_words_per_pixel(int(c))


def wmfma_bytes(k_out, c, kh, kw):
    return int(lib().xnor_wmfma_bytes(k_out, c, kh, kw))


def set_tuning(mfma_tile=0, lds_budget_bytes=0):
    _check("xnor_set_tuning", lib().xnor_set_tuning(int(mfma_tile), int(lds_budget_bytes)))


def make_desc(n, c, h_in, w_in, k_out, kh, kw, stride=(1, 1), pad=(0, 0)):
    if isinstance(stride, int):
        stride = (stride, stride)
    if isinstance(pad, int):
        pad = (pad, pad)
    return ConvDesc(n, c, h_in, w_in, k_out, kh, kw, stride[0], stride[1], pad[0], pad[1])


def output_hw(desc):
    ho, wo = ctypes.c_int(0), ctypes.c_int(0)
    st = lib().xnor_output_hw(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo))
    if st:
        raise XnorError("xnor_output_hw", st)
    return ho.value, wo.value


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libxnor takes device tensors")
    if not t.is_contiguous():
        raise ValueError("libxnor takes densely packed tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(fn, st):
    if st:
        raise XnorError(fn, st)


def xnor_binarize_pack(x, bn_scale, bn_shift, xbits, n, c, h, w, stream=None):
    _check("xnor_binarize_pack", lib().xnor_binarize_pack(
        _ptr(x, torch.float32), _ptr(bn_scale, torch.float32), _ptr(bn_shift, torch.float32),
        _ptr(xbits, torch.int32), n, c, h, w, _stream(stream)))


def xnor_compute_K(x, bn_scale, bn_shift, A, K, desc, stream=None):
    _check("xnor_compute_K", lib().xnor_compute_K(
        _ptr(x, torch.float32), _ptr(bn_scale, torch.float32), _ptr(bn_shift, torch.float32),
        _ptr(A, torch.float32), _ptr(K, torch.float32), ctypes.byref(desc), _stream(stream)))


def xnor_binactiv(x, bn_scale, bn_shift, xbits, A, K, desc, stream=None):
    _check("xnor_binactiv", lib().xnor_binactiv(
        _ptr(x, torch.float32), _ptr(bn_scale, torch.float32), _ptr(bn_shift, torch.float32),
        _ptr(xbits, torch.int32), _ptr(A, torch.float32), _ptr(K, torch.float32),
        ctypes.byref(desc), _stream(stream)))


def xnor_binactiv_streamed(x, bn_scale, bn_shift, xbits, A, K, desc, stream=None):
    _check("xnor_binactiv_streamed", lib().xnor_binactiv_streamed(
        _ptr(x, torch.float32), _ptr(bn_scale, torch.float32), _ptr(bn_shift, torch.float32),
        _ptr(xbits, torch.int32), _ptr(A, torch.float32), _ptr(K, torch.float32),
        ctypes.byref(desc), _stream(stream)))


def xnor_pool_binactiv(x, bn_scale, bn_shift, xbits, A, n, c, h_in, w_in, pool, stride, pad=(0, 0), relu=False,
                       stream=None):
    _check("xnor_pool_binactiv", lib().xnor_pool_binactiv(
        _ptr(x, torch.float32), _ptr(bn_scale, torch.float32), _ptr(bn_shift, torch.float32),
        _ptr(xbits, torch.int32), _ptr(A, torch.float32), n, c, h_in, w_in, pool[0], pool[1], stride[0], stride[1],
        pad[0], pad[1], int(bool(relu)), _stream(stream)))


def bwn_parts_bytes(n, c, h, w):
    return int(lib().xnor_bwn_parts_bytes(n, c, h, w))


def bwn_wimg_bytes(k_out, c, kh, kw):
    return int(lib().xnor_bwn_wimg_bytes(k_out, c, kh, kw))


def xnor_bwn_split(x, parts, n, c, h, w, stream=None):
    _check("xnor_bwn_split", lib().xnor_bwn_split(_ptr(x, torch.float32), _ptr(parts, torch.uint8), n, c, h, w,
                                                  _stream(stream)))


def xnor_bwn_pack_weights(w, alpha, wimg, k_out, c, kh, kw, stream=None):
    _check("xnor_bwn_pack_weights", lib().xnor_bwn_pack_weights(
        _ptr(w, torch.float32), _ptr(alpha, torch.float32), _ptr(wimg, torch.uint8), k_out, c, kh, kw,
        _stream(stream)))


def xnor_bwn_conv2d(parts, wimg, alpha, out, desc, stream=None):
    _check("xnor_bwn_conv2d", lib().xnor_bwn_conv2d(
        _ptr(parts, torch.uint8), _ptr(wimg, torch.uint8), _ptr(alpha, torch.float32), _ptr(out, torch.float32),
        ctypes.byref(desc), _stream(stream)))


def xnor_bingrad_pack_weights(w, wtbits, ones, wtmfma, k_out, c, kh, kw, stream=None):
    _check("xnor_bingrad_pack_weights", lib().xnor_bingrad_pack_weights(
        _ptr(w, torch.float32), _ptr(wtbits, torch.int32), _ptr(ones, torch.float32),
        _ptr(wtmfma, torch.uint8), k_out, c, kh, kw, _stream(stream)))


def xnor_bingrad_binarize(g_out, K, alpha, gbits, gmax, desc, stream=None):
    _check("xnor_bingrad_binarize", lib().xnor_bingrad_binarize(
        _ptr(g_out, torch.float32), _ptr(K, torch.float32), _ptr(alpha, torch.float32), _ptr(gbits, torch.int32),
        _ptr(gmax, torch.float32), ctypes.byref(desc), _stream(stream)))


def xnor_bingrad_conv2d(gbits, wtbits, wtmfma, gmax, ones, scale_plane, g_in, dot_out, desc, algo=XNOR_ALGO_AUTO,
                        stream=None):
    _check("xnor_bingrad_conv2d", lib().xnor_bingrad_conv2d(
        _ptr(gbits, torch.int32), _ptr(wtbits, torch.int32), _ptr(wtmfma, torch.uint8), _ptr(gmax, torch.float32),
        _ptr(ones, torch.float32), _ptr(scale_plane, torch.float32), _ptr(g_in, torch.float32),
        _ptr(dot_out, torch.int32), ctypes.byref(desc), int(algo), _stream(stream)))


def kbit_input_bytes(n, c, h, w):
    return int(lib().xnor_kbit_input_bytes(n, c, h, w))


def kbit_wimg_bytes(k_out, c, kh, kw):
    return int(lib().xnor_kbit_wimg_bytes(k_out, c, kh, kw))


def xnor_kbit_pack_input(x, xq, ka, n, c, h, w, stream=None):
    _check("xnor_kbit_pack_input", lib().xnor_kbit_pack_input(
        _ptr(x, torch.float32), _ptr(xq, torch.uint8), int(ka), n, c, h, w, _stream(stream)))


def xnor_kbit_pack_weights(w, scale, wq, ka, kw_bits, k_out, c, kh, kw, stream=None):
    _check("xnor_kbit_pack_weights", lib().xnor_kbit_pack_weights(
        _ptr(w, torch.float32), _ptr(scale, torch.float32), _ptr(wq, torch.uint8), int(ka), int(kw_bits),
        k_out, c, kh, kw, _stream(stream)))


def xnor_kbit_conv2d(xq, wq, scale, out, num_out, desc, ka, kw_bits, stream=None):
    _check("xnor_kbit_conv2d", lib().xnor_kbit_conv2d(
        _ptr(xq, torch.uint8), _ptr(wq, torch.uint8), _ptr(scale, torch.float32), _ptr(out, torch.float32),
        _ptr(num_out, torch.int32), ctypes.byref(desc), int(ka), int(kw_bits), _stream(stream)))


def xnor_pack_weights(w, wbits, alpha, wmfma, k_out, c, kh, kw, stream=None):
    _check("xnor_pack_weights", lib().xnor_pack_weights(
        _ptr(w, torch.float32), _ptr(wbits, torch.int32), _ptr(alpha, torch.float32),
        _ptr(wmfma, torch.uint8), k_out, c, kh, kw, _stream(stream)))


def xnor_conv2d(xbits, wbits, wmfma, K, A, alpha, out, dot_out, desc, algo=XNOR_ALGO_AUTO, stream=None):
    _check("xnor_conv2d", lib().xnor_conv2d(
        _ptr(xbits, torch.int32), _ptr(wbits, torch.int32), _ptr(wmfma, torch.uint8),
        _ptr(K, torch.float32), _ptr(A, torch.float32), _ptr(alpha, torch.float32), _ptr(out, torch.float32),
        _ptr(dot_out, torch.int32), ctypes.byref(desc), int(algo), _stream(stream)))


def xnor_conv2d_pool(xbits, wmfma, K, A, alpha, out_pool, desc, pool, pstride, relu=False, stream=None):
    _check("xnor_conv2d_pool", lib().xnor_conv2d_pool(
        _ptr(xbits, torch.int32), _ptr(wmfma, torch.uint8), _ptr(K, torch.float32), _ptr(A, torch.float32),
        _ptr(alpha, torch.float32), _ptr(out_pool, torch.float32), ctypes.byref(desc), pool[0], pool[1], pstride[0],
        pstride[1], int(bool(relu)), _stream(stream)))


def xnor_linear(xbits, wbits, wmfma, Krow, alpha, out, dot_out, batch, in_features, out_features,
                algo=XNOR_ALGO_AUTO, stream=None):
    _check("xnor_linear", lib().xnor_linear(
        _ptr(xbits, torch.int32), _ptr(wbits, torch.int32), _ptr(wmfma, torch.uint8),
        _ptr(Krow, torch.float32), _ptr(alpha, torch.float32), _ptr(out, torch.float32),
        _ptr(dot_out, torch.int32), batch, in_features, out_features, int(algo), _stream(stream)))


def conv2d_binactiv_workspace_bytes(desc):
    return int(lib().xnor_conv2d_binactiv_workspace_bytes(ctypes.byref(desc)))


def xnor_conv2d_binactiv(xbits, wbits, wmfma, K, A, alpha, bn_scale_next, bn_shift_next, xbits_next, A_next,
                         out, workspace, desc, algo=XNOR_ALGO_AUTO, stream=None):
    _check("xnor_conv2d_binactiv", lib().xnor_conv2d_binactiv(
        _ptr(xbits, torch.int32), _ptr(wbits, torch.int32), _ptr(wmfma, torch.uint8),
        _ptr(K, torch.float32), _ptr(A, torch.float32), _ptr(alpha, torch.float32),
        _ptr(bn_scale_next, torch.float32), _ptr(bn_shift_next, torch.float32),
        _ptr(xbits_next, torch.int32), _ptr(A_next, torch.float32), _ptr(out, torch.float32),
        _ptr(workspace, torch.uint8), ctypes.byref(desc), int(algo), _stream(stream)))


NOALLOC_SCRATCH_BYTES = 4 << 20      # XNOR_NOALLOC_SCRATCH_BYTES of include/xnor.h


def xnor_conv2d_binactiv_noalloc(xbits, wbits, wmfma, K, A, alpha, bn_scale_next, bn_shift_next, xbits_next,
                                 A_next, out, desc, algo=XNOR_ALGO_AUTO, stream=None):
    _check("xnor_conv2d_binactiv_noalloc", lib().xnor_conv2d_binactiv_noalloc(
        _ptr(xbits, torch.int32), _ptr(wbits, torch.int32), _ptr(wmfma, torch.uint8),
        _ptr(K, torch.float32), _ptr(A, torch.float32), _ptr(alpha, torch.float32),
        _ptr(bn_scale_next, torch.float32), _ptr(bn_shift_next, torch.float32),
        _ptr(xbits_next, torch.int32), _ptr(A_next, torch.float32), _ptr(out, torch.float32),
        ctypes.byref(desc), int(algo), _stream(stream)))


# ---------------------------------------------------------------------------------------------
# Buffer holders: allocation only (torch owns the device memory), no arithmetic.
class PackedWeights:
    """wbits / alpha / wmfma buffers of one layer, filled by xnor_pack_weights."""

    def __init__(self, w, device="cuda", with_mfma=True, stream=None):
        k_out, c, kh, kw = w.shape
        self.shape = (k_out, c, kh, kw)
        cw = words_per_pixel(c)
        self.wbits = torch.empty((k_out, kh, kw, cw), dtype=torch.int32, device=device)
        self.alpha = torch.empty((k_out,), dtype=torch.float32, device=device)
        self.wmfma = (torch.empty((wmfma_bytes(k_out, c, kh, kw),), dtype=torch.uint8, device=device)
                      if with_mfma else None)
        xnor_pack_weights(w, self.wbits, self.alpha, self.wmfma, k_out, c, kh, kw, stream)


class ConvBuffers:
    """Activation-side buffers of one layer: xbits, A, K, out (and optionally the int32 dot map)."""

    def __init__(self, desc, device="cuda", with_dot=False):
        self.desc = desc
        ho, wo = output_hw(desc)
        cw = words_per_pixel(desc.c)
        self.xbits = torch.empty((desc.n, desc.h_in, desc.w_in, cw), dtype=torch.int32, device=device)
        self.A = torch.empty((desc.n, desc.h_in, desc.w_in), dtype=torch.float32, device=device)
        self.K = torch.empty((desc.n, ho, wo), dtype=torch.float32, device=device)
        self.out = torch.empty((desc.n, desc.k_out, ho, wo), dtype=torch.float32, device=device)
        self.dot = (torch.empty((desc.n, desc.k_out, ho, wo), dtype=torch.int32, device=device)
                    if with_dot else None)


def binary_conv_block(x, bn_scale, bn_shift, weights, bufs, algo=XNOR_ALGO_AUTO, stream=None):
    """BatchNorm -> BinActiv -> BinConv on preallocated buffers: two library calls, two kernels
    (the convolution derives K from A in its epilogue)."""
    xnor_binactiv(x, bn_scale, bn_shift, bufs.xbits, bufs.A, None, bufs.desc, stream)
    xnor_conv2d(bufs.xbits, weights.wbits, weights.wmfma, None, bufs.A, weights.alpha, bufs.out, bufs.dot,
                bufs.desc, algo, stream)
    return bufs.out
