"""numpy front end of the C oracle (oracle/xnor_oracle.c).

TEST INFRASTRUCTURE ONLY.  Each function marshals numpy arrays into the plain C
routine of the same name and returns new arrays; the arithmetic lives in the C file,
whose header states the passages of the paper it follows and the readings taken.
Nothing here imports or calls the HIP library.
"""
import ctypes
import os

import numpy as np

from . import build_oracle

_lib = None


def _load():
    global _lib
    if _lib is None:
        # XNOR_ORACLE_SANITIZE=1: the build instrumented with UndefinedBehaviorSanitizer (tests/test_sanitizers.py)
        path = build_oracle.build(force=False, sanitize=os.environ.get("XNOR_ORACLE_SANITIZE") == "1")
        _lib = ctypes.CDLL(path)
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def out_hw(h, w, kh, kw, stride, pad):
    sh, sw = stride
    ph, pw = pad
    return (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1


def batchnorm(x, scale=None, shift=None):
    """y = fmaf(x, scale_c, shift_c) in float32 (block order, sec. 3.2); identity if scale is None."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    n, c, h, w = x.shape
    y = np.empty_like(x)
    if scale is not None:
        scale = np.ascontiguousarray(scale, dtype=np.float32)
        shift = np.ascontiguousarray(shift, dtype=np.float32)
        assert scale.shape == (c,) and shift.shape == (c,)
    _load().xo_batchnorm(_p(x, ctypes.c_float), _p(scale, ctypes.c_float), _p(shift, ctypes.c_float),
                         _p(y, ctypes.c_float), n, c, h, w)
    return y


def sign(v):
    """+1 where v >= 0, -1 elsewhere, as int8 (sec. 3.1)."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    s = np.empty(v.shape, dtype=np.int8)
    _load().xo_sign(_p(v, ctypes.c_float), _p(s, ctypes.c_int8), ctypes.c_size_t(v.size))
    return s


def alpha(W):
    """alpha_k = ||W_k||_1 / n per filter, float64 (sec. 3.1)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    k, c, kh, kw = W.shape
    a = np.empty(k, dtype=np.float64)
    _load().xo_alpha(_p(W, ctypes.c_float), _p(a, ctypes.c_double), k, c, kh, kw)
    return a


def A_map(I):
    """A = channel mean of |I|, float64 [n][h][w] (sec. 3.2)."""
    I = np.ascontiguousarray(I, dtype=np.float32)
    n, c, h, w = I.shape
    A = np.empty((n, h, w), dtype=np.float64)
    _load().xo_A(_p(I, ctypes.c_float), _p(A, ctypes.c_double), n, c, h, w)
    return A


def K_map(A, kh, kw, stride=(1, 1), pad=(0, 0)):
    """K = A box-filtered by 1/(kh*kw) at the conv's output positions, float64 (sec. 3.2)."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    n, h, w = A.shape
    ho, wo = out_hw(h, w, kh, kw, stride, pad)
    K = np.empty((n, ho, wo), dtype=np.float64)
    _load().xo_K(_p(A, ctypes.c_double), _p(K, ctypes.c_double), n, h, w, kh, kw,
                 stride[0], stride[1], pad[0], pad[1])
    return K


def dot_map(sI, sW, stride=(1, 1), pad=(0, 0)):
    """Exact int32 correlation of +-1 tensors with zero padding (what XNOR+bitcount reaches)."""
    sI = np.ascontiguousarray(sI, dtype=np.int8)
    sW = np.ascontiguousarray(sW, dtype=np.int8)
    n, c, h, w = sI.shape
    k, c2, kh, kw = sW.shape
    assert c == c2
    ho, wo = out_hw(h, w, kh, kw, stride, pad)
    d = np.empty((n, k, ho, wo), dtype=np.int32)
    _load().xo_dot(_p(sI, ctypes.c_int8), _p(sW, ctypes.c_int8), _p(d, ctypes.c_int32),
                   n, c, h, w, k, kh, kw, stride[0], stride[1], pad[0], pad[1])
    return d


def scale_output(dot, K, alpha_):
    """out = float32(dot * K * alpha) (right-hand side of the binary-convolution equation)."""
    dot = np.ascontiguousarray(dot, dtype=np.int32)
    K = np.ascontiguousarray(K, dtype=np.float64)
    alpha_ = np.ascontiguousarray(alpha_, dtype=np.float64)
    n, k, ho, wo = dot.shape
    assert K.shape == (n, ho, wo) and alpha_.shape == (k,)
    out = np.empty(dot.shape, dtype=np.float32)
    _load().xo_scale(_p(dot, ctypes.c_int32), _p(K, ctypes.c_double), _p(alpha_, ctypes.c_double),
                     _p(out, ctypes.c_float), n, k, ho, wo)
    return out


def binary_conv2d(x, W, stride=(1, 1), pad=(0, 0), bn_scale=None, bn_shift=None):
    """Whole block BatchNorm -> BinActiv -> BinConv.  Returns dict(dot, K, alpha, out, y)."""
    y = batchnorm(x, bn_scale, bn_shift)
    W = np.ascontiguousarray(W, dtype=np.float32)
    kh, kw = W.shape[2], W.shape[3]
    d = dot_map(sign(y), sign(W), stride, pad)
    K = K_map(A_map(y), kh, kw, stride, pad)
    a = alpha(W)
    return {"dot": d, "K": K, "alpha": a, "out": scale_output(d, K, a), "y": y}


def binactiv(x, bn_scale=None, bn_shift=None):
    """BatchNorm -> BinActiv of one block on a real tensor x [n][c][h][w] (block order of sec. 3.2):
    returns (y, sign(y) as int8 +-1, A = channel mean of |y| in float64).  Applied to the float
    output of a BinConv with the NEXT block's normalisation it is the definition of what the
    library's fused convolution epilogue emits."""
    y = batchnorm(x, bn_scale, bn_shift)
    return y, sign(y), A_map(y)


def max_pool(x, pool, stride, pad=(0, 0), relu=False):
    """Max-pooling of a real tensor x [n][c][h][w] (the Pool layer that follows BinConv in the block order
    of sec. 3.2), optionally followed by max(., 0) (the optional ReLU of the same section).  Window
    positions outside the image are skipped; the maximum starts at -inf and only a greater value
    replaces it, so NaN inputs are skipped.  Output extent floor((h + 2*pad - pool)/stride) + 1."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    n, c, h, w = x.shape
    (ph, pw), (sh, sw), (qh, qw) = pool, stride, pad
    ho, wo = (h + 2 * qh - ph) // sh + 1, (w + 2 * qw - pw) // sw + 1
    out = np.empty((n, c, ho, wo), dtype=np.float32)
    for oy in range(ho):
        y0, y1 = max(oy * sh - qh, 0), min(oy * sh - qh + ph, h)
        for ox in range(wo):
            x0, x1 = max(ox * sw - qw, 0), min(ox * sw - qw + pw, w)
            win = x[:, :, y0:y1, x0:x1].reshape(n, c, -1)
            out[:, :, oy, ox] = np.fmax.reduce(win, axis=2, initial=-np.inf)
    if relu:
        out = np.where(out > 0, out, np.float32(0.0)).astype(np.float32)
    return out


def bwn_conv2d(x, W, stride=(1, 1), pad=(0, 0)):
    """Binary-Weight-Network convolution (sec. 3.1): real input x, weights alpha_k * sign(W_k):
    out = alpha_k * sum I * sign(W) over the in-bounds window (float64 sums, rounded once)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    n, c, h, w = x.shape
    k, c2, kh, kw = W.shape
    assert c == c2
    ho, wo = out_hw(h, w, kh, kw, stride, pad)
    sW = sign(W)
    a = alpha(W)
    out = np.empty((n, k, ho, wo), dtype=np.float32)
    _load().xo_bwn(_p(x, ctypes.c_float), _p(sW, ctypes.c_int8), _p(a, ctypes.c_double), _p(out, ctypes.c_float),
                   n, c, h, w, k, kh, kw, stride[0], stride[1], pad[0], pad[1])
    return {"out": out, "alpha": a}


def binary_grad_input(g_out, W, K=None, alpha_=None, stride=(1, 1), pad=(0, 0), in_hw=None):
    """Binary-gradient data-gradient convolution (sec. 3.2, "Binary Gradient"): the gradient reaching the
    binary convolution, gd = g_out * alpha_k * K (float32 products), is replaced by max|gd| * sign(gd)
    (one maximum per image) and convolved with sign(W) by the transpose of the forward correlation.
    g_out [n][k][ho][wo], W [k][c][kh][kw], K [n][ho][wo] or None, alpha_ [k] or None; in_hw = (h, w) of the
    forward input (default: the smallest input that gives ho x wo).
    Returns dict(sg int8, gmax float32 [n], dot int32 [n][c][h][w], gin float32 [n][c][h][w])."""
    g_out = np.ascontiguousarray(g_out, dtype=np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    n, k, ho, wo = g_out.shape
    k2, c, kh, kw = W.shape
    assert k == k2
    if in_hw is None:
        in_hw = ((ho - 1) * stride[0] + kh - 2 * pad[0], (wo - 1) * stride[1] + kw - 2 * pad[1])
    h, w = in_hw
    assert out_hw(h, w, kh, kw, stride, pad) == (ho, wo)
    Kf = None if K is None else np.ascontiguousarray(K, dtype=np.float32)
    af = None if alpha_ is None else np.ascontiguousarray(alpha_, dtype=np.float32)
    sW = sign(W)
    sg = np.empty(g_out.shape, dtype=np.int8)
    gmax = np.empty((n,), dtype=np.float32)
    dot = np.empty((n, c, h, w), dtype=np.int32)
    gin = np.empty((n, c, h, w), dtype=np.float32)
    _load().xo_bingrad(_p(g_out, ctypes.c_float), _p(Kf, ctypes.c_float), _p(af, ctypes.c_float),
                       _p(sW, ctypes.c_int8), _p(sg, ctypes.c_int8), _p(gmax, ctypes.c_float),
                       _p(dot, ctypes.c_int32), _p(gin, ctypes.c_float),
                       n, c, h, w, k, kh, kw, stride[0], stride[1], pad[0], pad[1])
    return {"sg": sg, "gmax": gmax, "dot": dot, "gin": gin}


def qk_levels(x, k):
    """Numerators a = 2u - L (odd integers in [-L, L], L = 2^k - 1) of q_k(x) = a / L (sec. 3.2, "k-bit
    Quantization"); inputs clamped to [-1, 1], halves rounded up, level decided in float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    a = np.empty(x.shape, dtype=np.int32)
    _load().xo_qk_levels(_p(x, ctypes.c_float), _p(a, ctypes.c_int32), ctypes.c_size_t(x.size), int(k))
    return a


def kbit_conv2d(x, W, ka, kw_bits, stride=(1, 1), pad=(0, 0)):
    """Correlation of q_ka(x) with q_kw(W) (both in [-1, 1]; sec. 3.2, "k-bit Quantization"), zero padding.
    Returns dict(num int64 = sum of numerator products, out float32 = num / (La * Lw))."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    n, c, h, w = x.shape
    k, c2, kh, kw = W.shape
    assert c == c2
    ho, wo = out_hw(h, w, kh, kw, stride, pad)
    ax, aw = qk_levels(x, ka), qk_levels(W, kw_bits)
    num = np.empty((n, k, ho, wo), dtype=np.int64)
    _load().xo_kbit_dot(_p(ax, ctypes.c_int32), _p(aw, ctypes.c_int32), _p(num, ctypes.c_int64),
                        n, c, h, w, k, kh, kw, stride[0], stride[1], pad[0], pad[1])
    La, Lw = (1 << ka) - 1, (1 << kw_bits) - 1
    return {"num": num, "out": (num.astype(np.float64) / (La * Lw)).astype(np.float32)}


def binary_linear(x, W):
    """Fully connected layer as the convolution whose filter covers the whole input
    (footnote of sec. 1): x [batch][in_f], W [out_f][in_f].  Returns dict(dot, K, alpha, out)
    with dot/out [batch][out_f], K [batch]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    b, f = x.shape
    o, f2 = W.shape
    assert f == f2
    r = binary_conv2d(x.reshape(b, f, 1, 1), W.reshape(o, f, 1, 1))
    return {"dot": r["dot"].reshape(b, o), "K": r["K"].reshape(b), "alpha": r["alpha"],
            "out": r["out"].reshape(b, o)}


def threads():
    """Number of OpenMP threads xo_dot uses."""
    lib = ctypes.CDLL("libgomp.so.1")
    return int(lib.omp_get_max_threads())
