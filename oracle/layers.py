"""numpy-facing wrappers of the C oracle (oracle/sk_oracle.c): argument marshalling, plus the
backward rules of the up-convolution and of MergeCrop written out in numpy.

All arrays are fp64, C-contiguous, NCHW.  TEST INFRASTRUCTURE ONLY.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = C.CDLL(_build.build())
_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int32)
L = C.c_long


def _d(a):
    return a.ctypes.data_as(_dp) if a is not None else None


def _i(a):
    return a.ctypes.data_as(_ip) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


_lib.osk_mirror_pad.argtypes = [_dp, L, L, L, L, L, L, L, C.c_int, _dp]
_lib.osk_conv_sk.argtypes = [_dp, L, L, L, L, _dp, _dp, L, L, L, C.c_int, _dp]
_lib.osk_conv_sk_bwd_data.argtypes = [_dp, L, L, L, L, _dp, L, L, L, _dp]
_lib.osk_conv_sk_bwd_weights.argtypes = [_dp, _dp, L, L, L, L, L, L, L, _dp, _dp]
_lib.osk_maxpool_sk.argtypes = [_dp, L, L, L, L, L, L, _dp, _ip]
_lib.osk_maxpool_bwd.argtypes = [_dp, _ip, L, L, L, L, L, _dp]
_lib.osk_relu_bwd.argtypes = [_dp, _dp, L, _dp]
_lib.osk_softmax.argtypes = [_dp, L, L, L, _dp]
_lib.osk_softmax_loss.argtypes = [_dp, _ip, L, L, L, _dp]
_lib.osk_softmax_loss.restype = C.c_double
_lib.osk_upconv2x2.argtypes = [_dp, L, L, L, L, _dp, _dp, L, _dp]
_lib.osk_mergecrop.argtypes = [_dp, L, L, L, L, _dp, L, L, L, _dp]
_lib.osk_sgd.argtypes = [_dp, _dp, _dp, L, C.c_double, C.c_double, C.c_double]

for _f in ("osk_mirror_pad", "osk_conv_sk", "osk_conv_sk_bwd_data", "osk_conv_sk_bwd_weights",
           "osk_maxpool_sk", "osk_maxpool_bwd", "osk_relu_bwd", "osk_softmax", "osk_upconv2x2",
           "osk_mergecrop", "osk_sgd"):
    getattr(_lib, _f).restype = None


_lib.osk_get_num_threads.restype = C.c_int
_lib.osk_set_num_threads.argtypes = [C.c_int]
_lib.osk_set_num_threads.restype = None


def num_threads():
    """Threads the C loops run on (OpenMP's current maximum)."""
    return int(_lib.osk_get_num_threads())


def set_num_threads(n):
    _lib.osk_set_num_threads(int(n))


def mirror_pad(x, top, left, bottom, right, mode=0):
    """Extend every plane of x[n,c,h,w] by mirroring (Section 1.3). mode 0 reflect, 1 symmetric."""
    x = _f64(x)
    n, c, h, w = x.shape
    limit_h, limit_w = (h - 1, w - 1) if mode == 0 else (h, w)
    if max(top, bottom) > limit_h or max(left, right) > limit_w:
        raise ValueError("mirror border larger than the image allows")
    out = np.empty((n, c, h + top + bottom, w + left + right))
    _lib.osk_mirror_pad(_d(x), n * c, h, w, top, left, bottom, right, mode, _d(out))
    return out


def conv_sk(x, wgt, bias=None, d=1, relu=False):
    """SK convolution, Y[o,y,x] = b[o] + sum W[o,c,i,j] X[c,y+i*d,x+j*d] (Section 5.2.1)."""
    x, wgt = _f64(x), _f64(wgt)
    n, f_in, h, w = x.shape
    f_out, f_in2, k, k2 = wgt.shape
    assert f_in == f_in2 and k == k2
    ho, wo = h - (k - 1) * d, w - (k - 1) * d
    if ho < 1 or wo < 1:
        raise ValueError("input smaller than the external kernel size (k-1)*d+1")
    b = _f64(bias) if bias is not None else None
    y = np.empty((n, f_out, ho, wo))
    _lib.osk_conv_sk(_d(x), n, f_in, h, w, _d(wgt), _d(b), f_out, k, d, int(relu), _d(y))
    return y


def conv_sk_bwd_data(dy, wgt, d, in_hw):
    dy, wgt = _f64(dy), _f64(wgt)
    n, f_out, ho, wo = dy.shape
    _, f_in, k, _ = wgt.shape
    h, w = in_hw
    assert ho == h - (k - 1) * d and wo == w - (k - 1) * d
    dx = np.empty((n, f_in, h, w))
    _lib.osk_conv_sk_bwd_data(_d(dy), n, f_in, h, w, _d(wgt), f_out, k, d, _d(dx))
    return dx


def conv_sk_bwd_weights(x, dy, k, d):
    x, dy = _f64(x), _f64(dy)
    n, f_in, h, w = x.shape
    f_out = dy.shape[1]
    assert dy.shape == (n, f_out, h - (k - 1) * d, w - (k - 1) * d)
    dw = np.empty((f_out, f_in, k, k))
    db = np.empty(f_out)
    _lib.osk_conv_sk_bwd_weights(_d(x), _d(dy), n, f_in, h, w, f_out, k, d, _d(dw), _d(db))
    return dw, db


def maxpool_sk(x, k, d=1, s=1):
    """Max pool with kernel stride d and layer stride s; returns (values, argmax flat offsets)."""
    x = _f64(x)
    n, c, h, w = x.shape
    if h < (k - 1) * d + 1 or w < (k - 1) * d + 1:
        raise ValueError("input smaller than the external kernel size (k-1)*d+1")
    ho, wo = (h - (k - 1) * d - 1) // s + 1, (w - (k - 1) * d - 1) // s + 1
    y = np.empty((n, c, ho, wo))
    am = np.empty((n, c, ho, wo), dtype=np.int32)
    _lib.osk_maxpool_sk(_d(x), n * c, h, w, k, d, s, _d(y), _i(am))
    return y, am


def maxpool_bwd(dy, argmax, in_hw):
    dy = _f64(dy)
    argmax = np.ascontiguousarray(argmax, dtype=np.int32)
    n, c, ho, wo = dy.shape
    h, w = in_hw
    dx = np.empty((n, c, h, w))
    _lib.osk_maxpool_bwd(_d(dy), _i(argmax), n * c, h, w, ho, wo, _d(dx))
    return dx


def relu_bwd(y, dy):
    y, dy = _f64(y), _f64(dy)
    dx = np.empty_like(dy)
    _lib.osk_relu_bwd(_d(y), _d(dy), y.size, _d(dx))
    return dx


def softmax(z):
    z = _f64(z)
    n, c, h, w = z.shape
    p = np.empty_like(z)
    _lib.osk_softmax(_d(z), n, c, h * w, _d(p))
    return p


def softmax_loss(z, labels, want_grad=True):
    """Mean of -log p_label over the labelled pixels (Section 4.3); a pixel whose label is -1 is
    masked out of the error map (Section 4.2): no loss, zero gradient, not counted.  Returns (loss, dz)."""
    z = _f64(z)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    n, c, h, w = z.shape
    assert labels.shape == (n, h, w) and labels.min() >= -1 and labels.max() < c
    dz = np.empty_like(z) if want_grad else None
    loss = _lib.osk_softmax_loss(_d(z), _i(labels), n, c, h * w, _d(dz))
    return loss, dz


def upconv2x2(x, wgt, bias=None):
    """2x2 stride-2 up-convolution, wgt[c_in, c_out, 2, 2] (Section 3.4)."""
    x, wgt = _f64(x), _f64(wgt)
    n, f_in, h, w = x.shape
    assert wgt.shape[0] == f_in and wgt.shape[2:] == (2, 2)
    f_out = wgt.shape[1]
    b = _f64(bias) if bias is not None else None
    y = np.empty((n, f_out, 2 * h, 2 * w))
    _lib.osk_upconv2x2(_d(x), n, f_in, h, w, _d(wgt), _d(b), f_out, _d(y))
    return y


def mergecrop(a, b):
    """Maps of A followed by the maps of B centre-cropped to A's size (Section 5.3.1)."""
    a, b = _f64(a), _f64(b)
    n, fa, ha, wa = a.shape
    n2, fb, hb, wb = b.shape
    assert n == n2 and hb >= ha and wb >= wa
    out = np.empty((n, fa + fb, ha, wa))
    _lib.osk_mergecrop(_d(a), n, fa, ha, wa, _d(b), fb, hb, wb, _d(out))
    return out


def upconv2x2_bwd(x, wgt, dy):
    """Gradients of upconv2x2: every output pixel (2y+a, 2x+b) of map o depends on input pixel
    (y, x) of every map c through wgt[c,o,a,b] alone.  Returns (dx, dw, db)."""
    x, wgt, dy = _f64(x), _f64(wgt), _f64(dy)
    n, f_in, h, w = x.shape
    f_out = wgt.shape[1]
    assert dy.shape == (n, f_out, 2 * h, 2 * w)
    dx = np.zeros_like(x)
    dw = np.zeros_like(wgt)
    for a in range(2):
        for b in range(2):
            g = dy[:, :, a::2, b::2]                                   # [n, f_out, h, w]
            dx += np.einsum("co,noyx->ncyx", wgt[:, :, a, b], g)
            dw[:, :, a, b] = np.einsum("ncyx,noyx->co", x, g)
    return dx, dw, dy.sum(axis=(0, 2, 3))


def mergecrop_bwd(g, fa, b_shape, into_b=False):
    """Backward of mergecrop (Section 5.3.1): the error maps are copied back in the inverse direction.
    The first fa maps go to A.  For the U- and USK-Net the section enables backwarding for input A only,
    because B (the skip map) receives its differential on another path, from the down-sampling pool:
    into_b=False returns zeros for B.  into_b=True is the exact derivative of the copy: the rest of
    the maps go to the centre window of B, nothing to the part that was cropped away.
    Returns (dA, dB)."""
    g = _f64(g)
    n, f, ha, wa = g.shape
    _, fb, hb, wb = b_shape
    assert f == fa + fb
    oy, ox = (hb - ha) // 2, (wb - wa) // 2
    db = np.zeros(b_shape)
    if into_b:
        db[:, :, oy:oy + ha, ox:ox + wa] = g[:, fa:]
    return g[:, :fa].copy(), db


def sgd(wgt, dw, vel, lr, momentum=0.0, weight_decay=0.0):
    """In place: g = dW + wd*W; V = mu*V + lr*g; W -= V.  vel may be None (mu = 0)."""
    assert wgt.dtype == np.float64 and wgt.flags.c_contiguous
    dw = _f64(dw)
    _lib.osk_sgd(_d(wgt), _d(dw), _d(vel), wgt.size, lr, momentum, weight_decay)
    return wgt
