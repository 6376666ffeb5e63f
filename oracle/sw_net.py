"""Sliding-window network (Section 3.2) evaluated patch by patch: the plain definition that an
SK net must reproduce at every pixel (Sections 1.3 and 3.3.1).  Pure numpy, written separately
from the C oracle on purpose: it uses ordinary (d = 1) convolution, ordinary k = s pooling on
windows aligned to the patch origin, and an inner product over the whole remaining map.
TEST INFRASTRUCTURE ONLY.
"""
import numpy as np


def _conv_valid(x, wgt, bias):
    """x[c,h,w], wgt[o,c,k,k] -> y[o,h-k+1,w-k+1], cross-correlation."""
    f_out, f_in, k, _ = wgt.shape
    ho, wo = x.shape[1] - k + 1, x.shape[2] - k + 1
    y = np.zeros((f_out, ho, wo))
    for yy in range(ho):
        for xx in range(wo):
            y[:, yy, xx] = np.tensordot(wgt, x[:, yy:yy + k, xx:xx + k], axes=3)
    return y + bias[:, None, None]


def _pool_down(x, k):
    """k = s max pooling; the map side must be a multiple of k (Algorithm 1's check)."""
    c, h, w = x.shape
    assert h % k == 0 and w % k == 0
    return x.reshape(c, h // k, k, w // k, k).max(axis=(2, 4))


def sw_forward_patch(patch, sw_layers, weights, biases, softmax=True):
    """Run one (w_SW x w_SW) patch through the SW net; returns the class vector.
    weights[i] for a conv is [o,c,k,k]; for an inner product it is [o,c,kh,kw] with
    (kh,kw) = the remaining map (the same numbers the converted SK conv uses)."""
    x = np.asarray(patch, dtype=np.float64)
    wi = 0
    for l in sw_layers:
        if l["type"] == "conv":
            x = _conv_valid(x, weights[wi], biases[wi])
            if l.get("relu"):
                x = np.maximum(x, 0.0)
            wi += 1
        elif l["type"] == "pool":
            assert l["k"] == l["s"]
            x = _pool_down(x, l["k"])
        elif l["type"] == "ip":
            wgt = weights[wi]
            assert wgt.shape[1:] == x.shape, (wgt.shape, x.shape)
            x = (np.tensordot(wgt, x, axes=3) + biases[wi])[:, None, None]
            if l.get("relu"):
                x = np.maximum(x, 0.0)
            wi += 1
        else:
            raise ValueError(l["type"])
    z = x.reshape(-1)
    if not softmax:
        return z
    e = np.exp(z - z.max())
    return e / e.sum()


def sw_forward_image(padded, sw_layers, w0_sw, weights, biases, softmax=True):
    """Slide the patch over a padded image [c, H+w0-1, W+w0-1]; returns [classes, H, W]."""
    c, hp, wp = padded.shape
    h, w = hp - w0_sw + 1, wp - w0_sw + 1
    out = None
    for y in range(h):
        for x in range(w):
            v = sw_forward_patch(padded[:, y:y + w0_sw, x:x + w0_sw], sw_layers, weights, biases,
                                 softmax)
            if out is None:
                out = np.empty((v.size, h, w))
            out[:, y, x] = v
    return out
