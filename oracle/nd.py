"""Three-dimensional SK layers and a 3-D SK net forward (Section 5.2.2: the N-dimensional forms of the
kernel-strided convolution and max pool; three dimensions is the case built here), in fp64 numpy.
TEST INFRASTRUCTURE ONLY.

A volume is x[c, D, H, W].  Both layers are the 2-D definitions of Section 5.2.1 with one more spatial
index: the kernel stride d is the same along the three axes, nothing is padded, and every layer shrinks
each axis by (k-1)*d (Algorithm 1's rule, which holds per axis).
"""
import numpy as np


def conv_sk3d(x, wgt, bias=None, d=1, relu=False):
    """Y[o,z,y,x] = b[o] + sum_{c,a,i,j} W[o,c,a,i,j] X[c, z+a*d, y+i*d, x+j*d]  (cross-correlation)."""
    x = np.asarray(x, dtype=np.float64)
    wgt = np.asarray(wgt, dtype=np.float64)
    f_in, D, H, W = x.shape
    f_out, f_in2, k, k2, k3 = wgt.shape
    assert f_in == f_in2 and k == k2 == k3
    Do, Ho, Wo = D - (k - 1) * d, H - (k - 1) * d, W - (k - 1) * d
    if min(Do, Ho, Wo) < 1:
        raise ValueError("volume smaller than the external kernel size (k-1)*d+1")
    y = np.zeros((f_out, Do, Ho, Wo))
    for a in range(k):
        for i in range(k):
            for j in range(k):
                window = x[:, a * d:a * d + Do, i * d:i * d + Ho, j * d:j * d + Wo]
                y += np.tensordot(wgt[:, :, a, i, j], window, axes=([1], [0]))
    if bias is not None:
        y += np.asarray(bias, dtype=np.float64)[:, None, None, None]
    if relu:
        y = np.maximum(y, 0.0)
    return y


def maxpool_sk3d(x, k, d=1, s=1):
    """Y[c,z,y,x] = max_{a,i,j<k} X[c, s*z+a*d, s*y+i*d, s*x+j*d]."""
    x = np.asarray(x, dtype=np.float64)
    c, D, H, W = x.shape
    ext = (k - 1) * d + 1
    if min(D, H, W) < ext:
        raise ValueError("volume smaller than the external kernel size (k-1)*d+1")
    Do, Ho, Wo = (D - ext) // s + 1, (H - ext) // s + 1, (W - ext) // s + 1
    y = np.full((c, Do, Ho, Wo), -np.inf)
    for a in range(k):
        for i in range(k):
            for j in range(k):
                window = x[:, a * d:a * d + s * (Do - 1) + 1:s, i * d:i * d + s * (Ho - 1) + 1:s,
                           j * d:j * d + s * (Wo - 1) + 1:s]
                y = np.maximum(y, window)
    return y


def softmax3d(z):
    """Per-voxel softmax over the maps of z[c, D, H, W]."""
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max(axis=0, keepdims=True))
    return e / e.sum(axis=0, keepdims=True)


def sknet3d_forward(volume, sk_layers, weights, biases, keep=False):
    """volume[c, D, H, W] (context included) -> class probabilities [classes, D-v, H-v, W-v] for an SK net
    whose layers (the dictionaries of the 2-D nets: type, f_out, k, d, s, relu) act on three axes."""
    x = np.asarray(volume, dtype=np.float64)
    acts, wi = [x], 0
    for lay in sk_layers:
        if lay["type"] == "conv":
            x = conv_sk3d(x, weights[wi], biases[wi], lay["d"], lay.get("relu", False))
            wi += 1
        elif lay["type"] == "pool":
            x = maxpool_sk3d(x, lay["k"], lay["d"], lay.get("s", 1))
        else:
            raise ValueError(lay["type"])
        acts.append(x)
    prob = softmax3d(x)
    return (prob, acts) if keep else prob
