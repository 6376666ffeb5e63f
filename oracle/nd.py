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


def maxpool_sk3d(x, k, d=1, s=1, want_argmax=False):
    """Y[c,z,y,x] = max_{a,i,j<k} X[c, s*z+a*d, s*y+i*d, s*x+j*d].  With want_argmax also the flat offset
    ((z_in*H + y_in)*W + x_in) of the winning sample inside its map's input volume; taps are scanned in the
    order (a, i, j) and only a strictly greater value replaces the incumbent: the first maximum wins."""
    x = np.asarray(x, dtype=np.float64)
    c, D, H, W = x.shape
    ext = (k - 1) * d + 1
    if min(D, H, W) < ext:
        raise ValueError("volume smaller than the external kernel size (k-1)*d+1")
    Do, Ho, Wo = (D - ext) // s + 1, (H - ext) // s + 1, (W - ext) // s + 1
    y = np.full((c, Do, Ho, Wo), -np.inf)
    arg = np.zeros((c, Do, Ho, Wo), dtype=np.int64)
    zz, yy, xx = np.meshgrid(np.arange(Do) * s, np.arange(Ho) * s, np.arange(Wo) * s, indexing="ij")
    for a in range(k):
        for i in range(k):
            for j in range(k):
                window = x[:, a * d:a * d + s * (Do - 1) + 1:s, i * d:i * d + s * (Ho - 1) + 1:s,
                           j * d:j * d + s * (Wo - 1) + 1:s]
                better = window > y
                y = np.where(better, window, y)
                arg = np.where(better, (((zz + a * d) * H + yy + i * d) * W + xx + j * d)[None], arg)
    return (y, arg) if want_argmax else y


def maxpool3d_bwd(dy, argmax, in_dhw):
    """Every output's gradient goes to the input sample that won its window (summed where windows share one)."""
    dy = np.asarray(dy, dtype=np.float64)
    c = dy.shape[0]
    D, H, W = in_dhw
    dx = np.zeros((c, D * H * W))
    for m in range(c):
        np.add.at(dx[m], argmax[m].ravel(), dy[m].ravel())
    return dx.reshape(c, D, H, W)


def conv_sk3d_bwd(x, wgt, dy, d=1, need_dx=True):
    """Gradients of conv_sk3d (without its ReLU) for the output gradient dy: each product W[o,c,a,i,j] *
    X[c,z+a*d,y+i*d,x+j*d] of the forward sum sends dy[o,z,y,x] times the other factor to each of its factors.
    Returns (dx, dw, db)."""
    x = np.asarray(x, dtype=np.float64)
    wgt = np.asarray(wgt, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    f_out, f_in, k = wgt.shape[:3]
    _, Do, Ho, Wo = dy.shape
    dx = np.zeros_like(x) if need_dx else None
    dw = np.zeros_like(wgt)
    for a in range(k):
        for i in range(k):
            for j in range(k):
                sl = (slice(None), slice(a * d, a * d + Do), slice(i * d, i * d + Ho), slice(j * d, j * d + Wo))
                dw[:, :, a, i, j] = np.tensordot(dy, x[sl], axes=([1, 2, 3], [1, 2, 3]))
                if need_dx:
                    dx[sl] += np.tensordot(wgt[:, :, a, i, j], dy, axes=([0], [0]))
    return dx, dw, dy.sum(axis=(1, 2, 3))


def softmax3d(z):
    """Per-voxel softmax over the maps of z[c, D, H, W]."""
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max(axis=0, keepdims=True))
    return e / e.sum(axis=0, keepdims=True)


def sknet3d_forward(volume, sk_layers, weights, biases, keep=False):
    """volume[c, D, H, W] (context included) -> class probabilities [classes, D-v, H-v, W-v] for an SK net
    whose layers (the dictionaries of the 2-D nets: type, f_out, k, d, s, relu) act on three axes.
    keep=True also returns every layer's output and the pools' winners (for parity and for backward)."""
    x = np.asarray(volume, dtype=np.float64)
    acts, argmaxes, wi = [x], [], 0
    for lay in sk_layers:
        if lay["type"] == "conv":
            x = conv_sk3d(x, weights[wi], biases[wi], lay["d"], lay.get("relu", False))
            wi += 1
            argmaxes.append(None)
        elif lay["type"] == "pool":
            x, am = maxpool_sk3d(x, lay["k"], lay["d"], lay.get("s", 1), want_argmax=True)
            argmaxes.append(am)
        else:
            raise ValueError(lay["type"])
        acts.append(x)
    prob = softmax3d(x)
    return (prob, acts, argmaxes) if keep else prob


def softmax_loss3d(z, labels):
    """Mean of -log p_label over the labelled voxels of z[c, D, H, W] (Section 4.3: summed over the error
    volume, then normalised); a label of -1 masks a voxel (Section 4.2).  Returns (loss, dz)."""
    z = np.asarray(z, dtype=np.float64)
    labels = np.asarray(labels)
    keep = labels >= 0
    count = int(keep.sum())
    if count == 0:
        return 0.0, np.zeros_like(z)
    p = softmax3d(z)
    lab = np.where(keep, labels, 0)
    picked = np.take_along_axis(p, lab[None], axis=0)[0]
    loss = -np.log(picked[keep]).sum() / count
    onehot = np.zeros_like(z)
    np.put_along_axis(onehot, lab[None], 1.0, axis=0)
    dz = (p - onehot) * keep[None] / count
    return float(loss), dz


def sknet3d_backward(sk_layers, weights, acts, argmaxes, labels):
    """Loss and its exact gradient for every conv weight and bias: the layers of sknet3d_forward in reverse.
    A ReLU passes gradient where its output is > 0.  Returns (loss, dws, dbs)."""
    loss, g = softmax_loss3d(acts[-1], labels)
    n_conv = sum(1 for lay in sk_layers if lay["type"] == "conv")
    dws, dbs, wi = [None] * n_conv, [None] * n_conv, n_conv
    for li in range(len(sk_layers) - 1, -1, -1):
        lay = sk_layers[li]
        if lay["type"] == "conv":
            wi -= 1
            if lay.get("relu", False):
                g = g * (acts[li + 1] > 0)
            g, dws[wi], dbs[wi] = conv_sk3d_bwd(acts[li], weights[wi], g, lay["d"], need_dx=li > 0)
        else:
            g = maxpool3d_bwd(g, argmaxes[li], acts[li].shape[1:])
    return loss, dws, dbs
