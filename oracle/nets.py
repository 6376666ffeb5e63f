"""Whole-network oracle: SK-Net forward / backward / SGD and U-Net forward, composed from the
layer functions in oracle/layers.py in the order the paper's tables list them.
TEST INFRASTRUCTURE ONLY.
"""
import numpy as np

from . import layers as L
from .alg1 import context


def pad_amounts(v):
    """Split the context v over the borders: ceil(v/2) top/left, floor(v/2) bottom/right
    (Section 3.3.2: an odd v is handled by a one-pixel crop on the bottom and right)."""
    return (v + 1) // 2, (v + 1) // 2, v // 2, v // 2


def sknet_forward(image, sk_layers, weights, biases, pad=True, pad_mode=0, keep=False):
    """image[n,c,h,w] -> class probabilities [n,classes,h,w] (pad=True) for an SK net
    (laid out like the SK network configuration table of Section 3.3.2: conv SK + ReLU, max pool SK, ..., conv, softmax).
    keep=True also returns every intermediate (for per-layer parity and for backward)."""
    x = np.asarray(image, dtype=np.float64)
    if pad:
        t, l, b, r = pad_amounts(context(sk_layers))
        x = L.mirror_pad(x, t, l, b, r, pad_mode)
    acts, argmaxes = [x], []
    wi = 0
    for lay in sk_layers:
        if lay["type"] == "conv":
            x = L.conv_sk(x, weights[wi], biases[wi], lay["d"], lay.get("relu", False))
            wi += 1
            argmaxes.append(None)
        elif lay["type"] == "pool":
            x, am = L.maxpool_sk(x, lay["k"], lay["d"], lay.get("s", 1))
            argmaxes.append(am)
        else:
            raise ValueError(lay["type"])
        acts.append(x)
    prob = L.softmax(x)
    if keep:
        return prob, acts, argmaxes
    return prob


def sknet_backward(sk_layers, weights, acts, argmaxes, labels, diffs=None):
    """Exact gradient of the mean softmax loss w.r.t. every conv weight and bias.
    acts/argmaxes come from sknet_forward(keep=True).  Returns (loss, dW list, db list, d_input).
    diffs: an optional list that receives, per layer, the error map of that layer (the gradient of the
    loss with respect to its output, after the layer's own ReLU derivative)."""
    loss, g = L.softmax_loss(acts[-1], labels)
    if diffs is not None:
        diffs[:] = [None] * len(sk_layers)
    conv_ids = [i for i, l in enumerate(sk_layers) if l["type"] == "conv"]
    dws, dbs = [None] * len(conv_ids), [None] * len(conv_ids)
    wi = len(conv_ids) - 1
    for li in range(len(sk_layers) - 1, -1, -1):
        lay = sk_layers[li]
        x_in, y_out = acts[li], acts[li + 1]
        if lay["type"] == "conv":
            if lay.get("relu", False):
                g = L.relu_bwd(y_out, g)
            if diffs is not None:
                diffs[li] = g
            dws[wi], dbs[wi] = L.conv_sk_bwd_weights(x_in, g, lay["k"], lay["d"])
            g = L.conv_sk_bwd_data(g, weights[wi], lay["d"], x_in.shape[2:])
            wi -= 1
        else:
            if diffs is not None:
                diffs[li] = g
            g = L.maxpool_bwd(g, argmaxes[li], x_in.shape[2:])
    return loss, dws, dbs, g


def sgd_step(weights, biases, dws, dbs, lr, momentum=0.0, weight_decay=0.0, vel_w=None, vel_b=None):
    for i in range(len(weights)):
        L.sgd(weights[i], dws[i], None if vel_w is None else vel_w[i], lr, momentum, weight_decay)
        L.sgd(biases[i], dbs[i], None if vel_b is None else vel_b[i], lr, momentum, weight_decay)


# ---------------------------------------------------------------------------------------------
# U-Net (Section 3.4, the U network configuration table)

def unet_spec(depth=4, base=64):
    """Per-level channel counts of the U-Net table: 64,128,256,512 down, 1024 at the bottom."""
    return [base * 2 ** i for i in range(depth + 1)]


def unet_forward(image, params, depth=4, keep=False):
    """image[n,c,h,w] (already context-padded, e.g. 572) -> probabilities (e.g. 388).

    params is a dict of (weight, bias) pairs, in table order:
      "down{i}a", "down{i}b"  i = 0..depth   3x3 conv + ReLU (level `depth` is the bottom)
      "up{i}"                 i = depth-1..0 2x2 stride-2 up-convolution f -> f/2, no ReLU,
                                             weight [f, f/2, 2, 2]
      "dec{i}a", "dec{i}b"    3x3 conv + ReLU on mergecrop(up path, skip)
      "head"                  1x1 conv to the classes
    The paper's up step (fixed nearest-neighbour grouped deconvolution, then a 1x1 conv f -> f/2
    without ReLU) is the special case weight[c,o,a,b] = W1x1[o,c]; see upstep_from_paper().
    """
    x = np.asarray(image, dtype=np.float64)
    skips, trace = [], {}
    for i in range(depth + 1):
        x = L.conv_sk(x, *params["down%da" % i], d=1, relu=True)
        x = L.conv_sk(x, *params["down%db" % i], d=1, relu=True)
        trace["down%d" % i] = x
        if i < depth:
            skips.append(x)
            if x.shape[2] % 2 or x.shape[3] % 2:
                raise ValueError("U-Net pooling needs an even map size")
            x, _ = L.maxpool_sk(x, 2, 1, 2)
    for i in range(depth - 1, -1, -1):
        x = L.upconv2x2(x, *params["up%d" % i])
        trace["up%d" % i] = x
        x = L.mergecrop(x, skips[i])
        x = L.conv_sk(x, *params["dec%da" % i], d=1, relu=True)
        x = L.conv_sk(x, *params["dec%db" % i], d=1, relu=True)
        trace["dec%d" % i] = x
    z = L.conv_sk(x, *params["head"], d=1, relu=False)
    trace["logits"] = z
    prob = L.softmax(z)
    return (prob, trace) if keep else prob


def upstep_from_paper(w1x1):
    """Fold the paper's two-layer up step (nearest-neighbour 2x2 up-sampling of every map, then a
    1x1 convolution w1x1[o,c,1,1]) into one up-convolution weight [c,o,2,2]."""
    o, c = w1x1.shape[:2]
    return np.broadcast_to(w1x1.reshape(o, c).T[:, :, None, None], (c, o, 2, 2)).copy()


# ---------------------------------------------------------------------------------------------
# USK-Net (Section 3.5, the USK network configuration table): one contracting step of the U-Net,
# the SK layer sequence on the half-resolution maps, one expanding step.

def usknet_core(base=64):
    """The SK part of the USK table (conv3 .. ip2) as (kind, f_out, k, d, relu) rows; it sees a
    context of 5 + 1 + 6 + 2 + 12 + 4 + 56 = 86 pixels of the half-resolution map."""
    return [("conv", 2 * base, 6, 1, True), ("pool", 0, 2, 1, False),
            ("conv", 2 * base, 4, 2, True), ("pool", 0, 2, 2, False),
            ("conv", 2 * base, 4, 4, True), ("pool", 0, 2, 4, False),
            ("conv", 8 * base, 8, 8, True),              # ip1
            ("conv", 4 * base, 1, 1, True)]              # ip2


USK_CORE_NAMES = ("conv3", "pool2", "conv4", "pool3", "conv5", "pool4", "ip1", "ip2")


def usknet_forward(image, params, base=64, keep=False):
    """image[n,c,h,w] (context-padded, 692 in the table) -> probabilities (512 in the table).

    params: {"conv1", "conv2"}   3x3 conv + ReLU (U part, full resolution)
            {"conv3", "conv4", "conv5", "ip1", "ip2"}   SK convolutions + ReLU of usknet_core()
            "up1"                2x2 stride-2 up-convolution 4*base -> 2*base, no ReLU, weight
                                 [4*base, 2*base, 2, 2] (the table's upconv1 + conv6 pair is the
                                 special case of upstep_from_paper())
            {"conv7", "conv8"}   3x3 conv + ReLU on mergecrop(up path, conv2's maps)
            "ip3"                1x1 conv to the classes
    The max-pool between the parts is k = s = 2; the SK pools are k = 2, stride 1, at the layer's d.
    """
    x = np.asarray(image, dtype=np.float64)
    trace = {}
    x = L.conv_sk(x, *params["conv1"], d=1, relu=True)
    x = L.conv_sk(x, *params["conv2"], d=1, relu=True)
    trace["conv2"] = skip = x
    if x.shape[2] % 2 or x.shape[3] % 2:
        raise ValueError("USK-Net pooling needs an even map size")
    x, _ = L.maxpool_sk(x, 2, 1, 2)
    trace["pool1"] = x
    for name, (kind, _, k, d, relu) in zip(USK_CORE_NAMES, usknet_core(base)):
        if kind == "conv":
            x = L.conv_sk(x, *params[name], d=d, relu=relu)
        else:
            x, _ = L.maxpool_sk(x, k, d, 1)
        trace[name] = x
    x = L.upconv2x2(x, *params["up1"])
    trace["up1"] = x
    x = L.mergecrop(x, skip)
    x = L.conv_sk(x, *params["conv7"], d=1, relu=True)
    x = L.conv_sk(x, *params["conv8"], d=1, relu=True)
    trace["conv8"] = x
    z = L.conv_sk(x, *params["ip3"], d=1, relu=False)
    trace["logits"] = z
    prob = L.softmax(z)
    return (prob, trace) if keep else prob


# ---------------------------------------------------------------------------------------------
# Training pass of the U-Net and the USK-Net: the exact gradient of the (optionally masked) mean
# softmax loss with respect to every parameter, the layers' own backward rules applied in reverse
# order.  The skip map feeds two layers, the pool and MergeCrop.  Section 5.3.1 enables MergeCrop's
# backward for its input A (the up path) only: the skip map then takes its gradient from the pool
# alone (merge_into_b=False, the section's rule).  merge_into_b=True is the exact derivative of the
# composite instead: MergeCrop also copies its skip maps' gradient into the centre window of the skip
# map (nothing into the cropped-away border) and the skip map sums both contributions.

def _conv_fwd(x, p, d=1, relu=True):
    return L.conv_sk(x, p[0], p[1], d=d, relu=relu)


def _conv_bwd(x, y, g, p, d=1, relu=True, need_dx=True):
    """Backward of conv (+ReLU): returns (dx or None, (dW, db))."""
    if relu:
        g = L.relu_bwd(y, g)
    k = p[0].shape[2]
    grads = L.conv_sk_bwd_weights(x, g, k, d)
    dx = L.conv_sk_bwd_data(g, p[0], d, x.shape[2:]) if need_dx else None
    return dx, grads


def unet_backward(image, params, labels, depth=4, merge_into_b=False):
    """Returns (loss, {name: (dW, db)}) for the U-Net of unet_forward()."""
    x0 = np.asarray(image, dtype=np.float64)
    tape, skips = [], []
    x = x0
    for i in range(depth + 1):
        a = _conv_fwd(x, params["down%da" % i])
        b = _conv_fwd(a, params["down%db" % i])
        tape.append(("down", i, x, a, b))
        x = b
        if i < depth:
            skips.append(b)
            pooled, am = L.maxpool_sk(b, 2, 1, 2)
            tape.append(("pool", i, b, am))
            x = pooled
    for i in range(depth - 1, -1, -1):
        up = L.upconv2x2(x, *params["up%d" % i])
        m = L.mergecrop(up, skips[i])
        a = _conv_fwd(m, params["dec%da" % i])
        b = _conv_fwd(a, params["dec%db" % i])
        tape.append(("up", i, x, up, m, a, b))
        x = b
    z = _conv_fwd(x, params["head"], relu=False)
    loss, g = L.softmax_loss(z, labels)
    grads = {}
    g, grads["head"] = _conv_bwd(x, z, g, params["head"], relu=False)
    gskip = [None] * depth
    for rec in reversed(tape):
        if rec[0] == "up":
            _, i, xin, up, m, a, b = rec
            g, grads["dec%db" % i] = _conv_bwd(a, b, g, params["dec%db" % i])
            g, grads["dec%da" % i] = _conv_bwd(m, a, g, params["dec%da" % i])
            g, gskip[i] = L.mergecrop_bwd(g, up.shape[1], skips[i].shape, merge_into_b)
            g, dw, db = L.upconv2x2_bwd(xin, params["up%d" % i][0], g)
            grads["up%d" % i] = (dw, db)
        elif rec[0] == "pool":
            _, i, b, am = rec
            g = L.maxpool_bwd(g, am, b.shape[2:]) + gskip[i]
        else:
            _, i, xin, a, b = rec
            g, grads["down%db" % i] = _conv_bwd(a, b, g, params["down%db" % i])
            g, grads["down%da" % i] = _conv_bwd(xin, a, g, params["down%da" % i], need_dx=i > 0)
    return loss, grads


def usknet_backward(image, params, labels, base=64, merge_into_b=False):
    """Returns (loss, {name: (dW, db)}) for the USK-Net of usknet_forward()."""
    x0 = np.asarray(image, dtype=np.float64)
    c1 = _conv_fwd(x0, params["conv1"])
    c2 = _conv_fwd(c1, params["conv2"])
    p1, am1 = L.maxpool_sk(c2, 2, 1, 2)
    core = []                                   # (name, kind, d, input, output, argmax)
    x = p1
    for name, (kind, _, k, d, relu) in zip(USK_CORE_NAMES, usknet_core(base)):
        if kind == "conv":
            y = _conv_fwd(x, params[name], d=d, relu=relu)
            core.append((name, kind, d, x, y, None))
        else:
            y, am = L.maxpool_sk(x, k, d, 1)
            core.append((name, kind, d, x, y, am))
        x = y
    up = L.upconv2x2(x, *params["up1"])
    m = L.mergecrop(up, c2)
    c7 = _conv_fwd(m, params["conv7"])
    c8 = _conv_fwd(c7, params["conv8"])
    z = _conv_fwd(c8, params["ip3"], relu=False)
    loss, g = L.softmax_loss(z, labels)
    grads = {}
    g, grads["ip3"] = _conv_bwd(c8, z, g, params["ip3"], relu=False)
    g, grads["conv8"] = _conv_bwd(c7, c8, g, params["conv8"])
    g, grads["conv7"] = _conv_bwd(m, c7, g, params["conv7"])
    g, gskip = L.mergecrop_bwd(g, up.shape[1], c2.shape, merge_into_b)
    g, dw, db = L.upconv2x2_bwd(x, params["up1"][0], g)
    grads["up1"] = (dw, db)
    for name, kind, d, xin, y, am in reversed(core):
        if kind == "conv":
            g, grads[name] = _conv_bwd(xin, y, g, params[name], d=d)
        else:
            g = L.maxpool_bwd(g, am, xin.shape[2:])
    g = L.maxpool_bwd(g, am1, c2.shape[2:]) + gskip
    g, grads["conv2"] = _conv_bwd(c1, c2, g, params["conv2"])
    _, grads["conv1"] = _conv_bwd(x0, c1, g, params["conv1"], need_dx=False)
    return loss, grads
