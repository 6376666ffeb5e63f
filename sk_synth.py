"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only random images, labels, weights and the layer lists of
the benchmark configurations.  The GPU binding and the CPU oracle are both fed from here and
neither imports the other.

The images stand in for the electron-microscopy data of Chapter 2 (ssTEM 1024^2 and ISBI-2012
512^2 sections: textured cell interior crossed by dark membranes, about a fifth of the pixels
membrane); none of that data is reproduced.
"""
import numpy as np
from scipy import ndimage


def conv(f_out, k, d=1, relu=True):
    return {"type": "conv", "f_out": f_out, "k": k, "d": d, "relu": relu}


def pool(k, d=1, s=1):
    return {"type": "pool", "k": k, "d": d, "s": s}


def tiny_sknet_layers():
    """Config C1: conv 1->8 k4 d1, pool k2 d1, conv 8->16 k5 d2, pool k2 d2, 1x1 16->32, 1x1 32->2."""
    return [conv(8, 4, 1), pool(2, 1), conv(16, 5, 2), pool(2, 2), conv(32, 1, 1), conv(2, 1, 1, relu=False)]


def tiny_sw_layers():
    """The sliding-window net whose Algorithm-1 conversion is tiny_sknet_layers(); patch 15."""
    return [{"type": "conv", "f_out": 8, "k": 4, "relu": True}, {"type": "pool", "k": 2, "s": 2},
            {"type": "conv", "f_out": 16, "k": 5, "relu": True}, {"type": "pool", "k": 2, "s": 2},
            {"type": "ip", "f_out": 32, "relu": True}, {"type": "ip", "f_out": 2, "relu": False}]


def sknet_layers(width=48, hidden=200, classes=2, stages=4):
    """Configs C2-C4: `stages` x [conv k4 -> width + ReLU, pool k2 s1] with d = 1,2,4,8, then
    1x1 width->hidden + ReLU, 1x1 hidden->classes."""
    layers = []
    for s in range(stages):
        layers += [conv(width, 4, 2 ** s), pool(2, 2 ** s)]
    layers += [conv(hidden, 1, 1), conv(classes, 1, 1, relu=False)]
    return layers


def paper_sknet_layers(classes=2):
    """The SK network of Section 3.3.2's configuration table (3 input maps, context 101):
    conv k7 -> 48, pool, conv k5 d2 -> 128, pool d2, conv k3 d4 -> 192, pool d4, then the three
    inner-product layers as convolutions: k10 d8 -> 1024, 1x1 -> 512, 1x1 -> classes."""
    return [conv(48, 7, 1), pool(2, 1), conv(128, 5, 2), pool(2, 2), conv(192, 3, 4), pool(2, 4),
            conv(1024, 10, 8), conv(512, 1, 1), conv(classes, 1, 1, relu=False)]


def he_normal_weights(layers, c_in, seed, bias_scale=0.0):
    """Per conv, in order: N(0, sqrt(2/(f_in k^2))) weights [f_out,f_in,k,k] (Section 3.4's
    initialisation), biases bias_scale*N(0,1) (0 in the benchmark configs). fp32."""
    rng = np.random.default_rng(seed)
    ws, bs, f_in = [], [], c_in
    for l in layers:
        if l["type"] != "conv":
            continue
        k, f_out = l["k"], l["f_out"]
        w = rng.standard_normal((f_out, f_in, k, k)) * np.sqrt(2.0 / (f_in * k * k))
        b = rng.standard_normal(f_out) * bias_scale
        ws.append(w.astype(np.float32))
        bs.append(b.astype(np.float32))
        f_in = f_out
    return ws, bs


def sknet3d_layers(classes=2, maps=(16, 32, 128, 64)):
    """A 3-D SK net in the manner of Section 5.2.2 (the 2-D layer sequence with 3-D kernels and fewer maps,
    sized for memory): the Algorithm-1 conversion of the sliding-window net conv k3, pool 2, conv k3, pool 2,
    inner product, inner product, classes on an 18^3 patch.  Context 17 per axis."""
    a, b, c, e = maps
    return [conv(a, 3, 1), pool(2, 1), conv(b, 3, 2), pool(2, 2), conv(c, 3, 4), conv(e, 1, 1),
            conv(classes, 1, 1, relu=False)]


def sw3d_layers(classes=2, maps=(16, 32, 128, 64)):
    """The sliding-window net that sknet3d_layers() converts; patch 18 per axis."""
    a, b, c, e = maps
    return [{"type": "conv", "f_out": a, "k": 3, "relu": True}, {"type": "pool", "k": 2, "s": 2},
            {"type": "conv", "f_out": b, "k": 3, "relu": True}, {"type": "pool", "k": 2, "s": 2},
            {"type": "ip", "f_out": c, "relu": True}, {"type": "ip", "f_out": e, "relu": True},
            {"type": "ip", "f_out": classes, "relu": False}]


def he_normal_weights3d(layers, c_in, seed, bias_scale=0.0):
    """As he_normal_weights for kernels [f_out, f_in, k, k, k] (standard deviation sqrt(2/(f_in k^3)))."""
    rng = np.random.default_rng(seed)
    ws, bs, f_in = [], [], c_in
    for l in layers:
        if l["type"] != "conv":
            continue
        k, f_out = l["k"], l["f_out"]
        w = rng.standard_normal((f_out, f_in, k, k, k)) * np.sqrt(2.0 / (f_in * k ** 3))
        b = rng.standard_normal(f_out) * bias_scale
        ws.append(w.astype(np.float32))
        bs.append(b.astype(np.float32))
        f_in = f_out
    return ws, bs


def uniform_volume(c, dz, h, w, seed):
    return np.random.default_rng(seed).random((c, dz, h, w), dtype=np.float32)


def em_like_volume(dz, h, w, seed):
    """A stack of dz sections [1, dz, h, w]: consecutive sections are one slowly changing texture (blurred
    along the stack as well), each crossed by its own dark curves as in em_like_image."""
    rng = np.random.default_rng(seed)
    base = ndimage.gaussian_filter(rng.random((dz, h, w)), (1.5, 2.0, 2.0), mode="reflect", truncate=4.0)
    base = (base - base.min()) / (base.max() - base.min())
    marks = np.stack([em_like_image(h, w, seed + 1 + z) for z in range(dz)])
    vol = 0.5 * base + 0.5 * marks
    return vol[None].astype(np.float32)


def uniform_image(n, c, h, w, seed):
    return np.random.default_rng(seed).random((n, c, h, w), dtype=np.float32)


def em_like_image(h, w, seed):
    """Blurred uniform noise crossed by dark random-walk curves, normalised to [0,1]; [h,w] fp32."""
    rng = np.random.default_rng(seed)
    img = ndimage.gaussian_filter(rng.random((h, w)), 2.0, mode="reflect", truncate=4.0)
    img = (img - img.min()) / (img.max() - img.min())
    n_curves = max(1, int(round(40 * h * w / (512.0 * 512.0))))
    mask = np.zeros((h, w), dtype=bool)
    for _ in range(n_curves):
        y, x = rng.random() * h, rng.random() * w
        heading = rng.random() * 2 * np.pi
        length = int(rng.integers(100, 401))
        thick = int(rng.integers(2, 5))
        turns = rng.normal(0.0, 0.15, size=length)
        for t in range(length):
            heading += turns[t]
            y += np.sin(heading)
            x += np.cos(heading)
            yi, xi = int(round(y)), int(round(x))
            if 0 <= yi < h and 0 <= xi < w:
                mask[max(0, yi - thick // 2):yi + (thick + 1) // 2,
                     max(0, xi - thick // 2):xi + (thick + 1) // 2] = True
    img = img - 0.5 * mask
    img = ndimage.gaussian_filter(img, 1.0, mode="reflect", truncate=4.0)
    img = (img - img.min()) / (img.max() - img.min())
    return img.astype(np.float32)


def em_like_batch(n, h, w, first_seed):
    return np.stack([em_like_image(h, w, first_seed + i) for i in range(n)])[:, None]


def binary_labels(n, h, w, seed, p_one=0.2):
    return (np.random.default_rng(seed).random((n, h, w)) < p_one).astype(np.int32)


# ---- U-Net (config C5) -------------------------------------------------------------------

def unet_param_names(depth=4):
    names = []
    for i in range(depth + 1):
        names += ["down%da" % i, "down%db" % i]
    for i in range(depth - 1, -1, -1):
        names += ["up%d" % i, "dec%da" % i, "dec%db" % i]
    return names + ["head"]


def unet_params(c_in, classes, seed, depth=4, base=64, bias_scale=0.0):
    """He-normal weights for every U-Net layer (fan-in f_in*k^2 for convs, f_in for the
    up-convolutions); returns {name: (w, b)} fp32.
    conv weights [f_out,f_in,3,3]; up-convolution weights [f_in, f_in/2, 2, 2]; head [classes,base,1,1]."""
    rng = np.random.default_rng(seed)
    ch = [base * 2 ** i for i in range(depth + 1)]
    shapes = {}
    f_in = c_in
    for i in range(depth + 1):
        shapes["down%da" % i] = (ch[i], f_in, 3, 3)
        shapes["down%db" % i] = (ch[i], ch[i], 3, 3)
        f_in = ch[i]
    for i in range(depth - 1, -1, -1):
        shapes["up%d" % i] = (ch[i + 1], ch[i], 2, 2)
        shapes["dec%da" % i] = (ch[i], 2 * ch[i], 3, 3)
        shapes["dec%db" % i] = (ch[i], ch[i], 3, 3)
    shapes["head"] = (classes, base, 1, 1)
    out = {}
    for name in unet_param_names(depth):
        shp = shapes[name]
        if name.startswith("up"):
            fan_in, f_out = shp[0], shp[1]      # every output pixel sees one tap per input map
        else:
            fan_in, f_out = shp[1] * shp[2] * shp[3], shp[0]
        w = rng.standard_normal(shp) * np.sqrt(2.0 / fan_in)
        b = rng.standard_normal(f_out) * bias_scale
        out[name] = (w.astype(np.float32), b.astype(np.float32))
    return out


# ---- USK-Net (the USK network configuration table, 692 -> 512) ----------------------------------------

USKNET_PARAM_NAMES = ("conv1", "conv2", "conv3", "conv4", "conv5", "ip1", "ip2", "up1", "conv7", "conv8", "ip3")


def usknet_params(c_in, classes, seed, base=64, bias_scale=0.0):
    """He-normal weights for every USK-Net layer, {name: (w, b)} fp32, channel counts of the table
    scaled by base/64: conv weights [f_out, f_in, k, k], the up-convolution [4*base, 2*base, 2, 2]."""
    b = base
    shapes = {"conv1": (b, c_in, 3, 3), "conv2": (b, b, 3, 3),
              "conv3": (2 * b, b, 6, 6), "conv4": (2 * b, 2 * b, 4, 4), "conv5": (2 * b, 2 * b, 4, 4),
              "ip1": (8 * b, 2 * b, 8, 8), "ip2": (4 * b, 8 * b, 1, 1),
              "up1": (4 * b, 2 * b, 2, 2),
              "conv7": (2 * b, 3 * b, 3, 3), "conv8": (b, 2 * b, 3, 3), "ip3": (classes, b, 1, 1)}
    rng = np.random.default_rng(seed)
    out = {}
    for name in USKNET_PARAM_NAMES:
        shp = shapes[name]
        if name == "up1":
            fan_in, f_out = shp[0], shp[1]
        else:
            fan_in, f_out = shp[1] * shp[2] * shp[3], shp[0]
        w = rng.standard_normal(shp) * np.sqrt(2.0 / fan_in)
        bias = rng.standard_normal(f_out) * bias_scale
        out[name] = (w.astype(np.float32), bias.astype(np.float32))
    return out


# ---- label masking (Section 4.2, the masking inequality) ----------------------------------------------

def mask_labels_by_frequency(labels, classes, seed):
    """Label map with pixels masked (-1) at random so that every label is left about equally often:
    a pixel of label i is kept with probability min_j c_j / c_i (c = label frequencies in this map,
    labels that do not occur left out of the minimum), so the rarest label is never masked."""
    labels = np.asarray(labels)
    c = np.bincount(labels.reshape(-1), minlength=classes).astype(np.float64) / labels.size
    keep_p = np.where(c > 0, c[c > 0].min() / np.maximum(c, 1e-300), 1.0)
    u = np.random.default_rng(seed).random(labels.shape)
    return np.where(u < keep_p[labels], labels, -1).astype(np.int32)
