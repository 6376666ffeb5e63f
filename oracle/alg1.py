"""Algorithm 1 (Section 3.3.1): sliding-window net -> strided-kernel net, plus the size,
FLOP and parameter bookkeeping the paper's tables are built from.  Host arithmetic only.
TEST INFRASTRUCTURE ONLY.

A SW layer is a dict: {"type": "conv", "f_out", "k", "relu"}, {"type": "pool", "k", "s"},
{"type": "ip", "f_out", "relu"} or {"type": "other", "k"} (element-wise layers have k = 1).
A SK layer is {"type": "conv", "f_out", "k", "d", "relu"} or {"type": "pool", "k", "d", "s"}.
"""


class ConversionError(ValueError):
    pass


def convert_sw_to_sk(sw_layers, w0_sw):
    """Return (sk_layers, w_sw, w_sk): converted layers and the per-layer map sizes of both
    nets when the SK net is fed the SW patch size (so its last size is 1).

    What Algorithm 1 states, in one walk over the layers: a layer keeps its kernel and takes as kernel
    stride the product of the pooling strides in front of it (counted from the last inner product, which
    sees a 1 x 1 map again); a pool loses its layer stride; an inner product is a convolution whose kernel
    is the whole remaining patch.  Pools must divide their map and have k = s, anything else with a kernel
    cannot be converted, and the stride product must be back at 1 at the end."""
    sk, w_sw, w_sk = [], [w0_sw], [w0_sw]
    spacing = 1                                   # product of the pooling strides since the last inner product
    for lay in sw_layers:
        kind, patch = lay["type"], w_sw[-1]
        if kind in ("conv", "pool", "ip"):
            k = patch if kind == "ip" else lay["k"]
            if kind == "pool" and (lay["s"] != k or patch % k != 0):
                raise ConversionError("pooling needs w mod k = 0 and k = s (got w=%d k=%d s=%d)" % (patch, k, lay["s"]))
            if kind == "pool":
                sk.append({"type": "pool", "k": k, "d": spacing, "s": 1})
            else:
                sk.append({"type": "conv", "f_out": lay["f_out"], "k": k, "d": spacing, "relu": lay.get("relu", False)})
            w_sk.append(w_sk[-1] - (k - 1) * spacing)
            w_sw.append({"conv": patch - (k - 1), "pool": patch // k, "ip": 1}[kind])
            spacing = {"conv": spacing, "pool": spacing * k, "ip": 1}[kind]
        else:
            if lay.get("k", 1) > 1:
                raise ConversionError("a layer with k > 1 that is not conv/pool/ip cannot be converted")
            sk.append(dict(lay))
            w_sk.append(w_sk[-1])
            w_sw.append(patch)
        if w_sk[-1] < 1 or w_sw[-1] < 1:
            raise ConversionError("feature map shrank below one pixel")
    if spacing != 1:
        raise ConversionError("kernel stride is %d after the last layer; it must be 1" % spacing)
    return sk, w_sw, w_sk


def sk_sizes(sk_layers, w0):
    """Map size after every SK layer for input size w0: every layer with a kernel shrinks the map
    by (k-1)*d; a pool with layer stride s = k (U-Net) divides by k and needs w mod k = 0."""
    w = [w0]
    for l in sk_layers:
        if l["type"] == "conv":
            w.append(w[-1] - (l["k"] - 1) * l["d"])
        elif l["type"] == "pool":
            s = l.get("s", 1)
            if s == 1:
                w.append(w[-1] - (l["k"] - 1) * l["d"])
            else:
                if w[-1] % l["k"] != 0 or s != l["k"] or l.get("d", 1) != 1:
                    raise ConversionError("down-sampling pool needs w mod k = 0, s = k, d = 1")
                w.append(w[-1] // l["k"])
        elif l["type"] == "upconv":
            w.append(2 * w[-1])
        else:
            w.append(w[-1])
        if w[-1] < 1:
            raise ConversionError("feature map shrank below one pixel")
    return w


def context(sk_layers):
    """v = sum over layers of (k-1)*d: total context of a stride-1 SK net (= w_SW^(0) - 1)."""
    return sum((l["k"] - 1) * l["d"] for l in sk_layers if l["type"] in ("conv", "pool"))


def conv_flops(f_in, f_out, k, w_out, dims=2):
    """Section 5.5: M*N*(2K-1) with M = f_out, N = w^x, K = k^x * f_in."""
    return f_out * w_out ** dims * (2 * f_in * k ** dims - 1)


def free_parameters(conv_list):
    """Free-parameter equation of Section 3.3.2: |W| = sum f_in * f_out * k^2 over conv layers; conv_list = [(f_in, f_out, k)]."""
    return sum(fi * fo * k * k for fi, fo, k in conv_list)


def conv_buffer_elements(f_in, k, w_out, dims=2):
    """Convolution-buffer equation of Section 5.5: column-buffer size K*N = f_in * k^x * w^x (float elements)."""
    return f_in * k ** dims * w_out ** dims
