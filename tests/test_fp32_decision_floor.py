"""What single precision itself costs on the full-size U-Net training pass (1 x 572^2 -> 388^2, the
configuration table of Section 3.4), measured on the CPU with the library's reverse-mode differentiation:
the same pass in fp32 and in fp64, and the fp32 pass once more with every ReLU mask and pool winner taken
from the fp64 pass.  The first differs from fp64 by several 1e-4 of a gradient tensor's largest entry, the
second by far less than 1e-4: the gap is made by a handful of decisions (a pre-activation within rounding
of zero, two pool candidates within rounding of each other) that fall the other way, each of which moves
one whole pixel's term of sums that largely cancel, in its own layer and in every layer below it.  This is
the reason the GPU parity test at this size carries a wider bound than 1e-4 on gradients.  CPU only."""
import numpy as np
import torch
import torch.nn.functional as F

import sk_synth as S

DEPTH, BASE, SIZE = 4, 64, 572


def _pass(params, img, lab, dt, decisions=None):
    """One training pass in dtype dt.  decisions = None: the pass decides for itself and returns its ReLU
    masks and pool winners; else: a dict of those from another pass, applied instead."""
    tp = {k: (torch.from_numpy(w).to(dt).requires_grad_(), torch.from_numpy(b).to(dt).requires_grad_())
          for k, (w, b) in params.items()}
    made = {}

    def relu(name, x):
        if decisions is None:
            made[name] = x.detach() > 0
            return F.relu(x)
        return x * decisions[name].to(dt)

    def pool(name, x):
        if decisions is None:
            y, idx = F.max_pool2d(x, 2, return_indices=True)
            made[name] = idx
            return y
        idx = decisions[name]
        return torch.gather(x.flatten(2), 2, idx.flatten(2)).view(idx.shape)

    x = torch.from_numpy(img).to(dt)
    skips = []
    for i in range(DEPTH + 1):
        x = relu("down%da" % i, F.conv2d(x, *tp["down%da" % i]))
        x = relu("down%db" % i, F.conv2d(x, *tp["down%db" % i]))
        if i < DEPTH:
            skips.append(x)
            x = pool("pool%d" % i, x)
    for i in range(DEPTH - 1, -1, -1):
        x = F.conv_transpose2d(x, *tp["up%d" % i], stride=2)
        sk = skips[i].detach()                      # MergeCrop backwards into the up path only (Section 5.3.1)
        o = (sk.shape[2] - x.shape[2]) // 2
        x = torch.cat([x, sk[:, :, o:o + x.shape[2], o:o + x.shape[3]]], 1)
        x = relu("dec%da" % i, F.conv2d(x, *tp["dec%da" % i]))
        x = relu("dec%db" % i, F.conv2d(x, *tp["dec%db" % i]))
    z = F.conv2d(x, *tp["head"])
    loss = F.cross_entropy(z, torch.from_numpy(lab).long(), ignore_index=-1)
    loss.backward()
    grads = {k: w.grad.double().numpy() for k, (w, b) in tp.items()}
    return grads, made


def _worst(a, ref):
    return max(float(np.abs(a[k] - ref[k]).max() / np.abs(ref[k]).max()) for k in ref)


def test_fp32_floor_of_the_full_size_unet_training_pass_is_set_by_flipped_decisions():
    params = S.unet_params(1, 2, 1005, depth=DEPTH, base=BASE)
    img = np.ascontiguousarray(S.em_like_image(SIZE, SIZE, 1010)[None, None], dtype=np.float32)
    lab = S.mask_labels_by_frequency(S.binary_labels(1, 388, 388, 1011), 2, 1012)
    g64, dec64 = _pass(params, img, lab, torch.float64)
    g32, dec32 = _pass(params, img, lab, torch.float32)
    g32_same, _ = _pass(params, img, lab, torch.float32, decisions=dec64)
    flips = sum(int((dec64[k] != dec32[k]).sum()) for k in dec64)
    total = sum(dec64[k].numel() for k in dec64)
    free, same = _worst(g32, g64), _worst(g32_same, g64)
    print("fp32 vs fp64, own decisions: %.2e (%d of %d decisions differ); fp64's decisions: %.2e" % (free, flips, total, same))
    assert 0 < flips < 1e-5 * total          # a handful among 1e8
    assert free > 1e-4                       # plain fp32 misses the 1e-4 bar at this size ...
    assert free < 2e-3                       # ... but stays within the bound the GPU test uses
    assert same < 1e-4 and same < 0.2 * free # with equal decisions fp32 accumulation is far inside the bar
