"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

C3 (8 x 1024^2, bf16) is too large for the oracle as a whole, but every output pixel depends only
on its (v+1)^2 input window (Sections 1.3 and 3.1: output-size invariance), so the oracle computes
sampled output windows one by one from crops of the mirror-padded input.  C4 (512^2 bf16 training
step) is compared in full."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import layers as OL, nets as ON

pytestmark = pytest.mark.gpu

HALF_TOL = 2e-2


def make_net(layers, ws, bs, dtype):
    from paper_1509_03371_amd import binding as B
    net = B.SKNet(layers, 1, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    return net


def sample_windows(n, H, win, rng):
    """Per image: the four corners (mirror padding), four windows that straddle tile seams of the 16-bit
    convolution's tiling (columns 128k, rows 64k: every row-tile boundary 8*d of d = 1, 2, 4, 8 passes there)
    and two random places."""
    places = []
    for b in range(n):
        places += [(b, 0, 0), (b, 0, H - win), (b, H - win, 0), (b, H - win, H - win)]
        for _ in range(4):
            kx, ky = int(rng.integers(1, H // 128)), int(rng.integers(1, H // 64))
            places.append((b, 64 * ky - win // 2, 128 * kx - win // 2))
        places += [(b, int(rng.integers(0, H - win)), int(rng.integers(0, H - win))) for _ in range(2)]
    return places


@pytest.mark.parametrize("dtype,n", [("bf16", 8), ("f16", 2)])
def test_c3_forward_1024_sampled_windows(dtype, n):
    """The inference plan bench.py times (fused layers: probabilities only) and a plan that keeps every
    layer, whose fp32 logits carry the 2e-2 relative bound; both against oracle windows."""
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    H = 1024
    img = S.em_like_batch(n, H, H, 3)
    timg = torch.from_numpy(img).cuda()
    net = make_net(layers, ws, bs, dtype)
    net.plan(n, H, H, pad=True)                      # inference plan, as timed by bench.py
    prob = net.forward(timg).cpu().numpy()
    assert prob.shape == (n, 2, H, H)
    assert np.isfinite(prob).all()
    assert np.abs(prob.sum(1) - 1).max() < 1e-5
    net.plan(n, H, H, pad=True, keep=True)           # every layer kept: the logits are an output
    prob_keep = net.forward(timg).cpu().numpy()
    logits = net.get_activation(len(layers) - 1)
    net.close()
    v = 60
    half = v // 2
    win = 24
    places = sample_windows(n, H, win, np.random.default_rng(99))
    assert len(places) >= 10 * n
    padded = {}
    refs = []
    for b, y0, x0 in places:
        if b not in padded:
            padded[b] = OL.mirror_pad(img[b:b + 1], half, half, half, half)
        crop = padded[b][:, :, y0:y0 + win + v, x0:x0 + win + v]
        ref_prob, acts, _ = ON.sknet_forward(crop, layers, ws, bs, pad=False, keep=True)
        refs.append((ref_prob, acts[-1]))
    zmax = max(np.abs(z).max() for _, z in refs)
    worst_z = worst_p = 0.0
    for (b, y0, x0), (ref_prob, ref_z) in zip(places, refs):
        ez = np.abs(logits[b:b + 1, :, y0:y0 + win, x0:x0 + win] - ref_z).max() / zmax
        ep = max(np.abs(prob[b:b + 1, :, y0:y0 + win, x0:x0 + win] - ref_prob).max(),
                 np.abs(prob_keep[b:b + 1, :, y0:y0 + win, x0:x0 + win] - ref_prob).max())
        worst_z, worst_p = max(worst_z, ez), max(worst_p, ep)
        assert ez <= HALF_TOL and ep <= HALF_TOL, (b, y0, x0, ez, ep)
    print(dtype, "%d windows: logits rel err %.3e, probabilities abs err %.3e" % (len(places), worst_z, worst_p), flush=True)


@pytest.mark.parametrize("fused_head,n,size", [(False, 1, 512), (True, 1, 512), (True, 2, 1024)])
def test_c4_bf16_training_step_512(fused_head, n, size):
    """The training step at the benchmark's sizes and in its plan modes: layer by layer (mode 1), and with the head
    and the loss as one kernel per direction (mode 3, what bench.py times), also on 1024^2 images."""
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    img = S.em_like_batch(n, size, size, 2)
    labels = S.binary_labels(n, size, size, 2004)
    net = make_net(layers, ws, bs, "bf16")
    net.plan(n, size, size, pad=True, training=True, fused_head=fused_head)
    timg, tlab = torch.from_numpy(img).cuda(), torch.from_numpy(labels).cuda()
    prob = net.forward(timg).cpu().numpy()
    loss = net.backward(tlab)
    ow = [x.astype(np.float64) for x in ws]
    ob = [x.astype(np.float64) for x in bs]
    ref_prob, acts, ams = ON.sknet_forward(img, layers, ow, ob, keep=True)
    ref_loss, dws, dbs, _ = ON.sknet_backward(layers, ow, acts, ams, labels)
    assert np.abs(prob - ref_prob).max() <= HALF_TOL
    if not fused_head:                                   # the one-kernel head keeps no logits
        logits = net.get_activation(len(layers) - 1)
        assert np.abs(logits - acts[-1]).max() <= HALF_TOL * np.abs(acts[-1]).max()
    assert abs(loss.item() - ref_loss) <= HALF_TOL * abs(ref_loss)
    for i in range(net.num_convs()):
        dw, db = net.get_grad(i)
        scale = np.abs(dws[i]).max()
        assert np.abs(dw - dws[i]).max() <= 5e-2 * scale, ("dW", i, np.abs(dw - dws[i]).max() / scale)
        assert np.abs(db - dbs[i]).max() <= 5e-2 * max(np.abs(dbs[i]).max(), scale), ("db", i)
    before = [net.get_weights(i) for i in range(net.num_convs())]
    grads = [net.get_grad(i) for i in range(net.num_convs())]
    net.sgd_step(0.01)
    for i in range(net.num_convs()):
        w1, b1 = net.get_weights(i)
        assert np.abs(w1 - (before[i][0] - np.float32(0.01) * grads[i][0])).max() <= 1e-7
    net.close()
