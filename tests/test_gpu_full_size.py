"""GPU parity at BASELINE's full sizes, in the launch configuration bench.py times.

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


def test_c3_bf16_forward_8x1024_sampled_windows():
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    n, H = 8, 1024
    img = S.em_like_batch(n, H, H, 3)
    net = make_net(layers, ws, bs, "bf16")
    net.plan(n, H, H, pad=True)                      # inference plan, as timed by bench.py
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    assert prob.shape == (n, 2, H, H)
    assert np.isfinite(prob).all()
    assert np.abs(prob.sum(1) - 1).max() < 1e-5
    v = net.context()
    half = v // 2
    rng = np.random.default_rng(99)
    win = 24
    # corners (mirror padding), tile seams of the 128-column / 8-row tiling, and random places
    places = [(0, 0, 0), (7, H - win, H - win), (3, 0, H - win), (5, 500, 120), (2, 1000, 250)]
    places += [(int(rng.integers(0, n)), int(rng.integers(0, H - win)), int(rng.integers(0, H - win))) for _ in range(7)]
    worst = 0.0
    for b, y0, x0 in places:
        padded = OL.mirror_pad(img[b:b + 1], half, half, half, half)
        crop = padded[:, :, y0:y0 + win + v, x0:x0 + win + v]
        ref = ON.sknet_forward(crop, layers, ws, bs, pad=False)
        err = np.abs(prob[b:b + 1, :, y0:y0 + win, x0:x0 + win] - ref).max()
        worst = max(worst, err)
        assert err <= HALF_TOL, (b, y0, x0, err)
    net.close()


def test_c4_bf16_training_step_512():
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    img = S.em_like_batch(1, 512, 512, 2)
    labels = S.binary_labels(1, 512, 512, 2004)
    net = make_net(layers, ws, bs, "bf16")
    net.plan(1, 512, 512, pad=True, training=True)
    timg, tlab = torch.from_numpy(img).cuda(), torch.from_numpy(labels).cuda()
    prob = net.forward(timg).cpu().numpy()
    loss = net.backward(tlab)
    ow = [x.astype(np.float64) for x in ws]
    ob = [x.astype(np.float64) for x in bs]
    ref_prob, acts, ams = ON.sknet_forward(img, layers, ow, ob, keep=True)
    ref_loss, dws, dbs, _ = ON.sknet_backward(layers, ow, acts, ams, labels)
    assert np.abs(prob - ref_prob).max() <= HALF_TOL
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


def test_c3_fp16_matches_bf16_within_tolerance_on_one_image():
    """The fp16 instantiation of the same kernels at 1024^2 (one image): against the bf16 result."""
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    img = S.em_like_batch(1, 1024, 1024, 3)
    out = {}
    for dt in ("bf16", "f16"):
        net = make_net(layers, ws, bs, dt)
        net.plan(1, 1024, 1024, pad=True)
        out[dt] = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
        net.close()
    assert np.abs(out["bf16"] - out["f16"]).max() <= 2 * HALF_TOL
