"""GPU: training plans whose head (1x1 conv + ReLU, 1x1 conv, softmax loss; Sections 4.2, 4.3) runs as one kernel
in each direction (plan mode 3, 16-bit storage).  Loss and every weight / bias gradient against the fp64 oracle on
the unrounded fp32 weights, at the bounds of the layer-by-layer 16-bit training path; an SGD step and a second
pass (the packed head weights follow the update); the refusals."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import nets as ON

pytestmark = pytest.mark.gpu


def relerr(got, ref):
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def make_net(layers, c_in, ws, bs, dtype):
    from paper_1509_03371_amd import binding as B
    net = B.SKNet(layers, c_in, layers[-1]["f_out"], dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    return net


def labels_for(n, h, w, classes, seed, masked):
    rng = np.random.default_rng(seed)
    lab = rng.integers(0, classes, (n, h, w)).astype(np.int32)
    if masked:
        lab[rng.random((n, h, w)) < 0.3] = -1
    return lab


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("width,hidden,classes,stages,n,h,w,masked", [
    (16, 40, 2, 2, 1, 37, 45, False),      # 16 maps into the head (one map tile), 4 hidden tiles, pixels no multiple of 64
    (24, 100, 3, 2, 2, 30, 70, True),      # 24 maps (two tiles, one octet short), 8 hidden tiles, three classes, masked labels
    (48, 200, 2, 4, 2, 40, 50, True),      # the benchmark net's head: 48 -> 200 -> 2
    (40, 208, 4, 1, 1, 20, 33, False),     # 13 full hidden tiles, four classes
])
def test_fused_head_training_pass(dtype, width, hidden, classes, stages, n, h, w, masked):
    layers = S.sknet_layers(width=width, hidden=hidden, classes=classes, stages=stages)
    ws, bs = S.he_normal_weights(layers, 1, 500 + hidden, bias_scale=0.05)
    img = S.em_like_batch(n, h, w, 60)
    labels = labels_for(n, h, w, classes, 61, masked)
    net = make_net(layers, 1, ws, bs, dtype)
    net.plan(n, h, w, pad=True, training=True, fused_head=True)
    prob = net.forward(torch.from_numpy(img).cuda())
    loss = net.backward(torch.from_numpy(labels).cuda())
    ow = [x.astype(np.float64) for x in ws]
    ob = [x.astype(np.float64) for x in bs]
    ref_prob, acts, ams = ON.sknet_forward(img, layers, ow, ob, keep=True)
    ref_loss, dws, dbs, _ = ON.sknet_backward(layers, ow, acts, ams, labels)
    assert np.abs(prob.cpu().numpy() - ref_prob).max() <= 2e-2
    assert abs(loss.item() - ref_loss) <= 2e-2 * abs(ref_loss), (loss.item(), ref_loss)
    tol = 5e-2 if dtype == "bf16" else 1e-2
    grads = [net.get_grad(i) for i in range(net.num_convs())]
    for i, (dw, db) in enumerate(grads):
        print(dtype, "conv", i, "dW rel err %.3e" % relerr(dw, dws[i]), "db abs err %.3e of %.3e" % (np.abs(db - dbs[i]).max(), np.abs(dbs[i]).max()), flush=True)
    for i, (dw, db) in enumerate(grads):
        assert relerr(dw, dws[i]) <= tol, ("dW", i, relerr(dw, dws[i]))
        assert np.abs(db - dbs[i]).max() <= tol * max(np.abs(dbs[i]).max(), np.abs(dws[i]).max()), ("db", i)
    # one SGD step on the fp32 masters, then a second pass: its loss is that of the updated weights
    before = [net.get_weights(i) for i in range(net.num_convs())]
    net.sgd_step(0.002)
    after = [net.get_weights(i) for i in range(net.num_convs())]
    for i in range(net.num_convs()):
        assert np.abs(after[i][0] - (before[i][0] - np.float32(0.002) * grads[i][0])).max() <= 1e-6
    net.forward(torch.from_numpy(img).cuda())
    loss2 = net.backward(torch.from_numpy(labels).cuda()).item()
    _, acts2, ams2 = ON.sknet_forward(img, layers, [x.astype(np.float64) for x, _ in after], [b.astype(np.float64) for _, b in after], keep=True)
    ref_loss2 = ON.sknet_backward(layers, [x.astype(np.float64) for x, _ in after], acts2, ams2, labels)[0]
    assert abs(loss2 - ref_loss2) <= 2e-2 * abs(ref_loss2), (loss2, ref_loss2)
    assert loss2 < loss.item()
    net.close()


def test_fused_head_training_matches_layer_by_layer():
    """The same step in plan mode 1 (every layer a launch): both round to 16 bits at the same places, so the
    gradients agree far more closely with each other than either does with the fp64 oracle."""
    layers = S.sknet_layers(width=48, hidden=200, stages=2)
    ws, bs = S.he_normal_weights(layers, 1, 77, bias_scale=0.05)
    img = S.em_like_batch(2, 48, 64, 62)
    labels = labels_for(2, 48, 64, 2, 63, True)
    out = []
    for fused in (False, True):
        net = make_net(layers, 1, ws, bs, "f16")
        net.plan(2, 48, 64, pad=True, training=True, fused_head=fused)
        net.forward(torch.from_numpy(img).cuda())
        loss = net.backward(torch.from_numpy(labels).cuda()).item()
        out.append((loss, [net.get_grad(i) for i in range(net.num_convs())]))
        net.close()
    assert abs(out[0][0] - out[1][0]) <= 1e-4 * abs(out[0][0])
    for (dw0, db0), (dw1, db1) in zip(out[0][1], out[1][1]):
        assert relerr(dw1, dw0.astype(np.float64)) <= 3e-3
        assert np.abs(db1 - db0).max() <= 3e-3 * max(np.abs(db0).max(), np.abs(dw0).max())


def test_fused_head_training_refusals():
    from paper_1509_03371_amd import binding as B
    layers = S.sknet_layers(width=16, hidden=40, stages=1)
    net = B.SKNet(layers, 1, 2, dtype="f32")
    with pytest.raises(B.SknetError):                      # fp32 storage
        net.plan(1, 20, 20, training=True, fused_head=True)
    net.close()
    wide = S.sknet_layers(width=16, hidden=300, stages=1)   # more than 208 hidden maps
    net = B.SKNet(wide, 1, 2, dtype="bf16")
    with pytest.raises(B.SknetError):
        net.plan(1, 20, 20, training=True, fused_head=True)
    net.close()
    no_pool = [S.conv(16, 4, 1), S.conv(40, 1, 1), S.conv(2, 1, 1, relu=False)]   # a ReLU convolution right in front of the head
    net = B.SKNet(no_pool, 1, 2, dtype="bf16")
    with pytest.raises(B.SknetError):
        net.plan(1, 20, 20, training=True, fused_head=True)
    net.close()
    net = B.SKNet(layers, 1, 2, dtype="bf16")
    net.plan(1, 20, 20, training=True, fused_head=True)
    net.forward(torch.zeros((1, 1, 20, 20), device="cuda"))
    with pytest.raises(B.SknetError):                      # the hidden maps are never stored
        net.get_activation(len(layers) - 2)
    net.close()
