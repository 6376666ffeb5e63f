"""GPU parity: SK-Net training step (loss, gradients, SGD) against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import layers as OL, nets as ON

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4


def relerr(got, ref):
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def make_net(layers, c_in, ws, bs, **kw):
    from paper_1509_03371_amd import binding as B
    classes = [l for l in layers if l["type"] == "conv"][-1]["f_out"]
    net = B.SKNet(layers, c_in, classes, **kw)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    return net


def train_step_compare(layers, c_in, img, labels, ws, bs, lr=0.01, momentum=0.0, wd=0.0, tol=FP32_TOL, steps=1):
    net = make_net(layers, c_in, ws, bs)
    n, _, h, w = img.shape
    net.plan(n, h, w, pad=True, training=True)
    ow = [x.astype(np.float64) for x in ws]
    ob = [x.astype(np.float64) for x in bs]
    vw = [np.zeros_like(x) for x in ow]
    vb = [np.zeros_like(x) for x in ob]
    timg, tlab = torch.from_numpy(img).cuda(), torch.from_numpy(labels).cuda()
    for _ in range(steps):
        net.forward(timg)
        loss = net.backward(tlab)
        _, acts, ams = ON.sknet_forward(img, layers, ow, ob, keep=True)
        ref_loss, dws, dbs, _ = ON.sknet_backward(layers, ow, acts, ams, labels)
        assert abs(float(loss.item()) - ref_loss) <= tol * abs(ref_loss)
        for i in range(net.num_convs()):
            dw, db = net.get_grad(i)
            assert relerr(dw, dws[i]) <= tol, ("dW", i)
            assert np.abs(db - dbs[i]).max() <= tol * max(np.abs(dbs[i]).max(), np.abs(dws[i]).max()), ("db", i)
        net.sgd_step(lr, momentum, wd)
        ON.sgd_step(ow, ob, dws, dbs, lr, momentum, wd, vw, vb)
        for i in range(net.num_convs()):
            w_gpu, b_gpu = net.get_weights(i)
            assert relerr(w_gpu, ow[i]) <= 1e-6, ("W after SGD", i)
            assert np.abs(b_gpu - ob[i]).max() <= 1e-6 * max(1.0, np.abs(ob[i]).max())
    # the updated weights are the ones the next forward uses
    prob = net.forward(timg).cpu().numpy()
    ref_prob = ON.sknet_forward(img, layers, ow, ob)
    assert np.abs(prob - ref_prob).max() <= tol
    net.close()


def test_tiny_net_training_step():
    layers = S.tiny_sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1000, bias_scale=0.1)
    img = S.uniform_image(2, 1, 40, 52, 3)
    labels = S.binary_labels(2, 40, 52, 4)
    train_step_compare(layers, 1, img, labels, ws, bs, lr=0.05, momentum=0.9, wd=1e-3, steps=2)


def test_training_step_with_masked_labels():
    # Section 4.2's label masking: pixels masked (-1) by inverse label frequency carry no error; the
    # normaliser is the number of labelled pixels.  Three classes, two images, momentum SGD.
    layers = [S.conv(8, 3, 1, relu=True), S.pool(2, 1, 1), S.conv(12, 3, 2, relu=True), S.conv(3, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 2, 1200, bias_scale=0.1)
    img = S.uniform_image(2, 2, 44, 70, 5)
    raw = (np.random.default_rng(6).random((2, 44, 70)) < 0.2).astype(np.int32) + (np.random.default_rng(7).random((2, 44, 70)) < 0.05)
    labels = S.mask_labels_by_frequency(raw, 3, 8)
    assert (labels == -1).mean() > 0.3 and (labels >= 0).sum() > 100
    train_step_compare(layers, 2, img, labels, ws, bs, lr=0.05, momentum=0.5, steps=2)


def test_all_pixels_masked_gives_zero_loss_and_gradients():
    layers = S.tiny_sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1000, bias_scale=0.1)
    net = make_net(layers, 1, ws, bs)
    net.plan(1, 32, 40, pad=True, training=True)
    net.forward(torch.from_numpy(S.uniform_image(1, 1, 32, 40, 3)).cuda())
    loss = net.backward(torch.full((1, 32, 40), -1, dtype=torch.int32, device="cuda"))
    assert float(loss.item()) == 0.0
    for i in range(net.num_convs()):
        dw, db = net.get_grad(i)
        assert not dw.any() and not db.any()
    net.close()


def test_three_class_net_with_k3_and_ragged_sizes():
    layers = [S.conv(10, 3, 1), S.pool(2, 1), S.conv(20, 3, 2), S.pool(3, 2), S.conv(33, 2, 6), S.conv(3, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 3, 77, bias_scale=0.1)
    img = S.uniform_image(1, 3, 37, 71, 5)
    labels = np.random.default_rng(6).integers(0, 3, (1, 37, 71)).astype(np.int32)
    train_step_compare(layers, 3, img, labels, ws, bs)


def test_pool_backward_bit_exact_routing():
    """pool -> 1x1 conv: the image gradient is not needed, so check the routing through a net whose
    first layer is a conv: conv1x1 (identity-like) -> pool -> conv1x1."""
    layers = [S.conv(4, 1, 1, relu=False), S.pool(2, 3), S.conv(2, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 4, 9, bias_scale=0.3)
    img = np.maximum(np.random.default_rng(7).standard_normal((2, 4, 30, 45)), 0).astype(np.float32)
    labels = S.binary_labels(2, 30, 45, 8)
    train_step_compare(layers, 4, img, labels, ws, bs)


def compare_error_maps(layers, c_in, img, labels, ws, bs, dtype, tol, tag):
    """Error map of every layer (sknet_get_activation_grad) against the oracle's, every element."""
    n, _, h, w = img.shape
    net = make_net(layers, c_in, ws, bs, dtype=dtype)
    net.plan(n, h, w, pad=True, training=True)
    tlab = torch.from_numpy(labels).cuda()
    net.forward(torch.from_numpy(img).cuda())
    ow, ob = [x.astype(np.float64) for x in ws], [x.astype(np.float64) for x in bs]
    _, acts, ams = ON.sknet_forward(img, layers, ow, ob, keep=True)
    diffs = []
    ON.sknet_backward(layers, ow, acts, ams, labels, diffs=diffs)
    for li in range(len(layers) - 1, -1, -1):
        got = net.get_activation_grad(li, tlab)
        ref = diffs[li]
        assert got.shape == ref.shape and np.abs(ref).max() > 0, li
        e = relerr(got, ref)
        edge = max(relerr(got[:, :, :8], ref[:, :, :8]), relerr(got[:, :, -8:], ref[:, :, -8:]),
                   relerr(got[:, :, :, :8], ref[:, :, :, :8]), relerr(got[:, :, :, -8:], ref[:, :, :, -8:]))
        print(tag, dtype, "layer", li, layers[li]["type"], "error map rel err %.3e (8-wide borders %.3e)" % (e, edge), flush=True)
        assert e <= tol, (li, e)
    with pytest.raises(Exception):
        net.get_grad(0)                    # the partial walks overwrote gradients: a new backward is needed
    net.backward(tlab)
    net.get_grad(0)
    net.close()


@pytest.mark.parametrize("dtype,tol", [("f32", FP32_TOL), ("f16", 5e-3), ("bf16", 2e-2)])
def test_data_gradient_error_maps_borders_included(dtype, tol):
    """The data gradient of the dilated convolutions compared directly, element by element, not through
    the weight gradients of the layers below: the error map of every layer of a chain of 4x4 convolutions at
    d = 1, 2, 4, 8, including the (k-1)d-wide border that only partial sums reach.  The chain has no ReLU and
    no pool, so no decision can fall differently in the two precisions and the maps are held to the
    tolerance of the arithmetic.  Two images, non-square, masked labels."""
    layers = [S.conv(16, 1, 1, relu=False)] + [S.conv(16, 4, d, relu=False) for d in (1, 2, 4, 8)] + [S.conv(2, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 3, 21, bias_scale=0.1)
    n, h, w = 2, 50, 150
    img = np.ascontiguousarray(S.em_like_batch(n, h, w, 22).repeat(3, 1) * np.array([1.0, 0.5, -0.7], np.float32)[None, :, None, None])
    labels = S.binary_labels(n, h, w, 23)
    labels[0, :5, :] = -1
    compare_error_maps(layers, 3, img, labels, ws, bs, dtype, tol, "dgrad")


@pytest.mark.parametrize("dtype,tol", [("f32", FP32_TOL), ("f16", 5e-3), ("bf16", 2e-2)])
def test_pool_scatter_error_maps_with_ties(dtype, tol):
    """The pool gradient compared directly: identity 1x1 convolution + ReLU, then SK pools at d = 1, 2, 4, 8,
    then a 1x1 convolution to the classes.  The image holds multiples of 1/16 (exact in every storage type,
    many ties, negative values and zeros for the fused ReLU mask), so both sides pool identical numbers and
    pick identical winners; the error maps then differ by the arithmetic of the head alone."""
    layers = [S.conv(8, 1, 1, relu=True)] + [S.pool(2, d) for d in (1, 2, 4, 8)] + [S.conv(3, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 8, 31, bias_scale=0.1)
    ws[0] = np.eye(8, dtype=np.float32).reshape(8, 8, 1, 1)
    bs[0] = np.zeros(8, np.float32)
    n, h, w = 2, 45, 140
    img = (np.random.default_rng(32).integers(-16, 48, (n, 8, h, w)) / 16.0).astype(np.float32)
    labels = np.random.default_rng(33).integers(-1, 3, (n, h, w)).astype(np.int32)
    compare_error_maps(layers, 8, img, labels, ws, bs, dtype, tol, "pool")


def test_c4_sknet_training_step_512():
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    img = S.em_like_batch(1, 512, 512, 2)
    labels = S.binary_labels(1, 512, 512, 2004)
    train_step_compare(layers, 1, img, labels, ws, bs, lr=0.01)


def test_backward_is_deterministic():
    layers = S.sknet_layers(width=16, hidden=24)
    ws, bs = S.he_normal_weights(layers, 1, 5)
    img = S.em_like_batch(1, 96, 96, 12)
    labels = S.binary_labels(1, 96, 96, 13)
    net = make_net(layers, 1, ws, bs)
    net.plan(1, 96, 96, pad=True, training=True)
    timg, tlab = torch.from_numpy(img).cuda(), torch.from_numpy(labels).cuda()
    grads = []
    for _ in range(2):
        net.forward(timg)
        net.backward(tlab)
        grads.append([net.get_grad(i) for i in range(net.num_convs())])
    for (dw0, db0), (dw1, db1) in zip(*grads):
        assert np.array_equal(dw0, dw1) and np.array_equal(db0, db1)
    net.close()


def test_state_errors_on_gpu():
    from paper_1509_03371_amd import binding as B
    layers = S.tiny_sknet_layers()
    net = B.SKNet(layers, 1, 2)
    img = torch.zeros(1, 1, 32, 32, device="cuda")
    net._plan = (1, 32, 32, True, False)
    net._shapes = net.infer_shapes(32, 32)
    with pytest.raises(B.SknetError) as e:
        net.forward(img)                                  # no plan
    assert e.value.status_name == "SK_ESTATE"
    net.plan(1, 32, 32)
    net.forward(img)
    with pytest.raises(B.SknetError) as e:
        net.backward(torch.zeros(1, 32, 32, dtype=torch.int32, device="cuda"))   # not a training plan
    assert e.value.status_name == "SK_ESTATE"
    net.plan(1, 32, 32, training=True)
    with pytest.raises(B.SknetError) as e:
        net.backward(torch.zeros(1, 32, 32, dtype=torch.int32, device="cuda"))   # no forward yet
    assert e.value.status_name == "SK_ESTATE"
    net.close()
