"""GPU parity: 3-D SK net training pass (forward on a training plan, masked softmax loss, every weight and
bias gradient, pool winners, SGD step) through the C ABI against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import layers as OL, nd as OND

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4     # fp32 storage and fp32 MFMA accumulation against fp64, relative to the tensor's largest value


def relerr(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def to_dev(vol):
    return torch.from_numpy(np.ascontiguousarray(vol.transpose(1, 0, 2, 3))).cuda()


def run_training(layers, c_in, classes, size, seed, masked=True, tol=FP32_TOL):
    from paper_1509_03371_amd import binding as B
    ws, bs = S.he_normal_weights3d(layers, c_in, seed, bias_scale=0.1)
    net = B.SKNet3D(layers, c_in, classes)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    dz, h, w = size
    vol = S.uniform_volume(c_in, dz, h, w, seed + 1) - 0.3
    net.plan(dz, h, w, training=True)
    prob = net.forward(to_dev(vol)).cpu().numpy()
    od, _, oh, ow = net.out_shape()
    rng = np.random.default_rng(seed + 2)
    labels = rng.integers(0, classes, size=(od, oh, ow)).astype(np.int32)
    if masked:
        labels[rng.random(labels.shape) < 0.3] = -1
    loss = float(net.backward(torch.from_numpy(labels).cuda()).cpu())
    ref_prob, acts, argmaxes = OND.sknet3d_forward(vol, layers, ws, bs, keep=True)
    ref_loss, dws, dbs = OND.sknet3d_backward(layers, [w.astype(np.float64) for w in ws], acts, argmaxes, labels)
    assert np.abs(prob.transpose(1, 0, 2, 3) - ref_prob).max() <= tol
    assert abs(loss - ref_loss) <= tol * max(1.0, abs(ref_loss)), (loss, ref_loss)
    # pool winners: exact on the library's own input (a pool only selects, whatever the precision)
    pools = [i for i, l in enumerate(layers) if l["type"] == "pool"]
    for pi, li in enumerate(pools):
        src = net.get_activation(li - 1).transpose(1, 0, 2, 3) if li > 0 else vol
        _, am = OND.maxpool_sk3d(src, layers[li]["k"], layers[li]["d"], layers[li].get("s", 1), want_argmax=True)
        np.testing.assert_array_equal(net.get_pool_argmax(pi).transpose(1, 0, 2, 3), am.astype(np.int32))
    for i in range(len(ws)):
        dw, db = net.get_grad(i)
        assert np.abs(dws[i]).max() > 0, "degenerate test net: a reference gradient is all zero"
        ew, eb = relerr(dw, dws[i]), relerr(db, dbs[i])
        print("sk3d conv %d %s dW rel err %.3e  db rel err %.3e" % (i, dw.shape, ew, eb), flush=True)
        assert ew <= tol and eb <= tol, (i, ew, eb)
    return net, vol, labels, ws, bs, dws, dbs


def test_gradients_odd_map_counts_a_launch_per_depth_tap():
    # 5 / 7 / 9 maps: forward and data gradient of the d = 2 and d = 4 layers run one launch per depth tap
    layers = [S.conv(5, 2, 1), S.pool(2, 1), S.conv(7, 2, 2), S.pool(2, 2), S.conv(9, 3, 4), S.conv(3, 1, 1, relu=False)]
    net, *_ = run_training(layers, 2, 3, (18, 30, 75), 600)
    net.close()


def test_gradients_sixteen_map_multiples_one_launch():
    # 16 / 32 maps: forward and data gradient step over the slices between depth taps inside one launch
    layers = [S.conv(16, 3, 1), S.pool(2, 1), S.conv(32, 3, 2), S.pool(2, 2), S.conv(16, 2, 4), S.conv(2, 1, 1, relu=False)]
    net, *_ = run_training(layers, 1, 2, (20, 27, 80), 610)
    net.close()


def test_gradients_benchmark_net_map_counts():
    # the benchmark's net (16 / 32 / 128 / 64 maps, context 17) on a volume the oracle finishes in seconds:
    # the same kernels and launch forms as bench.py's training step, several column tiles and a ragged tail
    layers = S.sknet3d_layers(classes=2)
    net, *_ = run_training(layers, 1, 2, (25, 40, 150), 650)
    net.close()


@pytest.mark.parametrize("width", [88, 74])
def test_ragged_last_column_tile_as_its_own_launch(width):
    # 42 slices x 14 row tiles: the last column of the tile grid has more than 512 tiles, and the maps are 86 / 84
    # (width 88: two 16-column groups) or 72 / 70 wide (width 74: one group), so forward, data gradient (with the
    # ReLU mask fused) and their narrow launches all run; compared with the oracle like every other case
    layers = [S.conv(16, 3, 1), S.conv(8, 3, 1), S.conv(2, 1, 1, relu=False)]
    net, *_ = run_training(layers, 1, 2, (44, 108, width), 660 + width)
    net.close()


def test_gradients_converted_net_unmasked_and_wider_pool():
    layers = [S.conv(8, 3, 1), S.pool(3, 1), S.conv(12, 2, 3), S.conv(10, 1, 1), S.conv(2, 1, 1, relu=False)]
    net, *_ = run_training(layers, 1, 2, (12, 20, 70), 620, masked=False)
    net.close()


def test_sgd_step_updates_weights_and_packed_forms():
    layers = S.sknet3d_layers(classes=2, maps=(8, 16, 24, 12))
    net, vol, labels, ws, bs, dws, dbs = run_training(layers, 1, 2, (20, 24, 40), 630)
    lr, mu, wd = 0.05, 0.9, 1e-3
    net.sgd_step(lr, mu, wd)
    new_w, new_b = [], []
    for i in range(len(ws)):
        w64, b64 = ws[i].astype(np.float64), bs[i].astype(np.float64)
        OL.sgd(w64, dws[i], np.zeros_like(w64), lr, mu, wd)
        OL.sgd(b64, dbs[i], np.zeros_like(b64), lr, mu, wd)
        gw, gb = net.get_weights(i)
        assert relerr(gw, w64) <= 1e-5 and relerr(gb, b64) <= 1e-5, i
        new_w.append(gw)
        new_b.append(gb)
    # the next forward runs on the updated weights (packed forms rebuilt on the device)
    prob = net.forward(to_dev(vol)).cpu().numpy()
    ref = OND.sknet3d_forward(vol, layers, new_w, new_b)
    assert np.abs(prob.transpose(1, 0, 2, 3) - ref).max() <= FP32_TOL
    # a new plan keeps the trained weights
    net.plan(20, 24, 40)
    prob2 = net.forward(to_dev(vol)).cpu().numpy()
    assert np.abs(prob2.transpose(1, 0, 2, 3) - ref).max() <= FP32_TOL
    net.close()


def test_all_voxels_masked_gives_zero_loss_and_gradients():
    from paper_1509_03371_amd import binding as B
    layers = S.sknet3d_layers(classes=2, maps=(4, 4, 8, 4))
    ws, bs = S.he_normal_weights3d(layers, 1, 640, bias_scale=0.1)
    net = B.SKNet3D(layers, 1, 2)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    net.plan(19, 20, 21, training=True)
    net.forward(to_dev(S.uniform_volume(1, 19, 20, 21, 641)))
    loss = net.backward(torch.full((2, 3, 4), -1, dtype=torch.int32, device="cuda"))
    assert float(loss.cpu()) == 0.0
    for i in range(len(ws)):
        dw, db = net.get_grad(i)
        assert not dw.any() and not db.any()
    net.close()


def test_call_order_and_unsupported_training_plans():
    from paper_1509_03371_amd import binding as B
    layers = S.sknet3d_layers(classes=2, maps=(4, 4, 8, 4))
    net = B.SKNet3D(layers, 1, 2)
    labels = torch.zeros((2, 3, 4), dtype=torch.int32, device="cuda")
    net.plan(19, 20, 21)                                   # inference plan
    net.forward(torch.zeros((19, 1, 20, 21), device="cuda"))
    for call in (lambda: net.backward(labels), lambda: net.sgd_step(0.1), lambda: net.get_pool_argmax(0)):
        with pytest.raises(B.SknetError) as e:
            call()
        assert e.value.status_name == "SK_ESTATE"
    net.plan(19, 20, 21, training=True)
    with pytest.raises(B.SknetError) as e:
        net.backward(labels)                               # no forward on this plan yet
    assert e.value.status_name == "SK_ESTATE"
    with pytest.raises(B.SknetError) as e:
        net.get_grad(0)
    assert e.value.status_name == "SK_ESTATE"
    net.close()
    down = B.SKNet3D([S.conv(4, 3, 1), S.pool(2, 1, 2), S.conv(2, 1, 1, relu=False)], 1, 2)
    with pytest.raises(B.SknetError) as e:
        down.plan(10, 12, 14, training=True)
    assert e.value.status_name == "SK_EUNSUPPORTED"
    down.close()
