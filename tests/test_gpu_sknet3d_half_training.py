"""GPU parity: 3-D SK net training pass in 16-bit storage (bf16 / fp16 activations and error maps in the slice-major
octet layout, fp32 sums, fp32 weight gradients and master weights) through the C ABI against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import nd as OND

pytestmark = pytest.mark.gpu

# The bounds of the 2-D 16-bit training tests: one rounding to the storage type per activation and per error map, ReLU and
# pool decisions that fall differently from fp64 for values within a rounding step, and (fp16) error maps that carry the
# loss's 1 / (labelled voxels) into the subnormal range.  A wrong index moves a tensor by tens of per cent.
TOL = {"bf16": 8e-2, "f16": 3e-2}
PROB_TOL = 2e-2


def relerr(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def to_dev(vol):
    return torch.from_numpy(np.ascontiguousarray(vol.transpose(1, 0, 2, 3))).cuda()


def run_training(layers, c_in, classes, size, seed, dtype, masked=True):
    from paper_1509_03371_amd import binding as B
    ws, bs = S.he_normal_weights3d(layers, c_in, seed, bias_scale=0.1)
    net = B.SKNet3D(layers, c_in, classes, dtype=dtype)
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
    assert np.abs(prob.transpose(1, 0, 2, 3) - ref_prob).max() <= PROB_TOL
    assert abs(loss - ref_loss) <= PROB_TOL * max(1.0, abs(ref_loss)), (loss, ref_loss)
    # pool winners: exact on the library's own 16-bit input (a pool only selects; widening is exact)
    pools = [i for i, l in enumerate(layers) if l["type"] == "pool"]
    for pi, li in enumerate(pools):
        src = net.get_activation(li - 1).transpose(1, 0, 2, 3)
        _, am = OND.maxpool_sk3d(src, layers[li]["k"], layers[li]["d"], layers[li].get("s", 1), want_argmax=True)
        np.testing.assert_array_equal(net.get_pool_argmax(pi).transpose(1, 0, 2, 3), am.astype(np.int32))
    errs = []
    for i in range(len(ws)):
        dw, db = net.get_grad(i)
        assert np.abs(dws[i]).max() > 0, "degenerate test net: a reference gradient is all zero"
        ew = relerr(dw, dws[i])
        eb = float(np.abs(db - dbs[i]).max() / max(np.abs(dbs[i]).max(), np.abs(dws[i]).max()))
        errs.append((i, ew, eb))
        print("sk3d %s conv %d %s dW rel err %.3e  db err %.3e" % (dtype, i, dw.shape, ew, eb), flush=True)
    for i, ew, eb in errs:
        assert ew <= TOL[dtype] and eb <= TOL[dtype], (i, ew, eb)
    return net, vol, labels, ws, bs


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_gradients_sixteen_map_multiples(dtype):
    # 16 / 32 maps, kernel strides 1, 2 and 4 (depth taps 1, 2 and 4 slices apart), pools between
    layers = [S.conv(16, 3, 1), S.pool(2, 1), S.conv(32, 3, 2), S.pool(2, 2), S.conv(16, 2, 4), S.conv(2, 1, 1, relu=False)]
    net, *_ = run_training(layers, 1, 2, (20, 27, 80), 610, dtype)
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_gradients_odd_map_counts(dtype):
    # 5 / 7 / 9 maps: octets padded with zero maps in every layer, two input maps, three classes
    layers = [S.conv(5, 2, 1), S.pool(2, 1), S.conv(7, 2, 2), S.pool(2, 2), S.conv(9, 3, 4), S.conv(3, 1, 1, relu=False)]
    net, *_ = run_training(layers, 2, 3, (18, 30, 75), 600, dtype)
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_gradients_benchmark_net_map_counts(dtype):
    # the benchmark's net (16 / 32 / 128 / 64 maps, context 17) on a volume the oracle finishes in seconds
    layers = S.sknet3d_layers(classes=2)
    net, *_ = run_training(layers, 1, 2, (25, 40, 150), 650, dtype)
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_gradients_three_octets_per_depth_tap(dtype):
    # 20 input maps = three octets per depth tap: the merged weight gradient's map pairs straddle two depth taps, and
    # with kernel stride 2 every third octet jumps to the next tapped slice; the third layer has 12 maps = two octets
    layers = [S.conv(20, 3, 1), S.pool(2, 1), S.conv(12, 3, 2), S.conv(24, 2, 2), S.conv(2, 1, 1, relu=False)]
    net, *_ = run_training(layers, 3, 2, (16, 26, 90), 630, dtype)
    net.close()


def test_gradients_wider_pool_unmasked_bf16():
    layers = [S.conv(8, 3, 1), S.pool(3, 1), S.conv(12, 2, 3), S.conv(10, 1, 1), S.conv(2, 1, 1, relu=False)]
    net, *_ = run_training(layers, 1, 2, (12, 20, 70), 620, "bf16", masked=False)
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_sgd_step_repacks_the_16_bit_weights(dtype):
    from paper_1509_03371_amd import binding as B
    layers = S.sknet3d_layers(classes=2, maps=(8, 16, 24, 12))
    net, vol, labels, ws, bs = run_training(layers, 1, 2, (20, 24, 40), 630, dtype)
    before = [net.get_weights(i) for i in range(len(ws))]
    grads = [net.get_grad(i) for i in range(len(ws))]
    lr = np.float32(0.02)
    net.sgd_step(float(lr))
    after = [net.get_weights(i) for i in range(len(ws))]
    for i in range(len(ws)):
        assert np.abs(after[i][0] - (before[i][0] - lr * grads[i][0])).max() <= 1e-6
        assert np.abs(after[i][1] - (before[i][1] - lr * grads[i][1])).max() <= 1e-6
    # the next passes run on the re-packed weights: same result as a fresh net given the updated masters
    dev = to_dev(vol)
    prob1 = net.forward(dev).cpu().numpy()
    net.backward(torch.from_numpy(labels).cuda())
    g1 = net.get_grad(0)[0]
    fresh = B.SKNet3D(layers, 1, 2, dtype=dtype)
    for i in range(len(ws)):
        fresh.set_weights(i, *after[i])
    fresh.plan(20, 24, 40, training=True)
    assert np.array_equal(prob1, fresh.forward(dev).cpu().numpy())
    fresh.backward(torch.from_numpy(labels).cuda())
    assert np.array_equal(g1, fresh.get_grad(0)[0])
    fresh.close()
    net.close()
