"""GPU parity: the SK pool that 16-bit inference plans run inside its neighbours (the convolution in front of
it stores max(Y[y], Y[y+d]), the layer behind it reads max(X[x], X[x+d])) against the oracle's separate
layers, OL.maxpool_sk(OL.conv_sk(..)): bit-exact on inputs both sides hold exactly, ties included; bitwise
equal to the plan that keeps every layer; within the 16-bit tolerance of the oracle on random weights."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import layers as OL, nets as ON

pytestmark = pytest.mark.gpu


def make_net(layers, c_in, ws, bs, dtype):
    from paper_1509_03371_amd import binding as B
    net = B.SKNet(layers, c_in, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    return net


def tap_weights(maps, tap):
    """A 4x4 convolution that copies map c of its input, shifted by the tap, to map c of its output."""
    w = np.zeros((maps, maps, 4, 4), np.float32)
    w[np.arange(maps), np.arange(maps), tap[0], tap[1]] = 1.0
    return w


def exact_image(n, c, h, w, seed):
    # multiples of 1/16 in [-1, 3): exact in bf16 and fp16, many equal neighbours, a quarter negative (ReLU -> ties at 0)
    return (np.random.default_rng(seed).integers(-16, 48, (n, c, h, w)) / 16.0).astype(np.float32)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("maps,d,n,h,w", [
    (48, 1, 2, 70, 300), (48, 2, 1, 150, 140), (48, 4, 2, 90, 260), (48, 8, 1, 200, 129),   # few tiles per workgroup: overlapping tiles
    (16, 2, 8, 520, 500), (32, 8, 6, 600, 520),                                             # long runs: rows carried from tile to tile
])
def test_fused_pool_bit_exact_on_exact_inputs(dtype, maps, d, n, h, w):
    """conv A (copies its input shifted by a tap) + ReLU, SK pool k2 at A's d, conv B (copies again), then a 1x1
    head.  Every value is a multiple of 1/16, so both sides pool identical numbers and the output of conv B must
    equal the oracle's pooled maps bit for bit -- across tile seams, run boundaries and the ragged last tiles."""
    layers = [S.conv(maps, 4, d, relu=True), S.pool(2, d), S.conv(maps, 4, d, relu=True), S.conv(24, 1, 1, relu=True),
              S.conv(2, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, maps, 41, bias_scale=0.1)
    ws[0], ws[1] = tap_weights(maps, (1, 2)), tap_weights(maps, (3, 1))      # indexed by convolution
    bs[0][:], bs[1][:] = 0, 0
    img = exact_image(n, maps, h, w, 42 + d)
    net = make_net(layers, maps, ws, bs, dtype)
    net.plan(n, h, w, pad=False)                          # inference plan: the pool runs inside conv A and conv B
    assert [net.step_name(i) for i in range(net.num_steps())][1:3] == ["conv0_k4_d%d_o%d_vpool" % (d, maps), "conv2_k4_d%d_o%d_hpool" % (d, maps)]
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    got = net.get_activation(2)
    with pytest.raises(Exception):
        net.get_activation(1)                             # the pool's output does not exist in this plan
    net.close()
    # the oracle's layers one by one (the tap convolutions through the definition they reduce to: a shifted copy;
    # OL.conv_sk itself is used on the smaller cases)
    x = img.astype(np.float64)
    if n * h * w <= 200000:
        a = OL.conv_sk(x, ws[0], bs[0], d, relu=True)
    else:
        a = np.maximum(x[:, :, d:h - 2 * d, 2 * d:w - d], 0)
    pooled, _ = OL.maxpool_sk(a, 2, d, 1)
    if n * h * w <= 200000:
        ref = OL.conv_sk(pooled, ws[1], bs[1], d, relu=True)
    else:
        ph, pw = pooled.shape[2:]
        ref = pooled[:, :, 3 * d:ph, d:pw - 2 * d]
    assert got.shape == ref.shape
    assert np.array_equal(got.astype(np.float64), ref), int((got != ref).sum())
    assert np.isfinite(prob).all()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_fused_pools_equal_the_plan_that_keeps_every_layer(dtype):
    """Random weights, three stages, two of them followed by pools: the last convolution's output must be the
    same bits whether the pools run as layers (plan mode 2) or inside their neighbours (mode 0) -- max is exact
    and the convolution's arithmetic does not depend on the plan -- and within the 16-bit bound of the oracle."""
    layers = [S.conv(48, 4, 1), S.pool(2, 1), S.conv(40, 4, 2), S.pool(2, 2), S.conv(48, 4, 4), S.conv(24, 1, 1), S.conv(2, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 1, 51, bias_scale=0.1)
    n, h, w = 2, 150, 330
    img = S.em_like_batch(n, h, w, 52)
    timg = torch.from_numpy(img).cuda()
    net = make_net(layers, 1, ws, bs, dtype)
    net.plan(n, h, w, pad=True)
    names = [net.step_name(i) for i in range(net.num_steps())]
    assert names == ["pad", "conv0_k4_d1_o48_vpool", "conv2_k4_d2_o40_hpool_vpool", "conv4_k4_d4_o48_hpool", "head_fused"], names
    prob0 = net.forward(timg).cpu().numpy()
    act0 = net.get_activation(4)
    net.plan(n, h, w, pad=True, keep=True)
    prob2 = net.forward(timg).cpu().numpy()
    act2 = net.get_activation(4)
    net.close()
    assert np.array_equal(act0, act2), int((act0 != act2).sum())
    ref_prob, acts, _ = ON.sknet_forward(img, layers, ws, bs, keep=True)
    assert np.abs(act0 - acts[5]).max() <= 2e-2 * np.abs(acts[5]).max()
    assert np.abs(prob0 - ref_prob).max() <= 2e-2 and np.abs(prob2 - ref_prob).max() <= 2e-2


def test_layers_the_fused_kernels_do_not_cover_keep_their_pool():
    # a 3x3 convolution in front of the pool, and a pool whose d differs from the convolution's: plain layers
    layers = [S.conv(16, 3, 1), S.pool(2, 1), S.conv(16, 4, 2), S.pool(2, 1), S.conv(16, 4, 2), S.conv(8, 1, 1), S.conv(2, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 1, 61, bias_scale=0.1)
    img = S.em_like_batch(1, 60, 80, 62)
    net = make_net(layers, 1, ws, bs, "bf16")
    net.plan(1, 60, 80, pad=True)
    names = [net.step_name(i) for i in range(net.num_steps())]
    assert not any("pool" in s and "conv" in s for s in names), names
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    net.close()
    assert np.abs(prob - ON.sknet_forward(img, layers, ws, bs)).max() <= 2e-2
