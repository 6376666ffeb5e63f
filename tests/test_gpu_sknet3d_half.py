"""GPU parity: 3-D SK net forward (Section 5.2.2) in 16-bit storage (bf16 / fp16 activations in the slice-major octet
layout, fp32 accumulation) against the fp64 oracle on the unrounded fp32 weights and volume: 2e-2 of a layer's largest
value on every activation and on the probabilities; pools exact on the library's own 16-bit input."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import nd as OND

pytestmark = pytest.mark.gpu

HALF_TOL = 2e-2


def relerr(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def make_net(layers, c_in, classes, seed, dtype, bias_scale=0.1):
    from paper_1509_03371_amd import binding as B
    ws, bs = S.he_normal_weights3d(layers, c_in, seed, bias_scale=bias_scale)
    net = B.SKNet3D(layers, c_in, classes, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    return net, ws, bs


def check_layers(layers, c_in, classes, size, seed, dtype):
    net, ws, bs = make_net(layers, c_in, classes, seed, dtype)
    dz, h, w = size
    vol = S.uniform_volume(c_in, dz, h, w, seed + 1) - 0.3
    net.plan(dz, h, w, keep=True)
    dev = torch.from_numpy(np.ascontiguousarray(vol.transpose(1, 0, 2, 3))).cuda()
    prob = net.forward(dev).cpu().numpy()
    ref, acts, _ = OND.sknet3d_forward(vol, layers, ws, bs, keep=True)
    for i in range(len(layers)):
        got = net.get_activation(i).transpose(1, 0, 2, 3)
        assert got.shape == acts[i + 1].shape, i
        e = relerr(got, acts[i + 1])
        print(dtype, "sk3d layer %d %s %s rel err %.3e" % (i, layers[i]["type"], got.shape, e), flush=True)
        if layers[i]["type"] == "pool" and i > 0:
            src = net.get_activation(i - 1).transpose(1, 0, 2, 3)
            np.testing.assert_array_equal(got, OND.maxpool_sk3d(src, layers[i]["k"], layers[i]["d"], layers[i].get("s", 1)).astype(np.float32))
        assert e <= HALF_TOL, (i, e)
    assert np.abs(prob.transpose(1, 0, 2, 3) - ref).max() <= HALF_TOL
    net.close()
    return prob


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_converted_net_layer_by_layer_ragged_volume_half(dtype):
    # the Algorithm-1 conversion of the 18^3 sliding-window net: d = 1, 2 and 4 (the loader steps over the slices between
    # two depth taps), map counts off the octet
    layers = S.sknet3d_layers(classes=3, maps=(8, 12, 24, 20))
    prob = check_layers(layers, 2, 3, (22, 38, 87), 500, dtype)
    assert prob.shape == (5, 3, 21, 70)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_four_by_four_kernels_and_many_maps_half(dtype):
    # 4^3 kernels (lane groups on tap columns, one input octet per chunk) at d = 4 after 3^3 layers with 16 and 32 maps
    layers = [S.conv(16, 3, 1), S.pool(2, 1), S.conv(32, 3, 2), S.pool(2, 2), S.conv(24, 4, 4), S.conv(2, 1, 1, relu=False)]
    prob = check_layers(layers, 1, 2, (24, 29, 83), 505, dtype)
    assert prob.shape == (3, 2, 8, 62)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_single_input_map_odd_map_counts_general_pools_half(dtype):
    layers = [S.conv(5, 2, 1), S.pool(2, 1), S.conv(7, 2, 2), S.pool(2, 2), S.conv(9, 3, 4), S.conv(2, 1, 1, relu=False)]
    prob = check_layers(layers, 1, 2, (17, 30, 41), 510, dtype)
    assert prob.shape == (3, 2, 16, 27)
    layers = [S.conv(6, 3, 1), S.pool(3, 2), S.conv(8, 2, 1), S.pool(2, 1, 2), S.conv(4, 2, 1), S.conv(2, 1, 1, relu=False)]
    prob = check_layers(layers, 2, 2, (15, 21, 27), 520, dtype)
    assert prob.shape == (3, 2, 6, 9)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_fused_head_plan_and_new_weights_half(dtype):
    from paper_1509_03371_amd import binding as B
    layers = S.sknet3d_layers(classes=2, maps=(8, 16, 32, 24))
    net, ws, bs = make_net(layers, 1, 2, 530, dtype)
    vol = S.em_like_volume(25, 49, 60, 531)
    dev = torch.from_numpy(np.ascontiguousarray(vol.transpose(1, 0, 2, 3))).cuda()
    net.plan(25, 49, 60)
    prob = net.forward(dev).cpu().numpy()
    assert prob.shape == (8, 2, 32, 43)
    assert np.abs(prob.transpose(1, 0, 2, 3) - OND.sknet3d_forward(vol, layers, ws, bs)).max() <= HALF_TOL
    ws2, bs2 = S.he_normal_weights3d(layers, 1, 532, bias_scale=0.1)
    for i, (w, b) in enumerate(zip(ws2, bs2)):
        net.set_weights(i, w, b)
    prob2 = net.forward(dev).cpu().numpy()
    assert np.abs(prob2.transpose(1, 0, 2, 3) - OND.sknet3d_forward(vol, layers, ws2, bs2)).max() <= HALF_TOL
    net.close()


def test_benchmark_volume_sampled_against_oracle_bf16():
    # the benchmark's configuration and launch shapes (81 x 145 x 145 in, 64 x 128 x 128 out), blocks recomputed by the oracle
    layers = S.sknet3d_layers(classes=2)
    net, ws, bs = make_net(layers, 1, 2, 1100, "bf16", bias_scale=0.0)
    v = net.context()
    dz, h, w = 64 + v, 128 + v, 128 + v
    vol = S.em_like_volume(dz, h, w, 1101)
    net.plan(dz, h, w)
    prob = net.forward(torch.from_numpy(np.ascontiguousarray(vol.transpose(1, 0, 2, 3))).cuda()).cpu().numpy()
    assert prob.shape == (64, 2, 128, 128)
    for (z, y, x) in [(0, 0, 0), (62, 126, 126), (31, 64, 63), (5, 126, 17), (62, 0, 100)]:
        ref = OND.sknet3d_forward(vol[:, z:z + 2 + v, y:y + 2 + v, x:x + 2 + v], layers, ws, bs)
        got = prob[z:z + 2, :, y:y + 2, x:x + 2].transpose(1, 0, 2, 3)
        assert np.abs(got - ref).max() <= HALF_TOL, (z, y, x)
    net.close()
