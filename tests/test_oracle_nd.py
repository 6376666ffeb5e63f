"""Pins of the 3-D oracle (oracle/nd.py) to things other than itself: hand-computed values, the library's
dilated 3-D convolution and pooling, the pinned 2-D oracle on a one-slice case, and the sliding-window
equivalence that Algorithm 1 promises, taken voxel by voxel on 3-D patches."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import sk_synth as S
from oracle import alg1, layers as L, nd


def test_hand_conv3d_k2_d2_corner_sum():
    # a 2x2x2 kernel of ones with kernel stride 2 adds the eight corners of a 3x3x3 cube; on the volume
    # X[z,y,x] = 100z + 10y + x that sum is 8 * (value at the cube's centre)
    D = H = W = 5
    z, y, x = np.meshgrid(np.arange(D), np.arange(H), np.arange(W), indexing="ij")
    vol = (100 * z + 10 * y + x)[None].astype(np.float64)
    out = nd.conv_sk3d(vol, np.ones((1, 1, 2, 2, 2)), np.array([0.5]), d=2)
    assert out.shape == (1, 3, 3, 3)
    centre = 100 * (z[:3, :3, :3] + 1) + 10 * (y[:3, :3, :3] + 1) + (x[:3, :3, :3] + 1)
    np.testing.assert_allclose(out[0], 8 * centre + 0.5, rtol=0, atol=1e-12)


def test_hand_conv3d_single_tap_selects_shifted_voxel():
    # one nonzero weight at tap (a,i,j) = (2,0,1), d = 3: Y[z,y,x] = 2 * X[z+6, y, x+3]; catches swapped axes
    rng = np.random.default_rng(3)
    vol = rng.standard_normal((1, 9, 8, 10))
    w = np.zeros((1, 1, 3, 3, 3))
    w[0, 0, 2, 0, 1] = 2.0
    out = nd.conv_sk3d(vol, w, None, d=3)
    assert out.shape == (1, 3, 2, 4)
    np.testing.assert_allclose(out[0], 2.0 * vol[0, 6:9, 0:2, 3:7], rtol=0, atol=1e-14)


@pytest.mark.parametrize("k,d", [(1, 1), (2, 1), (3, 2), (2, 4), (4, 1)])
def test_conv3d_matches_library_dilated_convolution(k, d):
    rng = np.random.default_rng(10 * k + d)
    ext = (k - 1) * d
    x = rng.standard_normal((3, ext + 4, ext + 5, ext + 3))
    w = rng.standard_normal((5, 3, k, k, k))
    b = rng.standard_normal(5)
    ours = nd.conv_sk3d(x, w, b, d, relu=True)
    ref = F.relu(F.conv3d(torch.from_numpy(x)[None], torch.from_numpy(w), torch.from_numpy(b), dilation=d))[0].numpy()
    np.testing.assert_allclose(ours, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("k,d,s", [(2, 1, 1), (2, 2, 1), (2, 4, 1), (3, 2, 1), (2, 1, 2), (3, 1, 3)])
def test_pool3d_matches_library_dilated_pool(k, d, s):
    rng = np.random.default_rng(100 * k + 10 * d + s)
    ext = (k - 1) * d + 1
    x = rng.standard_normal((2, ext + 4 * s, ext + 3 * s, ext + 5 * s))
    ours = nd.maxpool_sk3d(x, k, d, s)
    ref = F.max_pool3d(torch.from_numpy(x)[None], kernel_size=k, stride=s, dilation=d)[0].numpy()
    assert ours.shape == ref.shape
    np.testing.assert_array_equal(ours, ref)


def test_one_slice_output_reduces_to_the_2d_layers():
    # a volume exactly (k-1)d+1 slices deep has one output slice: the 2-D SK convolution whose input maps are
    # the (map, depth tap) pairs, and the 2-D SK pool of the element-wise maximum of the tapped slices
    rng = np.random.default_rng(5)
    k, d, c, f = 3, 2, 2, 4
    x = rng.standard_normal((c, (k - 1) * d + 1, 11, 12))
    w = rng.standard_normal((f, c, k, k, k))
    b = rng.standard_normal(f)
    y3 = nd.conv_sk3d(x, w, b, d)
    x2 = x[:, ::d].reshape(1, c * k, 11, 12)
    y2 = L.conv_sk(x2, w.reshape(f, c * k, k, k), b, d)
    np.testing.assert_allclose(y3[:, 0], y2[0], rtol=1e-12, atol=1e-12)
    p3 = nd.maxpool_sk3d(x, k, d)
    p2, _ = L.maxpool_sk(x[:, ::d].max(axis=1)[None], k, d)
    np.testing.assert_array_equal(p3[:, 0], p2[0])


def _sw_net_on_patch(patch, sw_layers, weights, biases):
    """The sliding-window net on one patch [c, w, w, w]: ordinary convolutions, pools with s = k, inner
    products over the whole remaining volume.  Returns the class scores."""
    x, wi = patch, 0
    for lay in sw_layers:
        if lay["type"] == "conv":
            x = nd.conv_sk3d(x, weights[wi], biases[wi], 1, lay["relu"])
            wi += 1
        elif lay["type"] == "pool":
            x = nd.maxpool_sk3d(x, lay["k"], 1, lay["s"])
        else:
            wgt = weights[wi]
            assert wgt.shape[2:] == x.shape[1:]
            x = np.tensordot(wgt, x, axes=([1, 2, 3, 4], [0, 1, 2, 3])) + biases[wi]
            if lay["relu"]:
                x = np.maximum(x, 0.0)
            x = x[:, None, None, None]
            wi += 1
    return x[:, 0, 0, 0]


def test_sk3d_equals_sliding_window_voxel_by_voxel():
    maps = (3, 4, 5, 3)
    sw = S.sw3d_layers(classes=2, maps=maps)
    sk, _, w_sk = alg1.convert_sw_to_sk(sw, 18)
    assert sk == S.sknet3d_layers(classes=2, maps=maps) and w_sk[-1] == 1
    v = alg1.context(sk)
    assert v == 17
    ws, bs = S.he_normal_weights3d(sk, 2, seed=11, bias_scale=0.1)
    ws = [w.astype(np.float64) for w in ws]
    bs = [b.astype(np.float64) for b in bs]
    out = (2, 3, 2)
    vol = np.random.default_rng(12).standard_normal((2, out[0] + v, out[1] + v, out[2] + v))
    prob, acts, _ = nd.sknet3d_forward(vol, sk, ws, bs, keep=True)
    scores = acts[-1]
    assert scores.shape == (2,) + out
    for z in range(out[0]):
        for y in range(out[1]):
            for x in range(out[2]):
                patch = vol[:, z:z + 18, y:y + 18, x:x + 18]
                ref = _sw_net_on_patch(patch, sw, ws, bs)
                np.testing.assert_allclose(scores[:, z, y, x], ref, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(prob.sum(axis=0), 1.0, rtol=0, atol=1e-12)
    e = np.exp(scores[:, 1, 2, 0] - scores[:, 1, 2, 0].max())
    np.testing.assert_allclose(prob[:, 1, 2, 0], e / e.sum(), rtol=1e-12)


def test_size_errors():
    with pytest.raises(ValueError):
        nd.conv_sk3d(np.zeros((1, 4, 9, 9)), np.zeros((1, 1, 3, 3, 3)), None, d=2)
    with pytest.raises(ValueError):
        nd.maxpool_sk3d(np.zeros((1, 9, 2, 9)), 2, 2)


def test_pool3d_argmax_points_at_the_first_maximum():
    rng = np.random.default_rng(8)
    x = rng.integers(0, 3, size=(2, 7, 8, 9)).astype(np.float64)      # many ties
    k, d = 2, 2
    y, arg = nd.maxpool_sk3d(x, k, d, want_argmax=True)
    flat = x.reshape(2, -1)
    np.testing.assert_array_equal(np.take_along_axis(flat, arg.reshape(2, -1), axis=1).reshape(y.shape), y)
    # brute force: the first tap in (a, i, j) order that attains the maximum
    for (m, z, yy, xx) in [(0, 0, 0, 0), (1, 4, 5, 6), (0, 2, 3, 1), (1, 1, 0, 6)]:
        taps = [((z + a * d) * 8 + yy + i * d) * 9 + xx + j * d for a in range(k) for i in range(k) for j in range(k)]
        vals = [flat[m, t] for t in taps]
        assert arg[m, z, yy, xx] == taps[int(np.argmax(vals))]       # np.argmax returns the first maximum
    # a constant volume: every window's first tap wins
    _, arg0 = nd.maxpool_sk3d(np.ones((1, 5, 5, 5)), 2, 1, want_argmax=True)
    assert arg0[0, 1, 2, 3] == (1 * 5 + 2) * 5 + 3


def _torch_net(vol, layers, ws, bs):
    x, wi = vol[None], 0
    for lay in layers:
        if lay["type"] == "conv":
            x = F.conv3d(x, ws[wi], bs[wi], dilation=lay["d"])
            if lay.get("relu", False):
                x = F.relu(x)
            wi += 1
        else:
            x = F.max_pool3d(x, kernel_size=lay["k"], stride=lay.get("s", 1), dilation=lay["d"])
    return x[0]


def test_net_backward_matches_reverse_mode_differentiation_and_finite_differences():
    layers = S.sknet3d_layers(classes=3, maps=(3, 4, 5, 4))
    ws, bs = S.he_normal_weights3d(layers, 2, seed=21, bias_scale=0.1)
    ws = [w.astype(np.float64) for w in ws]
    bs = [b.astype(np.float64) for b in bs]
    vol = np.random.default_rng(22).standard_normal((2, 19, 20, 21))
    labels = np.random.default_rng(23).integers(-1, 3, size=(2, 3, 4))       # some voxels masked
    prob, acts, argmaxes = nd.sknet3d_forward(vol, layers, ws, bs, keep=True)
    loss, dws, dbs = nd.sknet3d_backward(layers, ws, acts, argmaxes, labels)
    tw = [torch.from_numpy(w).requires_grad_(True) for w in ws]
    tb = [torch.from_numpy(b).requires_grad_(True) for b in bs]
    z = _torch_net(torch.from_numpy(vol), layers, tw, tb)
    lab = torch.from_numpy(labels)
    ref = F.cross_entropy(z[None], lab[None].long(), ignore_index=-1, reduction="mean")
    ref.backward()
    assert abs(loss - ref.item()) <= 1e-12 * max(1.0, abs(ref.item()))
    for i in range(len(ws)):
        np.testing.assert_allclose(dws[i], tw[i].grad.numpy(), rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(dbs[i], tb[i].grad.numpy(), rtol=1e-9, atol=1e-12)
    # central difference on one weight of the dilated middle convolution
    idx, eps = (2, 1, 2, 0, 1), 1e-6
    vals = []
    for sgn in (1, -1):
        w2 = [w.copy() for w in ws]
        w2[1][idx] += sgn * eps
        _, a2, _ = nd.sknet3d_forward(vol, layers, w2, bs, keep=True)
        vals.append(nd.softmax_loss3d(a2[-1], labels)[0])
    assert abs((vals[0] - vals[1]) / (2 * eps) - dws[1][idx]) <= 1e-6 * max(1.0, abs(dws[1][idx]))


def test_loss3d_all_masked_and_closed_form():
    z = np.zeros((4, 2, 2, 2))
    loss, dz = nd.softmax_loss3d(z, np.full((2, 2, 2), -1))
    assert loss == 0.0 and not dz.any()
    lab = np.zeros((2, 2, 2), dtype=np.int64)
    lab[0, 0, 0] = -1
    loss, dz = nd.softmax_loss3d(z, lab)
    assert abs(loss - np.log(4.0)) <= 1e-15                   # uniform scores: -log(1/4) whatever the count
    np.testing.assert_allclose(dz[:, 1, 1, 1], np.array([0.25 - 1, 0.25, 0.25, 0.25]) / 7)
    assert not dz[:, 0, 0, 0].any()
