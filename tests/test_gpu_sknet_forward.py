"""GPU parity: SK-Net forward through the C ABI against the fp64 CPU oracle, same seeded inputs."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import layers as OL, nets as ON

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4   # max|gpu - ref| / max|ref| per tensor, fp32 path


def relerr(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def make_net(layers, c_in, ws, bs, **kw):
    from paper_1509_03371_amd import binding as B
    classes = [l for l in layers if l["type"] == "conv"][-1]["f_out"] if any(l["type"] == "conv" for l in layers) else c_in
    net = B.SKNet(layers, c_in, classes, **kw)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    return net


def run_and_compare(layers, c_in, img, ws, bs, pad=True, pad_mode=0, tol=FP32_TOL):
    net = make_net(layers, c_in, ws, bs, pad_mode=pad_mode)
    n, _, h, w = img.shape
    net.plan(n, h, w, pad=pad, keep=True)
    prob = net.forward(torch.from_numpy(img).cuda())
    torch.cuda.synchronize()
    ref_prob, acts, _ = ON.sknet_forward(img, layers, ws, bs, pad=pad, pad_mode=pad_mode, keep=True)
    assert np.array_equal(net.get_activation(-1).astype(np.float64), acts[0])      # padding is a copy: exact
    for li in range(len(layers)):
        got = net.get_activation(li)
        assert got.shape == acts[li + 1].shape
        assert relerr(got, acts[li + 1]) <= tol, ("layer", li, layers[li])
    got = prob.cpu().numpy()
    assert got.shape == ref_prob.shape
    assert np.abs(got - ref_prob).max() <= tol
    # the inference plan (mode 0) may fuse layers: same probabilities
    net.plan(n, h, w, pad=pad)
    fused = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    assert np.abs(fused - ref_prob).max() <= tol
    net.close()
    return got, ref_prob


def test_c1_tiny_sknet_forward():
    layers = S.tiny_sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1000)
    img = S.uniform_image(1, 1, 96, 96, 0)
    got, ref = run_and_compare(layers, 1, img, ws, bs)
    assert got.shape == (1, 2, 96, 96)
    assert np.abs(got.sum(1) - 1).max() < 1e-5


@pytest.mark.parametrize("k,d,c_in,c_out,h,w", [
    (4, 1, 1, 48, 70, 90), (4, 2, 48, 48, 41, 131), (4, 8, 48, 48, 57, 66), (5, 2, 8, 16, 33, 29),
    (3, 1, 64, 128, 20, 23), (1, 1, 48, 200, 19, 70), (1, 1, 200, 2, 19, 70), (3, 4, 3, 5, 30, 40),
    (2, 3, 5, 7, 9, 200), (7, 1, 3, 48, 25, 25), (4, 8, 6, 4, 25, 25), (10, 2, 4, 20, 30, 24),
    # the large kernels of the USK-Net and of the paper's SK-Net: map counts off the chunk of four, several map blocks
    (6, 1, 10, 40, 30, 75), (6, 3, 5, 70, 40, 90), (8, 8, 12, 130, 70, 140), (8, 2, 3, 16, 33, 29), (10, 8, 6, 50, 90, 160),
])
def test_conv_layer_shapes(k, d, c_in, c_out, h, w):
    """One SK convolution (+bias +ReLU) per case: several tiles, ragged tails, a row-phase count
    that does not divide the map, map counts that are not multiples of the MFMA tile."""
    layers = [S.conv(c_out, k, d, relu=True)]
    ws, bs = S.he_normal_weights(layers, c_in, 7 + k + d, bias_scale=0.5)
    img = np.random.default_rng(3).standard_normal((2, c_in, h, w)).astype(np.float32)
    net = make_net(layers, c_in, ws, bs)
    net.plan(2, h, w, pad=False, keep=True)
    net.forward(torch.from_numpy(img).cuda())
    got = net.get_activation(0)
    ref = OL.conv_sk(img, ws[0], bs[0], d, relu=True)
    assert got.shape == ref.shape
    assert relerr(got, ref) <= FP32_TOL
    net.close()


@pytest.mark.parametrize("k,d,s,h,w", [(2, 1, 1, 33, 70), (2, 2, 1, 40, 131), (2, 8, 1, 57, 66), (3, 2, 1, 20, 21),
                                       (2, 1, 2, 30, 62), (2, 4, 1, 9, 300)])
def test_pool_values_and_argmax_bit_exact(k, d, s, h, w):
    """Max pooling is exact in any precision: identical fp32 inputs -> identical values and winners,
    including the tie rule (many exact zeros, as after a ReLU)."""
    layers = [S.pool(k, d, s)]
    rng = np.random.default_rng(11)
    img = np.maximum(rng.standard_normal((2, 3, h, w)), 0).astype(np.float32)      # about half zeros
    net = make_net(layers, 3, [], [])
    net.plan(2, h, w, pad=False, training=(s == 1))
    net.forward(torch.from_numpy(img).cuda())
    ref, ref_am = OL.maxpool_sk(img, k, d, s)
    assert np.array_equal(net.get_activation(0).astype(np.float64), ref)
    if s == 1:
        assert np.array_equal(net.get_pool_argmax(0), ref_am)
    net.close()


@pytest.mark.parametrize("mode", [0, 1])
def test_mirror_pad_modes_and_odd_context(mode):
    layers = [S.conv(4, 4, 1), S.pool(2, 1), S.conv(3, 1, 1, relu=False)]        # v = 4 (even)
    layers_odd = [S.conv(4, 3, 1), S.pool(2, 1), S.conv(3, 2, 2, relu=False)]    # v = 2 + 1 + 2 = 5 (odd)
    for lay in (layers, layers_odd):
        ws, bs = S.he_normal_weights(lay, 2, 21, bias_scale=0.2)
        img = S.uniform_image(2, 2, 17, 23, 5)
        got, ref = run_and_compare(lay, 2, img, ws, bs, pad=True, pad_mode=mode)
        assert got.shape == (2, 3, 17, 23)


def test_softmax_many_classes():
    layers = [S.conv(9, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 4, 33, bias_scale=1.0)
    img = (np.random.default_rng(4).standard_normal((1, 4, 31, 37)) * 3).astype(np.float32)
    run_and_compare(layers, 4, img, ws, bs, pad=False)


@pytest.mark.parametrize("c_in,hidden,classes,h,w", [(48, 200, 2, 37, 53), (16, 32, 2, 20, 70), (5, 100, 3, 9, 200),
                                                       (130, 256, 8, 17, 19), (48, 7, 4, 33, 31)])
def test_fused_head_matches_oracle(c_in, hidden, classes, h, w):
    """1x1 conv + ReLU, 1x1 conv, softmax as one kernel (inference plan): probabilities against the
    oracle, and the layers are reported as not materialised."""
    from paper_1509_03371_amd import binding as B
    layers = [S.conv(hidden, 1, 1, relu=True), S.conv(classes, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, c_in, 55, bias_scale=0.3)
    img = np.random.default_rng(8).standard_normal((3, c_in, h, w)).astype(np.float32)
    net = make_net(layers, c_in, ws, bs)
    net.plan(3, h, w, pad=False)
    assert [net.step_name(i) for i in range(net.num_steps())] == ["pad", "head_fused"]
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    ref = ON.sknet_forward(img, layers, ws, bs, pad=False)
    assert np.abs(prob - ref).max() <= FP32_TOL
    with pytest.raises(B.SknetError) as e:
        net.get_activation(0)
    assert e.value.status_name == "SK_ESTATE"
    net.set_weights(0, ws[0] * 0.5, bs[0])          # re-packing after a weight change
    prob2 = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    ref2 = ON.sknet_forward(img, layers, [ws[0] * 0.5, ws[1]], bs, pad=False)
    assert np.abs(prob2 - ref2).max() <= FP32_TOL
    net.close()


def test_tile_and_stitch_on_gpu():
    """Output-size invariance (Section 3.1): four tiles with a context halo reproduce the whole image."""
    layers = S.tiny_sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1000)
    img = S.uniform_image(1, 1, 40, 40, 9)
    whole_net = make_net(layers, 1, ws, bs)
    whole_net.plan(1, 40, 40, pad=True)
    whole = whole_net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    padded = whole_net.get_activation(-1)
    v = whole_net.context()
    tile_net = make_net(layers, 1, ws, bs)
    tile_net.plan(1, 20 + v, 20 + v, pad=False)
    stitched = np.empty_like(whole)
    for y0 in (0, 20):
        for x0 in (0, 20):
            tile = np.ascontiguousarray(padded[:, :, y0:y0 + 20 + v, x0:x0 + 20 + v])
            stitched[:, :, y0:y0 + 20, x0:x0 + 20] = tile_net.forward(torch.from_numpy(tile).cuda()).cpu().numpy()
    assert np.abs(stitched - whole).max() <= 2e-6
    whole_net.close()
    tile_net.close()


def test_c2_sknet_forward_512():
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    img = S.em_like_batch(1, 512, 512, 2)
    got, ref = run_and_compare(layers, 1, img, ws, bs)
    assert got.shape == (1, 2, 512, 512)


def test_paper_sknet_configuration_forward():
    # the network of Section 3.3.2's SK table (k = 7, 5, 3 and the k = 10, d = 8 inner product, context 101,
    # odd: 51 rows/columns of mirror padding before, 50 after) on a small 3-channel image
    layers = S.paper_sknet_layers()
    ws, bs = S.he_normal_weights(layers, 3, 1003, bias_scale=0.05)
    img = S.uniform_image(1, 3, 60, 68, 11)          # reflect padding by 51 needs at least 52 rows/columns
    got, ref = run_and_compare(layers, 3, img, ws, bs)
    assert got.shape == (1, 2, 60, 68)
