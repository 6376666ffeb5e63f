"""GPU parity of the 16-bit (bf16 / fp16 storage, fp32 accumulate) SK-Net path against the fp64
oracle.  The oracle runs on the unrounded fp32 weights and images, so the error measured here
contains every rounding of the 16-bit path.  Tolerance: 2e-2 of the tensor's largest magnitude on
activations and logits (the spec bar for bf16/fp16); pooling is exact on identical inputs."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import layers as OL, nets as ON

pytestmark = pytest.mark.gpu

HALF_TOL = 2e-2


def relerr(got, ref):
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def make_net(layers, c_in, ws, bs, dtype):
    from paper_1509_03371_amd import binding as B
    convs = [l for l in layers if l["type"] == "conv"]
    net = B.SKNet(layers, c_in, convs[-1]["f_out"] if convs else c_in, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    return net


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("k,d,c_in,c_out,h,w", [
    (4, 1, 1, 48, 70, 150), (4, 2, 48, 48, 41, 131), (4, 8, 48, 48, 57, 300), (4, 4, 48, 48, 100, 129),
    (3, 1, 64, 128, 20, 23), (1, 1, 48, 200, 19, 70), (1, 1, 200, 2, 19, 140), (3, 4, 3, 5, 30, 40),
    (2, 3, 5, 7, 9, 200), (4, 8, 6, 4, 25, 25), (4, 2, 20, 72, 30, 135), (3, 2, 40, 48, 33, 260),
    # kernels beyond 4x4 (the paper's SK-Net: 7x7, 5x5 d2, 10x10 d8; the USK-Net: 6x6, 8x8 d8): lane groups on four
    # consecutive kernel columns, the columns past the kernel carry zero weights; ragged maps, several map blocks
    (5, 2, 8, 16, 33, 29), (5, 2, 48, 128, 40, 150), (6, 1, 10, 40, 30, 75), (6, 3, 5, 70, 40, 90), (7, 1, 3, 48, 25, 140),
    (8, 8, 12, 130, 70, 140), (8, 2, 3, 16, 33, 29), (10, 8, 6, 50, 90, 160), (10, 2, 4, 20, 30, 24), (10, 8, 24, 40, 80, 210),
    # 2x2 / 3x3 layers large enough for the launcher to prefer a squarer tile (fewer rounds of one tile per CU on 256
    # CUs): 64 x 8 pixels (600 x 192 outputs, d = 1 and d = 3), 32 x 16 pixels (550 x 70 outputs, d = 2)
    (3, 1, 16, 16, 602, 194), (2, 3, 8, 16, 603, 195), (3, 2, 16, 24, 554, 74),
    # ... and 6x6 / 8x8 / 10x10 layers that take the 64 x 8 tile (staged rows of two and of three 64-unit groups)
    (6, 3, 5, 70, 315, 207), (8, 8, 12, 130, 176, 248), (10, 8, 6, 50, 352, 264),
])
def test_conv_layer_shapes_half(dtype, k, d, c_in, c_out, h, w):
    dt = "f16" if dtype == "fp16" else dtype
    layers = [S.conv(c_out, k, d, relu=True), S.conv(c_out, 1, 1, relu=False)]   # 2nd conv: identity, exposes layer 0
    ws, bs = S.he_normal_weights(layers[:1], c_in, 7 + k + d, bias_scale=0.5)
    ws.append(np.eye(c_out, dtype=np.float32).reshape(c_out, c_out, 1, 1))
    bs.append(np.zeros(c_out, np.float32))
    img = np.random.default_rng(3).standard_normal((2, c_in, h, w)).astype(np.float32)
    net = make_net(layers, c_in, ws, bs, dt)
    net.plan(2, h, w, pad=False, keep=True)
    net.forward(torch.from_numpy(img).cuda())
    ref = OL.conv_sk(img, ws[0], bs[0], d, relu=True)
    got0 = net.get_activation(0)          # stored in 16 bits
    got1 = net.get_activation(1)          # fp32 logits of the identity conv on the stored values
    assert got0.shape == ref.shape
    assert relerr(got0, ref) <= HALF_TOL
    assert np.abs(got1 - got0).max() <= 1e-6 * max(1.0, np.abs(got0).max())
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("k,d,s,h,w", [(2, 1, 1, 33, 70), (2, 2, 1, 40, 131), (2, 8, 1, 57, 66), (3, 2, 1, 20, 21),
                                       (2, 1, 2, 30, 62), (2, 4, 1, 9, 300)])
def test_pool_bit_exact_half(dtype, k, d, s, h, w):
    layers = [S.pool(k, d, s)]
    rng = np.random.default_rng(11)
    img = np.maximum(rng.standard_normal((2, 11, h, w)), 0).astype(np.float32)
    net = make_net(layers, 11, [], [], dtype)
    net.plan(2, h, w, pad=False, training=(s == 1))
    net.forward(torch.from_numpy(img).cuda())
    stored = net.get_activation(-1)                       # the input as the library holds it (rounded to 16 bits)
    assert relerr(stored, img) <= 2.0 ** -8
    ref, ref_am = OL.maxpool_sk(stored, k, d, s)
    assert np.array_equal(net.get_activation(0).astype(np.float64), ref)
    if s == 1:
        assert np.array_equal(net.get_pool_argmax(0), ref_am)
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_small_sknet_forward_half(dtype):
    layers = S.sknet_layers(width=48, hidden=200)
    ws, bs = S.he_normal_weights(layers, 1, 1001, bias_scale=0.05)
    img = S.em_like_batch(2, 100, 140, 20)
    net = make_net(layers, 1, ws, bs, dtype)
    net.plan(2, 100, 140, pad=True, keep=True)
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    ref_prob, acts, _ = ON.sknet_forward(img, layers, ws, bs, keep=True)
    for li in range(len(layers)):
        got = net.get_activation(li)
        assert got.shape == acts[li + 1].shape
        assert relerr(got, acts[li + 1]) <= HALF_TOL, (li, layers[li])
    assert np.abs(prob - ref_prob).max() <= HALF_TOL
    assert np.abs(prob.sum(1) - 1).max() < 1e-5
    net.plan(2, 100, 140, pad=True)                     # inference plan: fused head
    assert net.step_name(net.num_steps() - 1) == "head_fused"
    fused = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    assert np.abs(fused - ref_prob).max() <= HALF_TOL
    net.close()


def test_mirror_pad_fused_into_packing():
    layers = [S.conv(4, 3, 1), S.pool(2, 1), S.conv(3, 2, 2, relu=False)]     # odd context v = 5
    ws, bs = S.he_normal_weights(layers, 2, 21, bias_scale=0.2)
    img = S.uniform_image(2, 2, 17, 23, 5)
    for mode in (0, 1):
        from paper_1509_03371_amd import binding as B
        net = B.SKNet(layers, 2, 3, dtype="bf16", pad_mode=mode)
        for i, (w, b) in enumerate(zip(ws, bs)):
            net.set_weights(i, w, b)
        net.plan(2, 17, 23, pad=True)
        prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
        ref = ON.sknet_forward(img, layers, ws, bs, pad_mode=mode)
        assert np.abs(prob - ref).max() <= HALF_TOL
        padded = net.get_activation(-1)
        rounded = torch.from_numpy(OL.mirror_pad(img, 3, 3, 2, 2, mode).astype(np.float32)).bfloat16().float().numpy()
        assert np.array_equal(padded, rounded)                  # padding is a copy; conversion is round-to-nearest-even
        net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_training_step_half(dtype):
    layers = S.sknet_layers(width=48, hidden=200)
    ws, bs = S.he_normal_weights(layers, 1, 1001, bias_scale=0.05)
    img = S.em_like_batch(1, 96, 130, 30)
    labels = S.binary_labels(1, 96, 130, 31)
    net = make_net(layers, 1, ws, bs, dtype)
    net.plan(1, 96, 130, pad=True, training=True)
    net.forward(torch.from_numpy(img).cuda())
    loss = net.backward(torch.from_numpy(labels).cuda())
    ow = [x.astype(np.float64) for x in ws]
    ob = [x.astype(np.float64) for x in bs]
    _, acts, ams = ON.sknet_forward(img, layers, ow, ob, keep=True)
    ref_loss, dws, dbs, _ = ON.sknet_backward(layers, ow, acts, ams, labels)
    assert abs(loss.item() - ref_loss) <= HALF_TOL * abs(ref_loss)
    worst = 0.0
    for i in range(net.num_convs()):
        dw, db = net.get_grad(i)
        worst = max(worst, relerr(dw, dws[i]))
        assert relerr(dw, dws[i]) <= 5e-2, ("dW", i, relerr(dw, dws[i]))
        assert np.abs(db - dbs[i]).max() <= 5e-2 * max(np.abs(dbs[i]).max(), np.abs(dws[i]).max()), ("db", i)
    # SGD keeps fp32 master weights: one step matches the closed form on the library's own gradients
    before = [net.get_weights(i) for i in range(net.num_convs())]
    grads = [net.get_grad(i) for i in range(net.num_convs())]
    net.sgd_step(0.01)
    for i in range(net.num_convs()):
        w1, b1 = net.get_weights(i)
        assert np.abs(w1 - (before[i][0] - np.float32(0.01) * grads[i][0])).max() <= 1e-7
        assert np.abs(b1 - (before[i][1] - np.float32(0.01) * grads[i][1])).max() <= 1e-7
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("c_in,spec,h,w", [
    (5, [(12, 3, 3), (10, 2, 1), (3, 1, 1)], 40, 75),        # odd kernel strides, ragged map counts (2-byte fragment reads)
    (9, [(24, 4, 6), (2, 1, 1)], 50, 90),                    # d = 6: 4-byte reads
    (3, [(16, 3, 12), (20, 2, 4), (2, 1, 1)], 60, 100),      # d = 12 and 4: 8-byte reads
    (4, [(8, 4, 1), (72, 4, 8), (2, 1, 1)], 45, 140),        # d = 8: 16-byte reads; 72 maps = several map tiles
    # 4x4 layers of at most 48 maps take the row-streaming kernel: strips of 64 columns (65 = one full, one of width 1),
    # input-map tiles of 16 (20 maps = one and a quarter), the widest kernel stride it stages (3d = 63), two chained layers
    (20, [(48, 4, 3), (2, 1, 1)], 70, 65),
    (48, [(5, 4, 21), (2, 1, 1)], 90, 63),
    (1, [(16, 4, 1), (40, 4, 2), (3, 1, 1)], 33, 129),
    # 16 input maps or more, kernels of two rows or more: the strip-walking kernel (input rows kept in an LDS ring).
    # Fewer output rows than the kernel stride (7 < 12: every strip is one step; a wide image, so that single ReLU flips average out), ragged last segments, 2x2 and 3x3, an odd number of input octets
    (16, [(32, 2, 12), (2, 1, 1)], 7, 700),
    (24, [(16, 3, 1), (72, 2, 3), (16, 3, 2), (3, 1, 1)], 37, 150),
])
def test_weight_gradient_kernel_strides_half(dtype, c_in, spec, h, w):
    """The 16-bit weight gradient reads its input fragments at the alignment the kernel stride allows:
    every alignment class, two images, map counts off the octet and off the 16-map tile."""
    layers = [S.conv(f, k, d, relu=(i + 1 < len(spec))) for i, (f, k, d) in enumerate(spec)]
    ws, bs = S.he_normal_weights(layers, c_in, 77, bias_scale=0.05)
    img = np.ascontiguousarray(S.em_like_batch(2, h, w, 40).repeat(c_in, 1) * np.linspace(0.5, 1.5, c_in, dtype=np.float32)[None, :, None, None])
    classes = spec[-1][0]
    labels = (np.random.default_rng(41).integers(0, classes, (2, h, w))).astype(np.int32)
    net = make_net(layers, c_in, ws, bs, dtype)
    net.plan(2, h, w, pad=True, training=True)
    net.forward(torch.from_numpy(img).cuda())
    loss = net.backward(torch.from_numpy(labels).cuda())
    ow = [x.astype(np.float64) for x in ws]
    ob = [x.astype(np.float64) for x in bs]
    _, acts, ams = ON.sknet_forward(img, layers, ow, ob, keep=True)
    ref_loss, dws, dbs, _ = ON.sknet_backward(layers, ow, acts, ams, labels)
    assert abs(loss.item() - ref_loss) <= HALF_TOL * abs(ref_loss)
    # gradients pass through up to three layers of 16-bit storage: 8 mantissa bits (bf16) leave a few
    # per cent on the largest entry, 11 bits (fp16) well under one per cent -- the fp16 bound is the
    # one that would catch a misread fragment
    tol = 8e-2 if dtype == "bf16" else 1e-2
    grads = [net.get_grad(i) for i in range(net.num_convs())]
    net.close()
    for i, (dw, db) in enumerate(grads):
        print(dtype, "conv", i, "dW rel err %.3e" % relerr(dw, dws[i]), "db abs err %.3e of %.3e" % (np.abs(db - dbs[i]).max(), np.abs(dbs[i]).max()), flush=True)
    for i, (dw, db) in enumerate(grads):
        assert relerr(dw, dws[i]) <= tol, ("dW", i, relerr(dw, dws[i]))
        assert np.abs(db - dbs[i]).max() <= tol * max(np.abs(dbs[i]).max(), np.abs(dws[i]).max()), ("db", i)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_paper_sknet_configuration_forward_half(dtype):
    # the network of Section 3.3.2's SK table (k = 7, 5 d2, 3 d4 and the k = 10, d = 8 inner product 192 -> 1024,
    # context 101) in 16-bit storage: every layer and the fp32 logits against the oracle
    layers = S.paper_sknet_layers()
    ws, bs = S.he_normal_weights(layers, 3, 1003, bias_scale=0.05)
    img = S.uniform_image(1, 3, 60, 68, 11)
    net = make_net(layers, 3, ws, bs, dtype)
    net.plan(1, 60, 68, pad=True, keep=True)
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    ref_prob, acts, _ = ON.sknet_forward(img, layers, ws, bs, keep=True)
    for li in range(len(layers)):
        e = relerr(net.get_activation(li), acts[li + 1])
        print(dtype, "paper SK-Net layer", li, layers[li]["type"], "rel err %.3e" % e, flush=True)
        assert e <= HALF_TOL, (li, layers[li], e)
    assert np.abs(prob - ref_prob).max() <= HALF_TOL
    net.plan(1, 60, 68, pad=True)
    assert np.abs(net.forward(torch.from_numpy(img).cuda()).cpu().numpy() - ref_prob).max() <= HALF_TOL
    net.close()


def test_unsupported_kernel_size_is_reported():
    from paper_1509_03371_amd import binding as B
    with pytest.raises(B.SknetError) as e:
        B.SKNet([S.conv(72, 3, 8, relu=True), S.conv(2, 1, 1, relu=False)], 1, 2, dtype="bf16")    # 3x3 at d = 8 to 72 maps: tile beyond the LDS
    assert e.value.status_name == "SK_EUNSUPPORTED"
    B.SKNet([S.conv(32, 3, 8, relu=True), S.conv(2, 1, 1, relu=False)], 1, 2, dtype="bf16").close()  # two map tiles fit
    with pytest.raises(B.SknetError) as e:
        B.SKNet([S.conv(2, 9, 2, relu=False)], 1, 2, dtype="bf16")                                 # no 9x9 instantiation
    assert e.value.status_name == "SK_EUNSUPPORTED"
    with pytest.raises(B.SknetError) as e:
        B.SKNet([S.conv(2, 10, 12, relu=False)], 1, 2, dtype="bf16")                               # 128 + 11*12 columns: beyond the staged tile
    assert e.value.status_name == "SK_EUNSUPPORTED"
    net = B.SKNet([S.conv(8, 6, 1, relu=True), S.conv(2, 1, 1, relu=False)], 1, 2, dtype="bf16")
    with pytest.raises(B.SknetError) as e:
        net.plan(1, 40, 40, pad=True, training=True)                                               # large kernels: forward only
    assert e.value.status_name == "SK_EUNSUPPORTED"
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("pad_mode", [0, 1])
@pytest.mark.parametrize("pad", [True, False])
def test_first_layer_reads_the_image_itself(dtype, pad_mode, pad):
    """Inference plans of a one-map net hand the caller's fp32 image to the first layer's kernel, which mirror-pads and
    rounds it while it stages its tile; a plan that keeps every layer converts the padded image first and runs the same
    kernel on that copy.  The two must agree bit for bit (both padding modes, two images, sizes off every tile), and
    with the oracle."""
    from paper_1509_03371_amd import binding as B
    layers = [S.conv(40, 4, 1), S.pool(2, 1), S.conv(24, 4, 2), S.pool(2, 2), S.conv(3, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights(layers, 1, 910, bias_scale=0.1)
    h, w = (75, 139) if pad else (83, 147)
    img = S.em_like_batch(2, h, w, 911)
    nets = []
    for keep in (False, True):
        net = B.SKNet(layers, 1, 3, dtype=dtype, pad_mode=pad_mode)
        for i, (wt, b) in enumerate(zip(ws, bs)):
            net.set_weights(i, wt, b)
        net.plan(2, h, w, pad=pad, keep=keep)
        nets.append(net)
    dev = torch.from_numpy(img).cuda()
    direct, kept = nets[0].forward(dev).cpu().numpy(), nets[1].forward(dev).cpu().numpy()
    assert np.array_equal(direct, kept)
    ow = [x.astype(np.float64) for x in ws]
    ob = [x.astype(np.float64) for x in bs]
    ref = ON.sknet_forward(img, layers, ow, ob, pad=pad, pad_mode=pad_mode) if pad else ON.sknet_forward(img, layers, ow, ob, pad=False)
    assert np.abs(direct - ref).max() <= HALF_TOL
    for net in nets:
        net.close()
