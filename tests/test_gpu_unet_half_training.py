"""GPU parity: training pass of the U-Net and the USK-Net in 16-bit storage (bf16 / fp16 activations and error maps,
fp32 sums, fp32 weight gradients and master weights) through the C ABI against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import nets as ON

pytestmark = pytest.mark.gpu

# Every activation and every error map is rounded once to the storage type (8 mantissa bits in bf16, 11 in fp16) and a
# gradient passes through up to a dozen such tensors; the oracle computes in fp64 from the unrounded weights.  Two more
# effects sit inside these bounds.  (1) A rounded activation close to zero, or two pool candidates closer than a rounding
# step, decide a ReLU or a pool differently from fp64, which moves one pixel's whole contribution: the sums need a
# thousand labelled pixels or more to average that out (on a 12x20 output the first layer is off by 2e-1 in bf16).
# (2) The loss is a mean over the P labelled pixels, so every error map carries a factor 1/P: fp16 error maps sit in
# its subnormal range (below 6e-5, spacing 6e-8) from about a thousand pixels on and lose bits to underflow, which
# bf16 with fp32's exponent range does not; hence fp16 is not 8x tighter than bf16 here.  A wrong index, a missing
# mask or the other MergeCrop rule moves a tensor by tens of per cent (checked below for the rule).
TOL = {"bf16": 8e-2, "f16": 3e-2}
LOSS_TOL = 2e-2
MASKED = {"bf16": 0.25, "f16": 0.25}


def relerr(got, ref):
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def image(n, c_in, h, w, seed):
    img = np.stack([np.stack([S.em_like_image(h, w, seed + 7 * i + c) for c in range(c_in)]) for i in range(n)])
    return np.ascontiguousarray(img, dtype=np.float32)


def masked_labels(n, h, w, classes, seed, masked=0.25):
    rng = np.random.default_rng(seed)
    lab = rng.integers(0, classes, (n, h, w)).astype(np.int32)
    lab[rng.random((n, h, w)) < masked] = -1
    return lab


def check_grads(net, names, loss, ref_loss, ref_grads, tag, tol):
    assert abs(float(loss.item()) - ref_loss) <= LOSS_TOL * abs(ref_loss)
    errs = []
    for i, name in enumerate(names):
        dw, db = net.get_grad(i)
        assert dw.shape == ref_grads[name][0].shape and db.shape == ref_grads[name][1].shape, name
        assert np.abs(ref_grads[name][0]).max() > 1e-6, name            # a dead net would pass anything
        e_w = relerr(dw, ref_grads[name][0])
        e_b = float(np.abs(db - ref_grads[name][1]).max() / max(np.abs(ref_grads[name][1]).max(), np.abs(ref_grads[name][0]).max()))
        errs.append((name, e_w, e_b))
        print("%s %-8s dW %.2e db %.2e" % (tag, name, e_w, e_b), flush=True)
    for name, e_w, e_b in errs:
        assert e_w <= tol and e_b <= tol, (name, e_w, e_b)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("merge_into_b", [0, 1])
@pytest.mark.parametrize("depth,base,h,w,n,seed", [(2, 8, 60, 76, 2, 502), (1, 16, 60, 68, 2, 601), (3, 8, 140, 124, 2, 503)])
def test_unet_backward_half(depth, base, h, w, n, seed, merge_into_b, dtype):
    from paper_1509_03371_amd import binding as B
    params = S.unet_params(2, 3, seed, depth=depth, base=base, bias_scale=0.1)
    names = S.unet_param_names(depth)
    net = B.UNet(2, 3, depth=depth, base_ch=base, dtype=dtype)
    for i, name in enumerate(names):
        net.set_weights(i, *params[name])
    img = image(n, 2, h, w, 510)
    net.plan(n, h, w, training=True)
    if merge_into_b:
        net.set_merge_backward(1)
    ho, wo = net.output_size(h, w)
    lab = masked_labels(n, ho, wo, 3, 511, MASKED[dtype])
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    loss = net.backward(torch.from_numpy(lab).cuda())
    p64 = {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in params.items()}
    assert np.abs(prob - ON.unet_forward(img, p64, depth=depth)).max() <= 2e-2
    ref_loss, ref_grads = ON.unet_backward(img, p64, lab, depth=depth, merge_into_b=bool(merge_into_b))
    if depth == 2 and dtype == "f16":      # the two MergeCrop rules differ by more than the tolerance
        _, other = ON.unet_backward(img, p64, lab, depth=depth, merge_into_b=not merge_into_b)
        assert relerr(other["down0a"][0], ref_grads["down0a"][0]) > 3 * TOL[dtype]
    check_grads(net, names, loss, ref_loss, ref_grads, "unet %s d%d m%d" % (dtype, depth, merge_into_b), TOL[dtype])
    # a second pass on the same plan (gradient buffers are reused) gives the same gradients
    first = net.get_grad(0)[0]
    net.forward(torch.from_numpy(img).cuda())
    net.backward(torch.from_numpy(lab).cuda())
    assert np.array_equal(first, net.get_grad(0)[0])
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_unet_backward_half_wide_maps(dtype):
    # 128 and 256 maps on a small image: the 16-bit weight gradient splits over map-tile and column-tile groups, each
    # staging the dY rows of its maps and only the input octets its columns touch
    from paper_1509_03371_amd import binding as B
    depth, base, h, w, n = 1, 128, 44, 52, 2
    params = S.unet_params(1, 2, 530, depth=depth, base=base, bias_scale=0.05)
    names = S.unet_param_names(depth)
    net = B.UNet(1, 2, depth=depth, base_ch=base, dtype=dtype)
    for i, name in enumerate(names):
        net.set_weights(i, *params[name])
    img = image(n, 1, h, w, 531)
    net.plan(n, h, w, training=True)
    ho, wo = net.output_size(h, w)
    lab = masked_labels(n, ho, wo, 2, 532, MASKED[dtype])
    net.forward(torch.from_numpy(img).cuda())
    loss = net.backward(torch.from_numpy(lab).cuda())
    p64 = {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in params.items()}
    ref_loss, ref_grads = ON.unet_backward(img, p64, lab, depth=depth)
    check_grads(net, names, loss, ref_loss, ref_grads, "unet wide " + dtype, TOL[dtype])
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_unet_sgd_step_half(dtype):
    # fp32 master weights take the closed-form step on the library's own gradients; the next forward pass runs on
    # the re-packed 16-bit weights (same probabilities as a fresh net given the updated weights)
    from paper_1509_03371_amd import binding as B
    depth, base, h, w, n = 1, 16, 44, 52, 1
    params = S.unet_params(1, 2, 540, depth=depth, base=base, bias_scale=0.1)
    names = S.unet_param_names(depth)
    net = B.UNet(1, 2, depth=depth, base_ch=base, dtype=dtype)
    for i, name in enumerate(names):
        net.set_weights(i, *params[name])
    img = torch.from_numpy(image(n, 1, h, w, 541)).cuda()
    net.plan(n, h, w, training=True)
    ho, wo = net.output_size(h, w)
    lab = torch.from_numpy(masked_labels(n, ho, wo, 2, 542)).cuda()
    net.forward(img)
    loss0 = float(net.backward(lab).item())
    before = [net.get_weights(i) for i in range(len(names))]
    grads = [net.get_grad(i) for i in range(len(names))]
    lr = np.float32(0.01)
    net.sgd_step(float(lr))
    after = [net.get_weights(i) for i in range(len(names))]
    for i in range(len(names)):
        assert np.abs(after[i][0] - (before[i][0] - lr * grads[i][0])).max() <= 1e-6, names[i]
        assert np.abs(after[i][1] - (before[i][1] - lr * grads[i][1])).max() <= 1e-6, names[i]
    prob1 = net.forward(img).cpu().numpy()
    loss1 = float(net.backward(lab).item())
    fresh = B.UNet(1, 2, depth=depth, base_ch=base, dtype=dtype)
    for i in range(len(names)):
        fresh.set_weights(i, *after[i])
    fresh.plan(n, h, w)
    assert np.array_equal(prob1, fresh.forward(img).cpu().numpy())
    fresh.close()
    assert loss1 < loss0, (loss0, loss1)
    net.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("merge_into_b", [0, 1])
def test_usknet_backward_half(merge_into_b, dtype):
    from paper_1509_03371_amd import binding as B
    base, h, w, n = 8, 212, 228, 2
    params = S.usknet_params(2, 3, 520, base=base, bias_scale=0.1)
    net = B.USKNet(2, 3, base_ch=base, dtype=dtype)
    for i, name in enumerate(S.USKNET_PARAM_NAMES):
        net.set_weights(i, *params[name])
    img = image(n, 2, h, w, 521)
    net.plan(n, h, w, training=True)
    net.set_merge_backward(merge_into_b)
    ho, wo = net.output_size(h, w)
    lab = masked_labels(n, ho, wo, 3, 522, MASKED[dtype])
    net.forward(torch.from_numpy(img).cuda())
    loss = net.backward(torch.from_numpy(lab).cuda())
    p64 = {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in params.items()}
    ref_loss, ref_grads = ON.usknet_backward(img, p64, lab, base=base, merge_into_b=bool(merge_into_b))
    check_grads(net, S.USKNET_PARAM_NAMES, loss, ref_loss, ref_grads, "usk %s m%d" % (dtype, merge_into_b), TOL[dtype])
    net.close()


def test_c5_unet_training_pass_572_bf16():
    # the configuration table's own sizes (1 x 572^2 -> 388^2, 64..1024 maps) in bf16 storage: the launch configuration
    # bench.py times; every parameter gradient against the oracle
    from paper_1509_03371_amd import binding as B
    params = S.unet_params(1, 2, 1005, depth=4, base=64)
    names = S.unet_param_names(4)
    net = B.UNet(1, 2, depth=4, base_ch=64, dtype="bf16")
    for i, name in enumerate(names):
        net.set_weights(i, *params[name])
    img = image(1, 1, 572, 572, 1010)
    net.plan(1, 572, 572, training=True)
    lab = S.mask_labels_by_frequency(S.binary_labels(1, 388, 388, 1011), 2, 1012)
    net.forward(torch.from_numpy(img).cuda())
    loss = net.backward(torch.from_numpy(lab).cuda())
    p64 = {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in params.items()}
    ref_loss, ref_grads = ON.unet_backward(img, p64, lab, depth=4)
    check_grads(net, names, loss, ref_loss, ref_grads, "unet 572 bf16", TOL["bf16"])
    net.close()
