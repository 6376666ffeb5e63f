"""GPU parity: training pass of the U-Net and the USK-Net (fp32) through the C ABI against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import nets as ON

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4     # relative to the largest entry of each gradient tensor (fp32 MFMA accumulation against fp64)


def relerr(got, ref):
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def check_grads(net, names, params, loss, ref_loss, ref_grads, tag):
    assert abs(float(loss.item()) - ref_loss) <= FP32_TOL * abs(ref_loss)
    errs = []
    for i, name in enumerate(names):
        dw, db = net.get_grad(i)
        assert dw.shape == ref_grads[name][0].shape and db.shape == ref_grads[name][1].shape, name
        e_w = relerr(dw, ref_grads[name][0])
        assert np.abs(ref_grads[name][0]).max() > 1e-6, name            # a dead net would pass anything
        e_b = float(np.abs(db - ref_grads[name][1]).max() / max(np.abs(ref_grads[name][1]).max(), np.abs(ref_grads[name][0]).max()))
        errs.append((name, e_w, e_b))
        print("%s %-8s dW %.2e db %.2e" % (tag, name, e_w, e_b), flush=True)
    for name, e_w, e_b in errs:
        assert e_w <= FP32_TOL and e_b <= FP32_TOL, (name, e_w, e_b)


def image(n, c_in, h, w, seed):
    img = np.stack([np.stack([S.em_like_image(h, w, seed + 7 * i + c) for c in range(c_in)]) for i in range(n)])
    return np.ascontiguousarray(img, dtype=np.float32)


def masked_labels(n, h, w, classes, seed, masked=0.25):
    rng = np.random.default_rng(seed)
    lab = rng.integers(0, classes, (n, h, w)).astype(np.int32)
    lab[rng.random((n, h, w)) < masked] = -1
    return lab


@pytest.mark.parametrize("depth,base,h,w,n,seed", [(2, 8, 60, 76, 2, 502), (1, 8, 28, 36, 1, 601), (3, 4, 108, 92, 1, 503)])
def test_unet_backward(depth, base, h, w, n, seed):
    from paper_1509_03371_amd import binding as B
    params = S.unet_params(2, 3, seed, depth=depth, base=base, bias_scale=0.1)
    names = S.unet_param_names(depth)
    net = B.UNet(2, 3, depth=depth, base_ch=base)
    for i, name in enumerate(names):
        net.set_weights(i, *params[name])
    img = image(n, 2, h, w, 510)
    net.plan(n, h, w, training=True)
    ho, wo = net.output_size(h, w)
    lab = masked_labels(n, ho, wo, 3, 511)
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    loss = net.backward(torch.from_numpy(lab).cuda())
    p64 = {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in params.items()}
    assert np.abs(prob - ON.unet_forward(img, p64, depth=depth)).max() <= FP32_TOL
    ref_loss, ref_grads = ON.unet_backward(img, p64, lab, depth=depth)
    check_grads(net, names, params, loss, ref_loss, ref_grads, "unet d%d" % depth)
    # a second pass on the same plan (gradient buffers are reused) gives the same gradients
    net.forward(torch.from_numpy(img).cuda())
    net.backward(torch.from_numpy(lab).cuda())
    again = net.get_grad(0)[0]
    net.forward(torch.from_numpy(img).cuda())
    net.backward(torch.from_numpy(lab).cuda())
    assert np.array_equal(again, net.get_grad(0)[0])
    net.close()


def test_usknet_backward():
    from paper_1509_03371_amd import binding as B
    base, h, w, n = 8, 212, 228, 2
    params = S.usknet_params(2, 3, 520, base=base, bias_scale=0.1)
    net = B.USKNet(2, 3, base_ch=base)
    for i, name in enumerate(S.USKNET_PARAM_NAMES):
        net.set_weights(i, *params[name])
    img = image(n, 2, h, w, 521)
    net.plan(n, h, w, training=True)
    ho, wo = net.output_size(h, w)
    lab = masked_labels(n, ho, wo, 3, 522)
    net.forward(torch.from_numpy(img).cuda())
    loss = net.backward(torch.from_numpy(lab).cuda())
    p64 = {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in params.items()}
    ref_loss, ref_grads = ON.usknet_backward(img, p64, lab, base=base)
    check_grads(net, S.USKNET_PARAM_NAMES, params, loss, ref_loss, ref_grads, "usk")
    net.close()


def test_unet_backward_state_and_type_errors():
    from paper_1509_03371_amd import binding as B
    net = B.UNet(1, 2, depth=1, base_ch=8)
    net.plan(1, 28, 28)
    net.forward(torch.zeros(1, 1, 28, 28, device="cuda"))
    with pytest.raises(B.SknetError):
        net.backward(torch.zeros(1, 12, 12, dtype=torch.int32, device="cuda"))     # inference plan
    net.plan(1, 28, 28, training=True)
    with pytest.raises(B.SknetError):
        net.backward(torch.zeros(1, 12, 12, dtype=torch.int32, device="cuda"))     # no forward on this plan yet
    with pytest.raises(B.SknetError):
        net.get_grad(0)
    net.close()
    half = B.UNet(1, 2, depth=1, base_ch=8, dtype="bf16")
    with pytest.raises(B.SknetError):
        half.plan(1, 28, 28, training=True)                                         # fp32 only
    half.close()
