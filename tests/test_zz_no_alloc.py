"""GPU: sknet_backward_noalloc -- the backward pass whose partial results live in the library's static device
buffer -- against sknet_backward on the same plan and inputs: loss and every gradient, two calls in a row, the
second on a smaller input; and its size limit."""
import numpy as np
import pytest
import torch

import sk_synth as S

pytestmark = pytest.mark.gpu


def relerr(got, ref):
    return float(np.abs(got.astype(np.float64) - ref.astype(np.float64)).max() / max(np.abs(ref).max(), 1e-30))


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-4), ("bf16", 1e-4)])
def test_noalloc_backward_matches_backward_twice_second_smaller(dtype, tol):
    # both entry points read the same stored activations, so even the 16-bit net's gradients agree to the
    # rounding of the fp32 sums (the number of private copies, hence the summation order, may differ)
    from paper_1509_03371_amd import binding as B
    layers = S.sknet_layers(width=48, hidden=40)
    ws, bs = S.he_normal_weights(layers, 1, 91, bias_scale=0.1)
    net = B.SKNet(layers, 1, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    for call, (n, h, w) in enumerate([(2, 150, 200), (1, 70, 90)]):
        net.plan(n, h, w, pad=True, training=True)
        img = torch.from_numpy(S.em_like_batch(n, h, w, 92 + call)).cuda()
        lab = S.binary_labels(n, h, w, 94 + call)
        lab[:, :3] = -1
        lab = torch.from_numpy(lab).cuda()
        net.forward(img)
        ref_loss = float(net.backward(lab).item())
        ref = [net.get_grad(i) for i in range(net.num_convs())]
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        net.forward(img)
        net.backward(lab, loss=loss, noalloc=True)
        got = [net.get_grad(i) for i in range(net.num_convs())]
        assert abs(float(loss.item()) - ref_loss) <= tol * abs(ref_loss), call
        for i, ((dw, db), (rw, rb)) in enumerate(zip(got, ref)):
            assert np.abs(rw).max() > 0
            print(dtype, "call", call, "conv", i, "dW %.2e db %.2e" % (relerr(dw, rw), relerr(db, rb)), flush=True)
            assert relerr(dw, rw) <= tol and np.abs(db - rb).max() <= tol * max(np.abs(rb).max(), np.abs(rw).max()), (call, i)
        # SGD accepts the gradients of either call
        net.sgd_step(0.01)
    net.close()


def test_noalloc_backward_rejects_a_gradient_beyond_the_static_buffer():
    from paper_1509_03371_amd import binding as B
    # 3000 x 3000 1x1 weights: one padded copy is 3008 * 3008 floats, more than the buffer's 8 Mi - 4096
    layers = [S.conv(3000, 1, 1, relu=True), S.conv(3000, 1, 1, relu=True), S.conv(2, 1, 1, relu=False)]
    net = B.SKNet(layers, 4, 2)
    net.plan(1, 8, 8, pad=True, training=True)
    img = torch.zeros(1, 4, 8, 8, device="cuda")
    lab = torch.zeros(1, 8, 8, dtype=torch.int32, device="cuda")
    loss = torch.zeros(1, device="cuda")
    net.forward(img)
    with pytest.raises(B.SknetError) as e:
        net.backward(lab, loss=loss, noalloc=True)
    assert e.value.status_name == "SK_EUNSUPPORTED" and "static buffer" in str(e.value)
    net.backward(lab, loss=loss)            # the plan's own scratch takes it
    net.close()
