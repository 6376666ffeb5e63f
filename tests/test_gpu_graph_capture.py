"""GPU: the forward pass can be recorded into a HIP graph (it allocates nothing, clears nothing with
memset nodes and never synchronises) and every replay equals the eager result on new input.  The
recorded call is the first forward after the plan: all one-time set-up belongs to the plan call."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import nets as ON

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_replays_from_a_hip_graph(dtype):
    from paper_1509_03371_amd import binding as B
    layers = S.sknet_layers(width=16, hidden=40)
    ws, bs = S.he_normal_weights(layers, 1, 77, bias_scale=0.1)
    net = B.SKNet(layers, 1, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    n, h, w = 2, 70, 90
    net.plan(n, h, w, pad=True)
    img = torch.zeros((n, 1, h, w), dtype=torch.float32, device="cuda")
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        g = torch.cuda.CUDAGraph()                     # the very first forward of this plan is the recorded one
        with torch.cuda.graph(g, stream=s):
            net.forward(img, prob, torch.cuda.current_stream())
        for rep in range(3):
            host = S.uniform_image(n, 1, h, w, 300 + rep)
            img.copy_(torch.from_numpy(host))
            net.forward(img, prob, torch.cuda.current_stream())     # the program's own eager work between replays
            torch.cuda.current_stream().synchronize()
            eager = prob.clone()
            prob.zero_()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(prob, eager), rep
            if rep == 0:
                ref = ON.sknet_forward(host, layers, ws, bs)
                assert np.abs(prob.cpu().numpy() - ref).max() <= (1e-4 if dtype == "f32" else 2e-2)
    net.close()


def test_3d_forward_replays_from_a_hip_graph():
    # the 3-D forward pass (one launch per convolution or an accumulating launch per depth tap, 3-D pools, fused
    # head) records nothing but kernels either
    from oracle import nd as OND
    from paper_1509_03371_amd import binding as B
    layers = [S.conv(16, 3, 1), S.pool(2, 1), S.conv(12, 3, 2), S.pool(2, 2), S.conv(20, 2, 4), S.conv(8, 1, 1), S.conv(2, 1, 1, relu=False)]
    ws, bs = S.he_normal_weights3d(layers, 1, 78, bias_scale=0.1)
    net = B.SKNet3D(layers, 1, 2)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    dz, h, w = 22, 30, 75
    net.plan(dz, h, w)
    vol = torch.zeros((dz, 1, h, w), dtype=torch.float32, device="cuda")
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            net.forward(vol, prob, torch.cuda.current_stream())
        for rep in range(3):
            host = S.uniform_volume(1, dz, h, w, 310 + rep)
            vol.copy_(torch.from_numpy(np.ascontiguousarray(host.transpose(1, 0, 2, 3))))
            net.forward(vol, prob, torch.cuda.current_stream())
            torch.cuda.current_stream().synchronize()
            eager = prob.clone()
            prob.zero_()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(prob, eager), rep
            if rep == 0:
                ref = OND.sknet3d_forward(host, layers, ws, bs)
                assert np.abs(prob.cpu().numpy().transpose(1, 0, 2, 3) - ref).max() <= 1e-4
    net.close()
