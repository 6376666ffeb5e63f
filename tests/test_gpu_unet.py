"""GPU parity: U-Net forward through the C ABI against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import nets as ON

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4


def relerr(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def run_unet(c_in, classes, depth, base, h, w, seed, n=1, bias_scale=0.1):
    from paper_1509_03371_amd import binding as B
    params = S.unet_params(c_in, classes, seed, depth=depth, base=base, bias_scale=bias_scale)
    net = B.UNet(c_in, classes, depth=depth, base_ch=base)
    for i, name in enumerate(S.unet_param_names(depth)):
        net.set_weights(i, *params[name])
    img = np.stack([S.em_like_image(h, w, seed + 1 + i) for i in range(n)])[:, None].repeat(c_in, 1)
    img = np.ascontiguousarray(img)
    net.plan(n, h, w)
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    ref, trace = ON.unet_forward(img, {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in params.items()},
                                 depth=depth, keep=True)
    for stage, r in trace.items():
        got = net.get_activation(stage)
        assert got.shape == r.shape, stage
        assert relerr(got, r) <= FP32_TOL, stage
    assert prob.shape == ref.shape
    assert np.abs(prob - ref).max() <= FP32_TOL
    net.close()
    return prob


def test_unet_depth2_small():
    prob = run_unet(2, 3, 2, 8, 60, 76, 100, n=2)
    assert prob.shape == (2, 3, 20, 36)


def test_unet_depth4_small_maps():
    # 188 -> 4: the smallest input the depth-4 net accepts
    prob = run_unet(1, 2, 4, 8, 188, 204, 101)
    assert prob.shape == (1, 2, 4, 20)


def test_c5_unet_572():
    prob = run_unet(1, 2, 4, 64, 572, 572, 1005, bias_scale=0.0)
    assert prob.shape == (1, 2, 388, 388)
