"""GPU parity: USK-Net forward (the USK network configuration table) through the C ABI against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import sk_synth as S
from oracle import nets as ON

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4     # fp32 storage and fp32 MFMA accumulation against fp64, relative to the stage's largest value


def relerr(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def run_usknet(c_in, classes, base, h, w, seed, n=1, bias_scale=0.1, dtype="f32"):
    from paper_1509_03371_amd import binding as B
    params = S.usknet_params(c_in, classes, seed, base=base, bias_scale=bias_scale)
    net = B.USKNet(c_in, classes, base_ch=base, dtype=dtype)
    # 16-bit storage: 2e-2 on logits and probabilities (the oracle sees the unrounded weights and image), twice that
    # on intermediate stages, as for the U-Net
    tol, stage_tol = (FP32_TOL, FP32_TOL) if dtype == "f32" else (2e-2, 4e-2)
    assert net.num_params() == len(S.USKNET_PARAM_NAMES)
    for i, name in enumerate(S.USKNET_PARAM_NAMES):
        assert net.param_shape(i) == params[name][0].shape, name
        net.set_weights(i, *params[name])
    img = np.stack([np.stack([S.em_like_image(h, w, seed + 1 + 7 * i + c) for c in range(c_in)]) for i in range(n)])
    img = np.ascontiguousarray(img, dtype=np.float32)
    net.plan(n, h, w)
    prob = net.forward(torch.from_numpy(img).cuda()).cpu().numpy()
    ref, trace = ON.usknet_forward(img, {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in params.items()},
                                   base=base, keep=True)
    for stage, r in trace.items():
        got = net.get_activation(stage)
        assert got.shape == r.shape, stage
        e = relerr(got, r)
        print("usk %s %s %s rel err %.3e" % (dtype, stage, r.shape, e), flush=True)
        assert e <= (tol if stage == "logits" else stage_tol), (stage, e)
    assert prob.shape == ref.shape
    assert np.abs(prob - ref).max() <= tol
    net.close()
    return prob


def test_usknet_small_two_images():
    # 212 x 228: 208x224 -> pool 104x112 -> SK core (context 86) 18x26 -> up 36x52 -> 32x48; crop offsets 86
    prob = run_usknet(2, 3, 8, 212, 228, 300, n=2)
    assert prob.shape == (2, 3, 32, 48)


def test_usknet_smallest_input():
    prob = run_usknet(1, 2, 8, 182, 182, 301)
    assert prob.shape == (1, 2, 2, 2)


def test_usknet_table_configuration_692():
    # the table's own sizes and map counts: 3 x 692^2 -> 2 x 512^2, every listed stage against the oracle
    prob = run_usknet(3, 2, 64, 692, 692, 1006, bias_scale=0.0)
    assert prob.shape == (1, 2, 512, 512)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_usknet_small_two_images_half(dtype):
    prob = run_usknet(2, 3, 8, 212, 228, 300, n=2, dtype=dtype)
    assert prob.shape == (2, 3, 32, 48)


def test_usknet_table_configuration_692_bf16():
    prob = run_usknet(3, 2, 64, 692, 692, 1006, bias_scale=0.0, dtype="bf16")
    assert prob.shape == (1, 2, 512, 512)


def test_usknet_rejections():
    from paper_1509_03371_amd import binding as B
    net = B.USKNet(1, 2, base_ch=8)
    with pytest.raises(B.SknetError):
        net.output_size(183, 182)          # 179 is odd: the 2x2 stride-2 pool does not divide it
    with pytest.raises(B.SknetError):
        net.output_size(180, 180)          # the SK part's context of 86 leaves nothing
    net.close()
    with pytest.raises(B.SknetError):
        B.USKNet(1, 2, base_ch=12, dtype="bf16")    # 16-bit storage keeps maps in groups of 8
    half = B.USKNet(1, 2, base_ch=8, dtype="bf16")
    with pytest.raises(B.SknetError) as e:
        half.plan(1, 183, 182, training=True)       # 16-bit training plans check the shape like every other plan
    assert e.value.status_name == "SK_ESHAPE"
    half.close()
