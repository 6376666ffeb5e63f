"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host
logic (Algorithm 1, shape inference, argument checks) works without a GPU."""
import os
import re

import numpy as np
import pytest

import sk_synth as S
from paper_1509_03371_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sknet.h")).read()
    declared = set(re.findall(r"\b((?:sknet3d|sknet|unet|usknet|sk_probe)_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(B.lib, name), name
    assert declared == set(B.EXPORTED)


def test_convert_sw_matches_paper_table(golden_rows):
    rows = golden_rows("sknet_table.txt")
    sw = []
    for name, typ, *_rest in rows[1:]:
        f_out, k = int(_rest[2]), int(_rest[3])
        if typ == "conv":
            sw.append({"type": "conv", "f_out": f_out, "k": k, "relu": True})
        elif typ == "pool":
            sw.append({"type": "pool", "k": k, "s": k})
        else:
            sw.append({"type": "ip", "f_out": f_out, "relu": name != "ip3"})
    sk = B.sknet_convert_sw(sw, 102)
    assert [l["k"] for l in sk] == [int(r[5]) for r in rows[1:]]
    assert [l["d"] for l in sk] == [int(r[6]) for r in rows[1:]]
    net = B.SKNet(sk, 3, 2)
    assert net.context() == 101
    shapes = net.infer_shapes(229, 229, pad=False)
    assert [s[1] for s in shapes] == [int(r[2]) for r in rows]
    assert [s[0] for s in shapes] == [int(r[4]) for r in rows]
    assert net.infer_shapes(128, 128, pad=True)[-1] == (2, 128, 128)
    with pytest.raises(B.SknetError) as e:              # the uncorrected table: 43 mod 2 != 0
        B.sknet_convert_sw(sw, 100)
    assert e.value.status_name == "SK_ESHAPE"


def test_convert_sw_error_cases():
    conv = {"type": "conv", "f_out": 4, "k": 3, "relu": True}
    for bad in ([conv, {"type": "pool", "k": 2, "s": 1}], [conv, {"type": "pool", "k": 2, "s": 2}],
                [{"type": "other", "k": 3}]):
        with pytest.raises(B.SknetError) as e:
            B.sknet_convert_sw(bad, 10)
        assert e.value.status_name == "SK_ESHAPE"
    assert B.sknet_convert_sw(S.tiny_sw_layers(), 15)[2] == S.conv(16, 5, 2)


def test_flop_counter(golden_rows):
    assert abs(B.sknet_conv_flops(192, 1024, 10, 128) / 1e9 - 644.23) < 0.005      # ip1 of the SK table
    assert abs(B.sknet_conv_flops(64, 64, 3, 568) / 1e9 - 23.77) < 0.005           # conv2 of the U table


def test_create_and_shape_errors():
    with pytest.raises(B.SknetError) as e:
        B.SKNet([S.conv(4, 3, 1)], 1, 2)                     # n_classes mismatch
    assert e.value.status_name == "SK_ESHAPE"
    with pytest.raises(B.SknetError) as e:
        B.SKNet([S.conv(4, 0, 1)], 1, 4)
    assert e.value.status_name == "SK_ESHAPE"
    with pytest.raises(B.SknetError) as e:
        B.SKNet([S.pool(2, 2, 2), S.conv(2, 1, 1)], 1, 2)    # s = k needs d = 1
    assert e.value.status_name == "SK_ESHAPE"
    net = B.SKNet(S.tiny_sknet_layers(), 1, 2)
    assert net.context() == 14
    assert net.infer_shapes(96, 96)[0] == (1, 110, 110) and net.infer_shapes(96, 96)[-1] == (2, 96, 96)
    with pytest.raises(B.SknetError) as e:
        net.infer_shapes(5, 96)                              # mirror border 7 does not fit 5 rows
    assert e.value.status_name == "SK_ESHAPE"
    with pytest.raises(B.SknetError) as e:
        net.infer_shapes(10, 10, pad=False)                  # smaller than the context
    assert e.value.status_name == "SK_ESHAPE"
    down = B.SKNet([S.conv(4, 3, 1), S.pool(2, 1, 2), S.conv(2, 1, 1, relu=False)], 1, 2)
    assert down.infer_shapes(12, 12, pad=False)[-1] == (2, 5, 5)
    with pytest.raises(B.SknetError):
        down.infer_shapes(13, 13, pad=False)                 # odd map at the pool
    with pytest.raises(B.SknetError):
        down.context()
    with pytest.raises(B.SknetError) as e:
        net.get_grad(0)
    assert e.value.status_name == "SK_ESTATE"


def test_weights_round_trip_on_host():
    net = B.SKNet(S.tiny_sknet_layers(), 1, 2)
    ws, bs = S.he_normal_weights(S.tiny_sknet_layers(), 1, 5, bias_scale=1.0)
    for i in range(net.num_convs()):
        assert net.conv_shape(i) == ws[i].shape
        net.set_weights(i, ws[i], bs[i])
    for i in range(net.num_convs()):
        w, b = net.get_weights(i)
        assert np.array_equal(w, ws[i]) and np.array_equal(b, bs[i])
    with pytest.raises(ValueError):
        net.set_weights(0, ws[1])


def test_unet_host_logic(golden_rows):
    u = B.UNet(3, 2, depth=4, base_ch=64)
    assert u.output_size(572, 572) == (388, 388)             # the U network configuration table
    with pytest.raises(B.SknetError):
        u.output_size(570, 570)                              # odd map at a pool
    names = S.unet_param_names(4)
    assert u.num_params() == len(names)
    params = S.unet_params(3, 2, 1, depth=4, base=64)
    total = 0
    for i, name in enumerate(names):
        assert u.param_shape(i) == params[name][0].shape, name
        if not name.startswith("up"):
            total += params[name][0].size
    # free parameters of the table's convolutions: the up step's 1x1 conv f -> f/2 has f*f/2 weights
    total += sum(params[n][0].size // 4 for n in names if n.startswith("up"))
    assert round(total / 1e6) == 29


def test_usknet_handle_host_logic(golden_rows):
    # parameter shapes, the table's 692 -> 512, and the refusals; no GPU call is made
    net = B.USKNet(3, 2, base_ch=64)
    want = S.usknet_params(3, 2, 1, base=64)
    assert net.num_params() == len(S.USKNET_PARAM_NAMES)
    for i, name in enumerate(S.USKNET_PARAM_NAMES):
        assert net.param_shape(i) == want[name][0].shape, name
    rows = {r[0]: int(r[2]) for r in golden_rows("usknet_table.txt")}
    assert net.output_size(rows["data"], rows["data"]) == (rows["ip3"], rows["ip3"])
    assert net.output_size(182, 190) == (2, 10)
    for bad in ((181, 182), (180, 180), (3, 3)):
        with pytest.raises(B.SknetError) as e:
            net.output_size(*bad)
        assert e.value.status_name == "SK_ESHAPE"
    net.close()
    B.USKNet(3, 2, base_ch=64, dtype="f16").close()          # 16-bit storage: maps in groups of 8
    with pytest.raises(B.SknetError) as e:
        B.USKNet(3, 2, base_ch=12, dtype="f16")
    assert e.value.status_name == "SK_EUNSUPPORTED"


def test_unet_training_plan_checks_the_shape_before_anything_is_allocated():
    # 16-bit and fp32 training plans alike: an image whose maps cannot be pooled is refused on the host
    for dtype in ("bf16", "f32"):
        net = B.UNet(1, 2, depth=2, base_ch=8, dtype=dtype)
        with pytest.raises(B.SknetError) as e:
            net.plan(1, 62, 62, training=True)      # 62 - 4 = 58 -> 29 - 4 = 25: odd at the second pool
        assert e.value.status_name == "SK_ESHAPE"
        net.close()


def test_sknet3d_handle_host_logic():
    # shapes, context and refusals of the 3-D handle; no GPU call is made
    layers = S.sknet3d_layers(classes=2)
    net = B.SKNet3D(layers, 1, 2)
    assert net.context() == 17 and net.num_convs() == 5
    assert net.conv_shape(0) == (16, 1, 3, 3, 3) and net.conv_shape(2) == (128, 32, 3, 3, 3) and net.conv_shape(4) == (2, 64, 1, 1, 1)
    shapes = net.infer_shapes(81, 145, 100)
    assert shapes[0] == (1, 81, 145, 100) and shapes[1] == (16, 79, 143, 98) and shapes[2] == (16, 78, 142, 97)
    assert shapes[3] == (32, 74, 138, 93) and shapes[4] == (32, 72, 136, 91) and shapes[-1] == (2, 64, 128, 83)
    with pytest.raises(B.SknetError) as e:
        net.infer_shapes(81, 17, 145)
    assert e.value.status_name == "SK_ESHAPE"
    with pytest.raises(ValueError):
        net.set_weights(0, np.zeros((16, 1, 3, 3), np.float32))
    net.close()
    with pytest.raises(B.SknetError) as e:
        B.SKNet3D(layers, 1, 3)                  # the last layer has 2 maps
    assert e.value.status_name == "SK_ESHAPE"
    with pytest.raises(B.SknetError) as e:
        B.SKNet3D([S.pool(2, 2, 2), S.conv(2, 1, 1, relu=False)], 1, 2)   # a down-sampling pool with d != 1
    assert e.value.status_name == "SK_ESHAPE"
    down = B.SKNet3D([S.conv(4, 3, 1), S.pool(2, 1, 2), S.conv(2, 1, 1, relu=False)], 1, 2)
    assert down.infer_shapes(10, 12, 14)[-1] == (2, 4, 5, 6)
    with pytest.raises(B.SknetError) as e:
        down.infer_shapes(11, 12, 14)
    assert e.value.status_name == "SK_ESHAPE"
    with pytest.raises(B.SknetError) as e:
        down.context()
    assert e.value.status_name == "SK_ESHAPE"
    down.close()
