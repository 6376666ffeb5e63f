"""Pins of the CPU oracle to things other than itself: numbers printed in the paper, the
sliding-window definition evaluated by brute force, closed forms, library routines on special
cases, and finite differences.  CPU only."""
import numpy as np
import pytest
import scipy.ndimage
import scipy.signal
import torch
import torch.nn.functional as F

import sk_synth as S
from oracle import alg1, layers as L, nets, sw_net

rng = np.random.default_rng


def _hand(golden_rows, key):
    for row in golden_rows("hand_examples.txt"):
        if row[0] == key:
            return np.array([float(v) for v in row[1:]])
    raise KeyError(key)


# ------------------------------------------------------------------ hand-computed examples
def test_hand_conv_k2_d2(golden_rows):
    x = np.arange(25.0).reshape(1, 1, 5, 5)
    y = L.conv_sk(x, np.array([[[[1.0, 2.0], [3.0, 4.0]]]]), None, d=2)
    assert np.array_equal(y.ravel(), _hand(golden_rows, "conv_k2_d2"))


def test_hand_pool_k2_d2(golden_rows):
    x = np.arange(25.0).reshape(1, 1, 5, 5)
    y, am = L.maxpool_sk(x, 2, 2, 1)
    assert np.array_equal(y.ravel(), _hand(golden_rows, "pool_k2_d2"))
    yy, xx = np.mgrid[0:3, 0:3]
    assert np.array_equal(am[0, 0], (yy + 2) * 5 + xx + 2)      # last tap wins on a rising ramp


def test_hand_conv_k3_d1(golden_rows):
    x = np.arange(25.0).reshape(1, 1, 5, 5)
    w = np.array([[[[1.0, 0, -1], [2, 0, -2], [1, 0, -1]]]])
    y = L.conv_sk(x, w, np.array([0.5]), d=1)
    assert np.array_equal(y.ravel(), _hand(golden_rows, "conv_k3_d1"))


def test_hand_conv_3x3(golden_rows):
    x = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    y = L.conv_sk(x, np.array([[[[1.0, -1.0], [2.0, 3.0]]]]), np.array([1.0]), d=1)
    assert np.array_equal(y.ravel(), _hand(golden_rows, "conv_3x3_k2"))


def test_pool_tie_first_maximum_wins():
    x = np.zeros((1, 2, 6, 6))
    _, am = L.maxpool_sk(x, 2, 2, 1)
    yy, xx = np.mgrid[0:4, 0:4]
    assert np.array_equal(am[0, 0], yy * 6 + xx)                 # tap (0,0)
    x[0, 1, 2, :] = 1.0                                          # ties between taps (1,0) and (1,1)
    _, am = L.maxpool_sk(x, 2, 2, 1)
    assert np.array_equal(am[0, 1, 0], 2 * 6 + np.arange(4))     # tap (1,0) comes first


# ------------------------------------------------------------------ Algorithm 1 and the tables
def _sw_from_table(rows):
    sw = []
    for name, typ, w_sk, f_in, f_out, k, d, w_sw in rows[1:]:
        if typ == "conv":
            sw.append({"type": "conv", "f_out": int(f_out), "k": int(k), "relu": True})
        elif typ == "pool":
            sw.append({"type": "pool", "k": int(k), "s": int(k)})
        else:
            sw.append({"type": "ip", "f_out": int(f_out), "relu": name != "ip3"})
    return sw


def test_alg1_reproduces_sk_table(golden_rows):
    rows = golden_rows("sknet_table.txt")
    sw = _sw_from_table(rows)
    sk, w_sw, w_sk = alg1.convert_sw_to_sk(sw, 102)
    assert w_sw == [int(r[7]) for r in rows]
    assert [l["k"] for l in sk] == [int(r[5]) for r in rows[1:]]
    assert [l["d"] for l in sk] == [int(r[6]) for r in rows[1:]]
    assert w_sk[-1] == 1
    assert alg1.sk_sizes(sk, 229) == [int(r[2]) for r in rows]
    assert alg1.context(sk) == 101                                # Section 3.3.2: v = 101
    # w_SK^(N) = w_SK^(0) - w_SW^(0) + 1
    for w0 in (102, 103, 150, 229):
        assert alg1.sk_sizes(sk, w0)[-1] == w0 - 102 + 1


def test_alg1_rejects_uncorrected_sw_table(golden_rows):
    sw = _sw_from_table(golden_rows("sknet_table.txt"))
    with pytest.raises(alg1.ConversionError):                     # 43 mod 2 != 0 at pool2
        alg1.convert_sw_to_sk(sw, 100)


def test_alg1_error_cases():
    conv = {"type": "conv", "f_out": 4, "k": 3, "relu": True}
    with pytest.raises(alg1.ConversionError):                     # k != s
        alg1.convert_sw_to_sk([conv, {"type": "pool", "k": 2, "s": 1}], 10)
    with pytest.raises(alg1.ConversionError):                     # ends with d != 1
        alg1.convert_sw_to_sk([conv, {"type": "pool", "k": 2, "s": 2}], 10)
    with pytest.raises(alg1.ConversionError):                     # non-elementwise unknown layer
        alg1.convert_sw_to_sk([{"type": "other", "k": 3}], 10)
    sk, _, _ = alg1.convert_sw_to_sk([{"type": "other", "k": 1}, conv], 10)
    assert sk[1]["d"] == 1


def test_figure_example_three_by_three_output():
    # Figure "SK feature maps": input two pixels larger than the SW patch -> 3x3 output
    sk, w_sw, _ = alg1.convert_sw_to_sk(S.tiny_sw_layers(), 15)
    assert alg1.sk_sizes(sk, 17)[-1] == 3
    # with k = 1 the kernel stride is immaterial (Section 3.3.2 sets it to 1 for such layers)
    norm = lambda ls: [dict(l, d=1) if l["k"] == 1 else l for l in ls]
    assert norm(sk) == S.tiny_sknet_layers()
    assert w_sw == [15, 12, 6, 2, 1, 1, 1]


def test_unet_and_usk_table_sizes(golden_rows):
    for fname in ("unet_table.txt", "usknet_table.txt"):
        rows = golden_rows(fname)
        w = int(rows[0][2])
        for r in rows[1:]:
            typ, k = r[1], int(r[5])
            d = int(r[7]) if len(r) > 7 else 1
            s = int(r[6])
            if typ == "conv":
                lay = [{"type": "conv", "f_out": 1, "k": k, "d": d}]
            elif typ == "pool":
                lay = [{"type": "pool", "k": k, "d": d, "s": s}]
            elif typ == "upconv":
                lay = [{"type": "upconv"}]
            else:
                lay = [{"type": "other", "k": 1}]
            w = alg1.sk_sizes(lay, w)[-1]
            assert w == int(r[2]), (fname, r[0])


def _table_layers(rows):
    lays = []
    for r in rows[1:]:
        typ, k, s = r[1], int(r[5]), int(r[6])
        d = int(r[7]) if len(r) > 7 else 1
        if typ == "conv":
            lays.append({"type": "conv", "f_out": int(r[4]), "k": k, "d": d})
        elif typ == "pool":
            lays.append({"type": "pool", "k": k, "d": d, "s": s})
        elif typ == "upconv":
            lays.append({"type": "upconv"})
        else:
            lays.append({"type": "other", "k": 1})
    return lays


def test_flop_counter_matches_printed_gflop(golden_rows):
    sk_rows = golden_rows("sknet_table.txt")
    tables = {"sk": (sk_rows, [int(r[2]) for r in sk_rows])}
    for net, fname, w0 in (("u", "unet_table.txt", 572), ("usk", "usknet_table.txt", 256 + 180)):
        rows = golden_rows(fname)
        tables[net] = (rows, alg1.sk_sizes(_table_layers(rows), w0))
    assert tables["usk"][1][-1] == 256 and tables["u"][1][-1] == 388
    for net, layer, gflop in golden_rows("conv_gflop.txt"):
        rows, sizes = tables[net]
        idx = [r[0] for r in rows].index(layer)
        f_in, f_out, k = int(rows[idx][3]), int(rows[idx][4]), int(rows[idx][5])
        got = alg1.conv_flops(f_in, f_out, k, sizes[idx]) / 1e9
        assert abs(got - float(gflop)) <= 0.00501, (net, layer, got, gflop)


def test_parameter_counts_and_buffer_limit(golden_rows):
    def convs(rows):
        return [(int(r[3]), int(r[4]), int(r[5])) for r in rows if r[1] in ("conv", "ip")]
    sk = alg1.free_parameters(convs(golden_rows("sknet_table.txt")))
    assert sk == 20567952 and round(sk / 1e6, 1) in (20.5, 20.6)  # "about 20.5e6"
    assert 192 * 1024 * 100 == 19660800                           # ip1 "about 19.6e6"
    u = alg1.free_parameters(convs(golden_rows("unet_table.txt")))
    assert round(u / 1e6) == 29                                    # "about 29e6"
    usk = alg1.free_parameters(convs(golden_rows("usknet_table.txt")))
    assert abs(usk / 1e6 - 5.5) < 0.1                              # "about 5.5e6"
    # Section 6.4: a 4 GiB column buffer limits ip1 (f_in 192, k 10) to w of about 236
    assert alg1.conv_buffer_elements(192, 10, 236) * 4 <= 4 * 2 ** 30
    assert alg1.conv_buffer_elements(192, 10, 237) * 4 > 4 * 2 ** 30


# ------------------------------------------------------------------ SK == SW, brute force
def _net_weights(sk_layers, c_in, seed):
    ws, bs = S.he_normal_weights(sk_layers, c_in, seed, bias_scale=0.3)
    return [w.astype(np.float64) for w in ws], [b.astype(np.float64) for b in bs]


@pytest.mark.parametrize("hw", [(1, 1), (3, 3), (6, 9)])
def test_sk_equals_sliding_window_tiny_net(hw):
    sw = S.tiny_sw_layers()
    sk, _, _ = alg1.convert_sw_to_sk(sw, 15)
    ws, bs = _net_weights(sk, 1, 11)
    h, w = hw
    img = rng(5).random((1, 1, h + 14, w + 14))
    dense = nets.sknet_forward(img, sk, ws, bs, pad=False)
    assert dense.shape == (1, 2, h, w)
    brute = sw_net.sw_forward_image(img[0], sw, 15, ws, bs)
    assert np.abs(dense[0] - brute).max() < 1e-12


def test_sk_equals_sliding_window_two_stage_k4_net_two_channels():
    # cut-down version of the benchmark net: patch 13 -> 10 -> 5 -> 2 -> 1; ip kernel 1
    sw = [{"type": "conv", "f_out": 5, "k": 4, "relu": True}, {"type": "pool", "k": 2, "s": 2},
          {"type": "conv", "f_out": 6, "k": 4, "relu": True}, {"type": "pool", "k": 2, "s": 2},
          {"type": "ip", "f_out": 7, "relu": True}, {"type": "ip", "f_out": 3, "relu": False}]
    sk, w_sw, _ = alg1.convert_sw_to_sk(sw, 13)
    assert w_sw == [13, 10, 5, 2, 1, 1, 1] and [l["d"] for l in sk] == [1, 1, 2, 2, 4, 1]
    ws, bs = _net_weights(sk, 2, 12)
    img = rng(6).random((1, 2, 12 + 5, 12 + 4))
    dense = nets.sknet_forward(img, sk, ws, bs, pad=False)
    brute = sw_net.sw_forward_image(img[0], sw, 13, ws, bs)
    assert dense.shape[2:] == (5, 4)
    assert np.abs(dense[0] - brute).max() < 1e-12


def test_sk_equals_sliding_window_with_spanning_inner_product():
    # an inner product that spans a 3x3 remaining map becomes a k=3 conv at d=2 (the figure's case)
    sw = [{"type": "conv", "f_out": 3, "k": 3, "relu": True}, {"type": "pool", "k": 2, "s": 2},
          {"type": "ip", "f_out": 4, "relu": True}, {"type": "ip", "f_out": 2, "relu": False}]
    sk, w_sw, _ = alg1.convert_sw_to_sk(sw, 8)
    assert w_sw == [8, 6, 3, 1, 1] and sk[2]["k"] == 3 and sk[2]["d"] == 2
    ws, bs = _net_weights(sk, 1, 13)
    img = rng(7).random((1, 1, 7 + 4, 7 + 6))
    dense = nets.sknet_forward(img, sk, ws, bs, pad=False)
    brute = sw_net.sw_forward_image(img[0], sw, 8, ws, bs)
    assert np.abs(dense[0] - brute).max() < 1e-12


def test_output_size_invariance_tile_and_stitch():
    # Section 3.1: any output size gives numerically identical results -> tiles with a halo stitch
    sk = S.tiny_sknet_layers()
    ws, bs = _net_weights(sk, 1, 14)
    img = rng(8).random((1, 1, 40, 40))
    v = alg1.context(sk)
    t, l, b, r = nets.pad_amounts(v)
    padded = L.mirror_pad(img, t, l, b, r)
    whole = nets.sknet_forward(padded, sk, ws, bs, pad=False)
    assert np.array_equal(whole, nets.sknet_forward(img, sk, ws, bs, pad=True))
    stitched = np.empty_like(whole)
    for y0 in (0, 20):
        for x0 in (0, 20):
            tile = padded[:, :, y0:y0 + 20 + v, x0:x0 + 20 + v]
            stitched[:, :, y0:y0 + 20, x0:x0 + 20] = nets.sknet_forward(tile, sk, ws, bs, pad=False)
    assert np.abs(stitched - whole).max() < 1e-13


# ------------------------------------------------------------------ special cases vs libraries
def test_conv_d1_equals_textbook_correlation():
    x = rng(1).standard_normal((2, 3, 9, 11))
    w = rng(2).standard_normal((4, 3, 3, 3))
    b = rng(3).standard_normal(4)
    y = L.conv_sk(x, w, b, d=1)
    for n in range(2):
        for o in range(4):
            ref = sum(scipy.signal.correlate2d(x[n, c], w[o, c], mode="valid") for c in range(3)) + b[o]
            assert np.abs(y[n, o] - ref).max() < 1e-12


@pytest.mark.parametrize("k,d", [(4, 1), (4, 2), (5, 2), (3, 4), (2, 8), (1, 1)])
def test_conv_dilated_matches_torch(k, d):
    x = rng(4).standard_normal((2, 3, 30, 33))
    w = rng(5).standard_normal((5, 3, k, k))
    b = rng(6).standard_normal(5)
    y = L.conv_sk(x, w, b, d=d, relu=True)
    ref = F.relu(F.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), dilation=d))
    assert y.shape == tuple(ref.shape)
    assert np.abs(y - ref.numpy()).max() < 1e-11


def test_pool_d1_equals_maximum_filter():
    x = rng(7).standard_normal((1, 2, 12, 13))
    y, _ = L.maxpool_sk(x, 2, 1, 1)
    for c in range(2):
        ref = scipy.ndimage.maximum_filter(x[0, c], size=2, origin=(-1, -1), mode="nearest")[:-1, :-1]
        assert np.array_equal(y[0, c], ref)


@pytest.mark.parametrize("k,d,s", [(2, 1, 1), (2, 2, 1), (2, 4, 1), (2, 8, 1), (3, 2, 1), (2, 1, 2)])
def test_pool_matches_torch_and_argmax_points_at_max(k, d, s):
    x = rng(8).standard_normal((2, 3, 26, 28))
    y, am = L.maxpool_sk(x, k, d, s)
    ref = F.max_pool2d(torch.from_numpy(x), k, stride=s, dilation=d)
    assert np.array_equal(y, ref.numpy())
    flat = x.reshape(2, 3, -1)
    assert np.array_equal(np.take_along_axis(flat, am.reshape(2, 3, -1).astype(np.int64), 2).reshape(y.shape), y)
    # the winner lies inside the window of its output
    ho, wo = y.shape[2:]
    yy, xx = np.mgrid[0:ho, 0:wo]
    ay, ax = am // 28, am % 28
    assert ((ay - s * yy) % d == 0).all() and ((ax - s * xx) % d == 0).all()
    assert ((ay - s * yy) // d < k).all() and ((ax - s * xx) // d < k).all() and (ay >= s * yy).all()


@pytest.mark.parametrize("mode,npmode", [(0, "reflect"), (1, "symmetric")])
def test_mirror_pad_matches_numpy(mode, npmode):
    x = rng(9).standard_normal((2, 2, 7, 9))
    y = L.mirror_pad(x, 4, 5, 3, 6, mode)
    ref = np.pad(x, ((0, 0), (0, 0), (4, 3), (5, 6)), mode=npmode)
    assert np.array_equal(y, ref)
    with pytest.raises(ValueError):
        L.mirror_pad(x, 8, 0, 0, 0, 0)


def test_pad_amounts_odd_context():
    assert nets.pad_amounts(101) == (51, 51, 50, 50)              # Section 3.3.2
    assert nets.pad_amounts(60) == (30, 30, 30, 30)


# ------------------------------------------------------------------ softmax and loss
def test_softmax_closed_forms():
    z = rng(10).standard_normal((2, 2, 5, 6)) * 4
    p = L.softmax(z)
    assert np.abs(p.sum(1) - 1).max() < 1e-15
    assert np.abs(p[:, 1] - 1.0 / (1.0 + np.exp(z[:, 0] - z[:, 1]))).max() < 1e-15
    assert np.abs(L.softmax(z + 123.0) - p).max() < 1e-13          # shift invariance
    z3 = rng(11).standard_normal((1, 5, 3, 3))
    e = np.exp(z3)
    assert np.abs(L.softmax(z3) - e / e.sum(1, keepdims=True)).max() < 1e-15
    assert np.isfinite(L.softmax(z * 500)).all()


def test_softmax_loss_closed_forms():
    lab = rng(12).integers(0, 3, (2, 4, 5)).astype(np.int32)
    loss, dz = L.softmax_loss(np.full((2, 3, 4, 5), 0.7), lab)
    assert abs(loss - np.log(3.0)) < 1e-15                         # uniform logits -> ln C
    z = rng(13).standard_normal((2, 3, 4, 5))
    loss, dz = L.softmax_loss(z, lab)
    p = L.softmax(z)
    pick = np.take_along_axis(p, lab[:, None].astype(np.int64), 1)
    assert abs(loss + np.log(pick).mean()) < 1e-14
    onehot = np.eye(3)[lab].transpose(0, 3, 1, 2)
    assert np.abs(dz - (p - onehot) / 40.0).max() < 1e-16
    ref = F.cross_entropy(torch.from_numpy(z), torch.from_numpy(lab).long())
    assert abs(loss - ref.item()) < 1e-14


def test_softmax_loss_with_masked_pixels():
    # masked pixels (label -1): the loss is the plain loss of the unmasked subset, their gradient is zero,
    # the normaliser is the number of unmasked pixels; the library's ignore_index is the same rule
    z = rng(14).standard_normal((2, 3, 6, 7))
    lab = rng(15).integers(0, 3, (2, 6, 7)).astype(np.int32)
    masked = lab.copy()
    masked[rng(16).random(lab.shape) < 0.4] = -1
    keep = masked >= 0
    loss, dz = L.softmax_loss(z, masked)
    p = L.softmax(z)
    pick = np.take_along_axis(p, lab[:, None].astype(np.int64), 1)[:, 0]
    assert abs(loss + np.log(pick[keep]).mean()) < 1e-14
    onehot = np.eye(3)[lab].transpose(0, 3, 1, 2)
    expect = (p - onehot) / keep.sum() * keep[:, None]
    assert np.abs(dz - expect).max() < 1e-16
    assert (dz[np.broadcast_to(~keep[:, None], dz.shape)] == 0).all()
    ref = F.cross_entropy(torch.from_numpy(z), torch.from_numpy(masked).long(), ignore_index=-1)
    assert abs(loss - ref.item()) < 1e-14
    # nothing masked: the rule reduces to the mean over all pixels
    assert L.softmax_loss(z, lab)[0] == L.softmax_loss(z, np.where(keep, lab, lab))[0]
    # everything masked: zero loss, zero gradient
    loss0, dz0 = L.softmax_loss(z, np.full_like(lab, -1))
    assert loss0 == 0.0 and not dz0.any()


def test_label_masking_balances_the_histogram():
    # Section 4.2: after masking, every label that occurs is left about equally often and the rarest
    # one is never masked
    lab = (rng(17).random((4, 200, 200)) < 0.15).astype(np.int32) + (rng(18).random((4, 200, 200)) < 0.02)
    masked = S.mask_labels_by_frequency(lab, 3, 19)
    before = np.bincount(lab.reshape(-1), minlength=3)
    after = np.bincount(masked[masked >= 0], minlength=3)
    assert ((masked == lab) | (masked == -1)).all()
    assert after[before.argmin()] == before.min()
    assert after.max() / after.min() < 1.15


# ------------------------------------------------------------------ backward passes
def _fd(f, x, eps=1e-6):
    g = np.zeros_like(x)
    flat, gf = x.reshape(-1), g.reshape(-1)
    for i in range(flat.size):
        old = flat[i]
        flat[i] = old + eps
        fp = f()
        flat[i] = old - eps
        fm = f()
        flat[i] = old
        gf[i] = (fp - fm) / (2 * eps)
    return g


@pytest.mark.parametrize("k,d", [(3, 1), (2, 2), (4, 2), (2, 3)])
def test_conv_backward_finite_differences_and_adjoint(k, d):
    x = rng(20).standard_normal((2, 2, 6 + (k - 1) * d, 5 + (k - 1) * d))
    w = rng(21).standard_normal((3, 2, k, k))
    b = rng(22).standard_normal(3)
    dy = rng(23).standard_normal((2, 3, 6, 5))
    f = lambda: float((L.conv_sk(x, w, b, d) * dy).sum())
    dx = L.conv_sk_bwd_data(dy, w, d, x.shape[2:])
    dw, db = L.conv_sk_bwd_weights(x, dy, k, d)
    assert np.abs(dx - _fd(f, x)).max() < 1e-7
    assert np.abs(dw - _fd(f, w)).max() < 1e-7
    assert np.abs(db - _fd(f, b)).max() < 1e-7
    # adjoint identity <conv(X), dY> = <X, dgrad(dY)> (zero bias)
    assert abs((L.conv_sk(x, w, None, d) * dy).sum() - (x * dx).sum()) < 1e-10
    # and against the library's autograd
    xt = torch.from_numpy(x).requires_grad_()
    wt = torch.from_numpy(w).requires_grad_()
    (F.conv2d(xt, wt, dilation=d) * torch.from_numpy(dy)).sum().backward()
    assert np.abs(dx - xt.grad.numpy()).max() < 1e-11 and np.abs(dw - wt.grad.numpy()).max() < 1e-11


@pytest.mark.parametrize("k,d,s", [(2, 1, 1), (2, 2, 1), (2, 4, 1), (2, 1, 2)])
def test_pool_backward_scatter(k, d, s):
    x = rng(24).standard_normal((1, 2, 12, 14))                   # tie-free with probability 1
    y, am = L.maxpool_sk(x, k, d, s)
    dy = rng(25).standard_normal(y.shape)
    dx = L.maxpool_bwd(dy, am, x.shape[2:])
    assert abs(dx.sum() - dy.sum()) < 1e-12
    f = lambda: float((L.maxpool_sk(x, k, d, s)[0] * dy).sum())
    assert np.abs(dx - _fd(f, x, 1e-7)).max() < 1e-6
    xt = torch.from_numpy(x).requires_grad_()
    (F.max_pool2d(xt, k, stride=s, dilation=d) * torch.from_numpy(dy)).sum().backward()
    assert np.abs(dx - xt.grad.numpy()).max() < 1e-13


def test_relu_backward_zero_at_zero():
    y = np.array([0.0, 1.0, 0.0, 2.5])
    assert np.array_equal(L.relu_bwd(y, np.array([5.0, 6.0, 7.0, 8.0])), [0.0, 6.0, 0.0, 8.0])


def test_whole_net_backward_finite_differences():
    sk = [S.conv(3, 2, 1), S.pool(2, 1), S.conv(4, 2, 2), S.pool(2, 2), S.conv(5, 1, 1),
          S.conv(2, 1, 1, relu=False)]
    ws, bs = _net_weights(sk, 2, 30)
    img = rng(31).standard_normal((2, 2, 5, 6))
    lab = rng(32).integers(0, 2, (2, 5, 6)).astype(np.int32)

    def loss():
        _, acts, _ = nets.sknet_forward(img, sk, ws, bs, pad=True, keep=True)
        return L.softmax_loss(acts[-1], lab, want_grad=False)[0]

    _, acts, ams = nets.sknet_forward(img, sk, ws, bs, pad=True, keep=True)
    l0, dws, dbs, _ = nets.sknet_backward(sk, ws, acts, ams, lab)
    assert abs(l0 - loss()) < 1e-15
    for i in range(len(ws)):
        assert np.abs(dws[i] - _fd(loss, ws[i])).max() < 1e-7, i
        assert np.abs(dbs[i] - _fd(loss, bs[i])).max() < 1e-7, i


def test_sgd_closed_form_and_first_order_decrease():
    w = np.array([1.0, -2.0, 0.5])
    g = np.array([0.1, 0.2, -0.3])
    vel = np.array([0.01, 0.0, -0.02])
    w1 = L.sgd(w.copy(), g, None, 0.5)
    assert np.allclose(w1, w - 0.5 * g, atol=1e-16)
    w2, v2 = w.copy(), vel.copy()
    L.sgd(w2, g, v2, 0.5, 0.9, 0.01)
    vref = 0.9 * vel + 0.5 * (g + 0.01 * w)
    assert np.allclose(v2, vref, atol=1e-16) and np.allclose(w2, w - vref, atol=1e-16)
    # one small step lowers the loss by about lr * |g|^2
    sk = S.tiny_sknet_layers()
    ws, bs = _net_weights(sk, 1, 40)
    img = rng(41).random((1, 1, 12, 12))
    lab = rng(42).integers(0, 2, (1, 12, 12)).astype(np.int32)
    _, acts, ams = nets.sknet_forward(img, sk, ws, bs, keep=True)
    l0, dws, dbs, _ = nets.sknet_backward(sk, ws, acts, ams, lab)
    lr = 1e-5
    nets.sgd_step(ws, bs, dws, dbs, lr)
    _, acts, _ = nets.sknet_forward(img, sk, ws, bs, keep=True)
    l1 = L.softmax_loss(acts[-1], lab, want_grad=False)[0]
    g2 = sum((d ** 2).sum() for d in dws) + sum((d ** 2).sum() for d in dbs)
    assert abs((l0 - l1) - lr * g2) < 1e-3 * lr * g2


# ------------------------------------------------------------------ U-Net pieces
def test_nearest_neighbour_upconv_fills_two_by_two_blocks():
    x = rng(50).standard_normal((1, 3, 4, 5))
    w = np.zeros((3, 3, 2, 2))
    for c in range(3):
        w[c, c] = 1.0
    y = L.upconv2x2(x, w)
    assert np.array_equal(y, np.repeat(np.repeat(x, 2, 2), 2, 3))


def test_upconv_matches_transposed_convolution_and_paper_two_layer_form():
    x = rng(51).standard_normal((2, 4, 3, 5))
    w = rng(52).standard_normal((4, 2, 2, 2))
    b = rng(53).standard_normal(2)
    y = L.upconv2x2(x, w, b)
    ref = F.conv_transpose2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), stride=2)
    assert np.abs(y - ref.numpy()).max() < 1e-13
    # paper's form: nearest-neighbour up-sampling of every map, then a 1x1 convolution
    w1 = rng(54).standard_normal((2, 4, 1, 1))
    two_layer = L.conv_sk(np.repeat(np.repeat(x, 2, 2), 2, 3), w1, b, d=1)
    fused = L.upconv2x2(x, nets.upstep_from_paper(w1), b)
    assert np.abs(two_layer - fused).max() < 1e-13


def test_mergecrop_order_and_offsets():
    for wa, wb, off in ((56, 64, 4), (104, 136, 16), (200, 280, 40), (392, 568, 88)):
        assert (wb - wa) // 2 == off
    a = rng(55).standard_normal((1, 2, 4, 6))
    b = rng(56).standard_normal((1, 3, 8, 12))
    out = L.mergecrop(a, b)
    assert np.array_equal(out[:, :2], a) and np.array_equal(out[:, 2:], b[:, :, 2:6, 3:9])
    # backward: the copy's adjoint (<mergecrop(a, b), g> = <a, dA> + <b, dB>) when B takes gradient, and
    # Section 5.3.1's rule for the U- and USK-Net (A only: B gets nothing from this layer)
    g = rng(57).standard_normal(out.shape)
    da, db = L.mergecrop_bwd(g, 2, b.shape, into_b=True)
    assert abs((out * g).sum() - (a * da).sum() - (b * db).sum()) < 1e-12
    assert np.count_nonzero(db) == 3 * 4 * 6 and np.array_equal(db[:, :, 2:6, 3:9], g[:, 2:])
    da2, db2 = L.mergecrop_bwd(g, 2, b.shape)
    assert np.array_equal(da2, g[:, :2]) and not db2.any()


def test_unet_small_forward_shape_and_torch_crosscheck():
    # depth-2 U-Net on 44x44: 44-40-20-16-8-4 | up 8-4 | up 8-4 -> output 4x4
    params = {k: (w.astype(np.float64), b.astype(np.float64))
              for k, (w, b) in S.unet_params(1, 2, 60, depth=2, base=4, bias_scale=0.2).items()}
    img = rng(61).random((1, 1, 44, 44))
    prob, tr = nets.unet_forward(img, params, depth=2, keep=True)
    assert prob.shape == (1, 2, 4, 4)
    t = lambda a: torch.from_numpy(a)
    x = t(img)
    skips = []
    for i in range(3):
        x = F.relu(F.conv2d(x, t(params["down%da" % i][0]), t(params["down%da" % i][1])))
        x = F.relu(F.conv2d(x, t(params["down%db" % i][0]), t(params["down%db" % i][1])))
        if i < 2:
            skips.append(x)
            x = F.max_pool2d(x, 2)
    for i in (1, 0):
        x = F.conv_transpose2d(x, t(params["up%d" % i][0]), t(params["up%d" % i][1]), stride=2)
        sk = skips[i]
        o = (sk.shape[2] - x.shape[2]) // 2
        x = torch.cat([x, sk[:, :, o:o + x.shape[2], o:o + x.shape[3]]], 1)
        x = F.relu(F.conv2d(x, t(params["dec%da" % i][0]), t(params["dec%da" % i][1])))
        x = F.relu(F.conv2d(x, t(params["dec%db" % i][0]), t(params["dec%db" % i][1])))
    z = F.conv2d(x, t(params["head"][0]), t(params["head"][1]))
    assert np.abs(tr["logits"] - z.numpy()).max() < 1e-12
    assert np.abs(prob - F.softmax(z, 1).numpy()).max() < 1e-14


def test_usknet_forward_table_sizes_and_torch_crosscheck(golden_rows):
    # The USK table's sizes (692 -> 512) with 1/32 of its channels, and the same composition written
    # with the library's dilated convolution / pooling / transposed convolution.
    base = 2
    params = {k: (w.astype(np.float64), b.astype(np.float64))
              for k, (w, b) in S.usknet_params(3, 2, 70, base=base, bias_scale=0.2).items()}
    img = rng(71).random((1, 3, 692, 692))
    prob, tr = nets.usknet_forward(img, params, base=base, keep=True)
    table = {r[0]: int(r[2]) for r in golden_rows("usknet_table.txt")}
    for stage, row in (("conv2", "conv2"), ("pool1", "pool1"), ("conv3", "conv3"), ("pool2", "pool2"), ("conv4", "conv4"),
                       ("pool3", "pool3"), ("conv5", "conv5"), ("pool4", "pool4"), ("ip1", "ip1"), ("ip2", "ip2"),
                       ("up1", "conv6"), ("conv8", "conv8"), ("logits", "ip3")):
        assert tr[stage].shape[2] == tr[stage].shape[3] == table[row], (stage, tr[stage].shape)
    assert tr["ip1"].shape[1] == 8 * base and tr["up1"].shape[1] == 2 * base
    t = lambda a: torch.from_numpy(a)
    cv = lambda x, name, d=1: F.conv2d(x, t(params[name][0]), t(params[name][1]), dilation=d)
    x = F.relu(cv(F.relu(cv(t(img), "conv1")), "conv2"))
    skip = x
    x = F.max_pool2d(x, 2)
    for name, d in (("conv3", 1), ("conv4", 2), ("conv5", 4)):
        x = F.max_pool2d(F.relu(cv(x, name, d)), 2, stride=1, dilation=d)
    x = F.relu(cv(F.relu(cv(x, "ip1", 8)), "ip2"))
    x = F.conv_transpose2d(x, t(params["up1"][0]), t(params["up1"][1]), stride=2)
    o = (skip.shape[2] - x.shape[2]) // 2
    assert o == 86
    x = torch.cat([x, skip[:, :, o:o + x.shape[2], o:o + x.shape[3]]], 1)
    x = F.relu(cv(F.relu(cv(x, "conv7")), "conv8"))
    z = cv(x, "ip3")
    assert np.abs(tr["logits"] - z.numpy()).max() < 1e-11
    assert np.abs(prob - F.softmax(z, 1).numpy()).max() < 1e-13


def _torch_grads(loss, tparams):
    loss.backward()
    return {k: (w.grad.numpy(), b.grad.numpy()) for k, (w, b) in tparams.items()}


@pytest.mark.parametrize("merge_into_b", [False, True])
def test_unet_backward_matches_autograd(merge_into_b):
    # depth-2 U-Net on 44x44 with masked labels: every parameter gradient against the library's
    # reverse-mode differentiation of the same composition.  merge_into_b=False is Section 5.3.1's rule
    # (MergeCrop backwards into the up path only): the skip map enters the concatenation as a constant;
    # merge_into_b=True is the exact derivative of the whole composite.
    params = {k: (w.astype(np.float64), b.astype(np.float64))
              for k, (w, b) in S.unet_params(2, 3, 80, depth=2, base=4, bias_scale=0.2).items()}
    img = rng(81).random((2, 2, 44, 44))
    lab = rng(82).integers(-1, 3, (2, 4, 4)).astype(np.int32)
    loss, grads = nets.unet_backward(img, params, lab, depth=2, merge_into_b=merge_into_b)
    tp = {k: (torch.from_numpy(w).requires_grad_(), torch.from_numpy(b).requires_grad_()) for k, (w, b) in params.items()}
    x = torch.from_numpy(img)
    skips = []
    for i in range(3):
        x = F.relu(F.conv2d(x, *tp["down%da" % i]))
        x = F.relu(F.conv2d(x, *tp["down%db" % i]))
        if i < 2:
            skips.append(x)
            x = F.max_pool2d(x, 2)
    for i in (1, 0):
        x = F.conv_transpose2d(x, *tp["up%d" % i], stride=2)
        sk = skips[i] if merge_into_b else skips[i].detach()
        o = (sk.shape[2] - x.shape[2]) // 2
        x = torch.cat([x, sk[:, :, o:o + x.shape[2], o:o + x.shape[3]]], 1)
        x = F.relu(F.conv2d(x, *tp["dec%da" % i]))
        x = F.relu(F.conv2d(x, *tp["dec%db" % i]))
    z = F.conv2d(x, *tp["head"])
    tl = F.cross_entropy(z, torch.from_numpy(lab).long(), ignore_index=-1)
    assert abs(loss - tl.item()) < 1e-13
    ref = _torch_grads(tl, tp)
    for k in params:
        for got, want in zip(grads[k], ref[k]):
            assert np.abs(got - want).max() <= 1e-12 * max(1.0, np.abs(want).max()), k


@pytest.mark.parametrize("merge_into_b", [False, True])
def test_usknet_backward_matches_autograd(merge_into_b):
    base = 2
    params = {k: (w.astype(np.float64), b.astype(np.float64))
              for k, (w, b) in S.usknet_params(2, 3, 83, base=base, bias_scale=0.2).items()}
    img = rng(84).random((1, 2, 190, 186))
    ho, wo = 2 * ((190 - 4) // 2 - 86) - 4, 2 * ((186 - 4) // 2 - 86) - 4
    lab = rng(85).integers(-1, 3, (1, ho, wo)).astype(np.int32)
    loss, grads = nets.usknet_backward(img, params, lab, base=base, merge_into_b=merge_into_b)
    tp = {k: (torch.from_numpy(w).requires_grad_(), torch.from_numpy(b).requires_grad_()) for k, (w, b) in params.items()}
    cv = lambda x, name, d=1: F.conv2d(x, *tp[name], dilation=d)
    x = F.relu(cv(F.relu(cv(torch.from_numpy(img), "conv1")), "conv2"))
    skip = x
    x = F.max_pool2d(x, 2)
    for name, d in (("conv3", 1), ("conv4", 2), ("conv5", 4)):
        x = F.max_pool2d(F.relu(cv(x, name, d)), 2, stride=1, dilation=d)
    x = F.relu(cv(F.relu(cv(x, "ip1", 8)), "ip2"))
    x = F.conv_transpose2d(x, *tp["up1"], stride=2)
    oy, ox = (skip.shape[2] - x.shape[2]) // 2, (skip.shape[3] - x.shape[3]) // 2
    if not merge_into_b:
        skip = skip.detach()
    x = torch.cat([x, skip[:, :, oy:oy + x.shape[2], ox:ox + x.shape[3]]], 1)
    x = F.relu(cv(F.relu(cv(x, "conv7")), "conv8"))
    z = cv(x, "ip3")
    assert z.shape[2:] == (ho, wo)
    tl = F.cross_entropy(z, torch.from_numpy(lab).long(), ignore_index=-1)
    assert abs(loss - tl.item()) < 1e-13
    ref = _torch_grads(tl, tp)
    for k in params:
        for got, want in zip(grads[k], ref[k]):
            assert np.abs(got - want).max() <= 1e-12 * max(1.0, np.abs(want).max()), k
