"""Benchmark of the SK-Net hot path on one MI355X.  Prints ONE JSON line.

Default workload (BASELINE configs[1], the one the headline metric is quoted on): SK-Net forward on
one 1x1x512x512 fp32 image -- mirror padding, four stages of [conv k4 -> 48 maps + ReLU, max pool
k2 s1] at kernel strides 1/2/4/8, 1x1 conv 48 -> 200 + ReLU, 1x1 conv 200 -> 2, per-pixel softmax.
A step is one such pass over one synthetic image that is resident in HBM before the timed region.

--workload c3      : the same net in bf16 (fp32 accumulate) on 8 images of 1024x1024 (configs[2])
--workload c4      : one bf16 training step at 512x512 (configs[3]): forward, softmax loss, backward, SGD
--workload c3train : the same training step on 8 images of 1024x1024 (where the pool, pool-gradient and softmax-loss
                     kernels are bound by HBM, not by their launch)
--workload c5 / c5bf16 : U-Net forward on one 572x572 image (configs[4]) in fp32 / bf16
--workload papersk / paperskbf16, usk / uskbf16 : the paper's own SK-Net (128^2 tile) and USK-Net (692^2), fp32 / bf16
--workload sk3d / sk3dbf16 / sk3dtrain : 3-D SK net on a stack of 81 sections of 145x145 (Section 5.2.2), fp32 (bf16: forward)
--workload unettrain / usktrain : U-Net / USK-Net training step, fp32 (unettrainbf16 / usktrainbf16 / sk3dtrainbf16: bf16 storage)
--workload copy    : only the streaming-copy probe on 2 x 1 GiB (the known-size kernel that the HBM
                     byte counters of a profiler run are calibrated against)
The default run also appends short measurements of the other workloads under "extras" (skip with --no-extras).

Timing: the K steps are bracketed by synchronisation and a wall clock (ms_per_step, value); every step is also
bracketed by two HIP events on the stream it is launched on (median / min in ms_per_step_events).  Kernel times of
the roofline blocks come from HIP events inside the library (sknet_time_step, sknet_time_backward_step), on the same
stream.  HBM traffic beyond L2 is read from profiles/hbm_traffic.json (rocprofv3 --pmc runs of this script).
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0}   # MI355X dense MFMA peaks
HBM_PEAK_GBS = 8000.0
METRIC = "labelled pixels/sec SK-Net fwd (and fwd+bwd) 1 GPU; conv % MFMA peak"
NET_DESC = "4x[conv k4 48 + ReLU, pool k2] d=1/2/4/8, 1x1 48->200 + ReLU, 1x1 200->2, softmax"


def traffic_table():
    """Bytes moved beyond L2 per launch of the dominant kernels, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
    this script, already scaled by what the same counters read for the streaming copy of known size; the file names
    the summaries under profiles/ it was made from.  Missing file or entry: traffic is reported as null."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {}


def traffic_of(table, key):
    e = table.get(key)
    if not e:
        return None, None
    return int(e["bytes_per_launch"]), e.get("source")


def timed_steps(torch, fn, steps, warmup):
    """warmup untimed calls, then `steps` timed ones: wall clock over all of them, HIP events around each."""
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        fn()
        b.record(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per = [a.elapsed_time(b) for a, b in ev]
    return dt, {"median": round(statistics.median(per), 4), "min": round(min(per), 4)}


def build_net(B, S, dtype, n, H, W, training):
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    net = B.SKNet(layers, 1, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    # 16-bit training: the head (48 -> 200 -> 2) and the loss as one kernel in each direction (plan mode 3)
    net.plan(n, H, W, pad=True, training=training, fused_head=training and dtype != "f32")
    return net, layers, ws, bs


def layer_flops(layers, shapes, n):
    """(flops of every conv layer, maps entering every layer)"""
    fl, f_in_of, f_in = {}, {}, 1
    for li, l in enumerate(layers):
        f_in_of[li] = f_in
        if l["type"] == "conv":
            c, ho, wo = shapes[li + 1]
            fl[li] = 2.0 * f_in * l["k"] ** 2 * l["f_out"] * ho * wo * n
            f_in = l["f_out"]
    return fl, f_in_of


def measure_forward(torch, B, S, dtype, n, H, W, steps, warmup, first_seed, kernel_iters=20):
    net, layers, ws, bs = build_net(B, S, dtype, n, H, W, False)
    img = S.em_like_batch(n, H, W, first_seed)
    timg = torch.from_numpy(img).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    dt, per = timed_steps(torch, lambda: net.forward(timg, prob, stream), steps, warmup)
    ms_per_step = dt / steps * 1e3

    # per-kernel durations: HIP events recorded on the same stream, inside the library
    shapes = net.infer_shapes(H, W)
    esize = 4 if dtype == "f32" else 2
    flops, f_in_of = layer_flops(layers, shapes, n)
    step_ms, conv_flops, conv_ms = {}, 0.0, 0.0
    conv_bytes, conv_launches, conv_names = 0.0, 0, []
    pool_bytes, pool_ms = 0.0, 0.0
    for step in range(net.num_steps()):
        ms = net.time_step(step, kernel_iters, stream)
        name = net.step_name(step)
        step_ms[name] = round(ms, 5)
        m = re.match(r"(conv|pool)(\d+)_", name)
        if not m:
            continue
        li = int(m.group(2))
        l = layers[li]
        c, ho, wo = shapes[li + 1]
        if m.group(1) == "conv":
            if f_in_of[li] == 48 and l["f_out"] == 48:      # the dominant kernel: 48 -> 48, k4, dilated
                conv_flops += flops[li]
                conv_ms += ms
                hi, wi = shapes[li][1:]
                # every input and output element once (a fused pool shrinks neither: the convolution's output is
                # stored with W columns and H - d rows, its input arrives with d extra columns)
                conv_bytes += esize * n * 48.0 * (hi * wi + ho * wo)
                conv_launches += 1
                conv_names.append(name)
        else:                                         # pool as a layer of its own: one element read + one written
            pool_bytes += 2.0 * esize * n * c * ho * wo
            pool_ms += ms
    res = {
        "ms_per_step": ms_per_step, "events": per, "pixels_per_s": n * H * W * steps / dt, "step_ms": step_ms,
        "conv_tflops": conv_flops / (conv_ms * 1e-3) / 1e12, "conv_ms_avg": conv_ms / max(conv_launches, 1),
        "forward_tflops": sum(flops.values()) / (ms_per_step * 1e-3) / 1e12,
        "pool_gbs": (pool_bytes / (pool_ms * 1e-3) / 1e9) if pool_ms > 0 else None,
        "conv_alg_bytes": conv_bytes / max(conv_launches, 1), "conv_alg_flops": conv_flops / max(conv_launches, 1),
        "conv_names": conv_names, "layers": layers, "ws": ws, "bs": bs, "img": img,
    }
    if dtype != "f32" and any("pool" in nm for nm in conv_names):
        # the same layers as plain convolutions (a plan that keeps every layer: pools are launches of their own there),
        # to tell the convolution's own speed from the pool work its fused form carries
        net.plan(n, H, W, pad=True, keep=True)
        net.forward(timg, prob, stream)
        pf, pm, pn = 0.0, 0.0, 0
        for step in range(net.num_steps()):
            m = re.match(r"conv(\d+)_", net.step_name(step))
            if m and f_in_of[int(m.group(1))] == 48 and layers[int(m.group(1))]["f_out"] == 48:
                pm += net.time_step(step, kernel_iters, stream)
                pf += flops[int(m.group(1))]
                pn += 1
        if pn:
            res["conv_plain"] = {"avg_launch_ms": round(pm / pn, 5), "tflops": round(pf / (pm * 1e-3) / 1e12, 2)}
    net.close()
    return res


def forward_roofline(r, dtype, table, key):
    peak = PEAK_TFLOPS[dtype]
    traffic, src = traffic_of(table, key)
    return {"bound": "mfma", "achieved": round(r["conv_tflops"], 2), "peak": peak, "unit": "TFLOP/s",
            "frac": round(r["conv_tflops"] / peak, 4), "traffic": traffic,
            "traffic_unit": "bytes beyond L2 per launch (read + written)", "traffic_source": src,
            "algorithmic_bytes": int(r["conv_alg_bytes"]), "algorithmic_flops": int(r["conv_alg_flops"]),
            "avg_launch_ms": round(r["conv_ms_avg"], 5),
            "same_layers_without_pool_work": (dict(r["conv_plain"], frac=round(r["conv_plain"]["tflops"] / peak, 4),
                                                   what="the three layers in a plan that keeps the pools as launches (mode 2)")
                                              if r.get("conv_plain") else None),
            "kernel": "48->48 k4 SK convolutions at d=2,4,8 (%s): %s"
                      % ("conv_f32_pf_kernel<3,1,4,4,2,false,4>" if dtype == "f32" else "conv_h_ring_kernel, producer-wave variant",
                         ", ".join(r["conv_names"]))}


def measure_train(torch, B, S, dtype, n, H, W, steps, warmup, first_seed, kernel_iters=10, detail=True):
    net, layers, ws, bs = build_net(B, S, dtype, n, H, W, True)
    timg = torch.from_numpy(S.em_like_batch(n, H, W, first_seed)).cuda()
    labels = torch.from_numpy(S.binary_labels(n, H, W, 2004)).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def one():
        net.forward(timg, prob, stream)
        net.backward(labels, loss, stream)
        net.sgd_step(0.01, stream=stream)

    dt, per = timed_steps(torch, one, steps, warmup)
    res = {"pixels_per_s": n * H * W * steps / dt, "ms_per_step": dt / steps * 1e3, "events": per, "steps": steps}
    if detail:
        shapes = net.infer_shapes(H, W)
        esize = 4 if dtype == "f32" else 2
        flops, f_in_of = layer_flops(layers, shapes, n)
        net.forward(timg, prob, stream)
        parts, wg_ms, wg_flops, wg_bytes, wg_n = {}, 0.0, 0.0, 0.0, 0
        pool_bwd_bytes, pool_bwd_ms, pool_fwd_bytes, pool_fwd_ms = 0.0, 0.0, 0.0, 0.0
        for step in range(net.num_steps()):
            name = net.step_name(step)
            m = re.match(r"pool(\d+)_", name)
            if m:
                li = int(m.group(1))
                c, ho, wo = shapes[li + 1]
                ms = net.time_step(step, kernel_iters, stream)
                pool_fwd_ms += ms
                pool_fwd_bytes += n * c * ho * wo * (2.0 * esize + 1)          # element in, element out, one winner code
        parts["loss_ms"] = round(net.time_backward_step(labels, 0, 2, kernel_iters, stream), 5)
        head_fused = dtype != "f32"                                      # its two layers have no steps of their own
        if head_fused:
            parts["head_loss_backward_ms"] = parts.pop("loss_ms")
        for li, l in enumerate(layers):
            if head_fused and li >= len(layers) - 2:
                continue
            c, ho, wo = shapes[li + 1]
            if l["type"] == "conv":
                ms = net.time_backward_step(labels, li, 0, kernel_iters, stream)
                parts["wgrad%d_ms" % li] = round(ms, 5)
                if f_in_of[li] == 48 and l["f_out"] == 48:
                    hi, wi = shapes[li][1:]
                    wg_ms += ms
                    wg_flops += flops[li]
                    wg_bytes += esize * n * 48.0 * (hi * wi + ho * wo)
                    wg_n += 1
                if li > 0:
                    parts["dgrad%d_ms" % li] = round(net.time_backward_step(labels, li, 1, kernel_iters, stream), 5)
            elif li > 0:
                ms = net.time_backward_step(labels, li, 1, kernel_iters, stream)
                parts["poolbwd%d_ms" % li] = round(ms, 5)
                hi, wi = shapes[li][1:]
                pool_bwd_ms += ms
                # gradient and winner code of every output in, gradient of every input out (+ its ReLU mask source in)
                pool_bwd_bytes += n * c * (ho * wo * (esize + 1.0) + hi * wi * 2.0 * esize)
        ho, wo = shapes[-1][1:]
        # labels in (count pass), logits + labels in and fp32 gradient out (2 classes); 16-bit storage: the gradient is
        # read once more and written as one 16-byte octet per pixel for the layers below
        loss_bytes = n * ho * wo * (4 + (2 * 4 + 4 + 2 * 4.0) + (0.0 if dtype == "f32" else 2 * 4 + 16))
        head_flops = None
        if head_fused:
            # one kernel: h and z recomputed, dx = W1^T dh, dW1 = dh x^T, dW2 = dz h^T (2 FLOP per multiply-add)
            f1, hid, cls = f_in_of[len(layers) - 2], layers[-2]["f_out"], layers[-1]["f_out"]
            head_flops = n * ho * wo * 2.0 * (3 * f1 * hid + 2 * hid * cls)
        res.update({
            "parts_ms": parts,
            "step_tflops": round(3.0 * sum(flops.values()) / (res["ms_per_step"] * 1e-3) / 1e12, 2),   # forward + two gradients per conv
            "wgrad": {"tflops": wg_flops / (wg_ms * 1e-3) / 1e12, "avg_ms": wg_ms / max(wg_n, 1), "alg_bytes": wg_bytes / max(wg_n, 1),
                      "alg_flops": wg_flops / max(wg_n, 1)},
            "pool_fwd_gbs": round(pool_fwd_bytes / (pool_fwd_ms * 1e-3) / 1e9, 1) if pool_fwd_ms else None,
            "pool_bwd_gbs": round(pool_bwd_bytes / (pool_bwd_ms * 1e-3) / 1e9, 1) if pool_bwd_ms else None,
            "softmax_loss_gbs": None if head_fused else round(loss_bytes / (parts["loss_ms"] * 1e-3) / 1e9, 1),
            "head_backward_tflops": round(head_flops / (parts["head_loss_backward_ms"] * 1e-3) / 1e12, 1) if head_fused else None,
        })
    net.close()
    return res


def measure_softmax_kernels(torch, B, S, dtype, n, H, W, kernel_iters=10):
    """The stand-alone softmax and softmax-loss kernels (what a layer-by-layer plan runs; the fused plans of the
    timed steps have them inside the head kernels): GB/s over their algorithmic bytes."""
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    net = B.SKNet(layers, 1, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    net.plan(n, H, W, pad=True, training=True)
    timg = torch.from_numpy(S.em_like_batch(n, H, W, 3)).cuda()
    labels = torch.from_numpy(S.binary_labels(n, H, W, 2004)).cuda()
    stream = torch.cuda.current_stream()
    net.forward(timg, None, stream)
    px, cls = n * H * W, 2
    sm_ms = None
    for step in range(net.num_steps()):
        if net.step_name(step) == "softmax":
            sm_ms = net.time_step(step, kernel_iters, stream)
    loss_ms = net.time_backward_step(labels, 0, 2, kernel_iters, stream)
    net.close()
    # softmax: logits in, probabilities out.  loss: labels (count pass), logits + labels in, fp32 gradient out,
    # and for 16-bit storage the gradient once more as one 16-byte octet per pixel
    sm_bytes = px * 2.0 * 4 * cls
    loss_bytes = px * (4 + 4 * cls + 4 + 4 * cls + (0 if dtype == "f32" else 16.0))
    return {"softmax_ms": round(sm_ms, 5) if sm_ms else None, "softmax_gbs": round(sm_bytes / (sm_ms * 1e-3) / 1e9, 1) if sm_ms else None,
            "softmax_loss_ms": round(loss_ms, 5), "softmax_loss_gbs": round(loss_bytes / (loss_ms * 1e-3) / 1e9, 1)}


def train_roofline(r, dtype, table, key):
    peak = PEAK_TFLOPS[dtype]
    w = r["wgrad"]
    traffic, src = traffic_of(table, key)
    return {"bound": "mfma", "achieved": round(w["tflops"], 2), "peak": peak, "unit": "TFLOP/s", "frac": round(w["tflops"] / peak, 4),
            "traffic": traffic, "traffic_unit": "bytes beyond L2 per launch (read + written)", "traffic_source": src,
            "algorithmic_bytes": int(w["alg_bytes"]), "algorithmic_flops": int(w["alg_flops"]), "avg_launch_ms": round(w["avg_ms"], 5),
            "kernel": "weight gradient of the 48->48 k4 SK convolutions (wgrad kernel + reduction of its private copies), average of d=2,4,8",
            "step": {"achieved": r["step_tflops"], "frac": round(r["step_tflops"] / peak, 4), "unit": "TFLOP/s",
                     "what": "3 x forward conv FLOPs (forward, data gradient, weight gradient) over the whole training step"},
            "hbm_bound_kernels": {"pool_fwd_gbs": r["pool_fwd_gbs"], "pool_bwd_gbs": r["pool_bwd_gbs"], "softmax_loss_gbs": r["softmax_loss_gbs"],
                                  "peak_gbs": HBM_PEAK_GBS, "head_and_loss_backward_tflops": r.get("head_backward_tflops"),
                                  "frac": {k: (None if r[k] is None else round(r[k] / HBM_PEAK_GBS, 4)) for k in ("pool_fwd_gbs", "pool_bwd_gbs", "softmax_loss_gbs")}}}


def measure_unet(torch, B, S, dtype, steps, warmup):
    """U-Net forward of the paper's configuration table on one 572x572 image (configs[4])."""
    params = S.unet_params(1, 2, 1005, depth=4, base=64, bias_scale=0.0)
    net = B.UNet(1, 2, depth=4, base_ch=64, dtype=dtype)
    for i, name in enumerate(S.unet_param_names(4)):
        net.set_weights(i, *params[name])
    net.plan(1, 572, 572)
    img = torch.from_numpy(S.em_like_image(572, 572, 1006)[None, None].copy()).cuda()
    prob = torch.empty((1, 2, 388, 388), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    dt, per = timed_steps(torch, lambda: net.forward(img, prob, stream), steps, warmup)
    dt /= steps
    net.close()
    gflop = 300.9            # 1-channel input; the paper's table (3 channels) sums to 301.6
    tf = gflop / dt / 1e3
    return {"ms_per_step": round(dt * 1e3, 4), "events": per, "labelled_pixels_per_s": round(388 * 388 / dt, 1), "tflops": round(tf, 1),
            "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                         "frac": round(tf / PEAK_TFLOPS[dtype], 4), "traffic": None,
                         "kernel": "whole forward pass (23 convolutions, 4 pools, 4 up-convolutions): 300.9 GFLOP over the step time"}}


def measure_usknet(torch, B, S, steps, warmup, dtype="f32"):
    """USK-Net forward of the paper's USK configuration table (3 x 692^2 -> 2 x 512^2)."""
    import numpy as np
    params = S.usknet_params(3, 2, 1006, base=64)
    net = B.USKNet(3, 2, base_ch=64, dtype=dtype)
    for i, name in enumerate(S.USKNET_PARAM_NAMES):
        net.set_weights(i, *params[name])
    net.plan(1, 692, 692)
    img = torch.from_numpy(np.stack([S.em_like_image(692, 692, 1007 + c) for c in range(3)])[None].copy()).cuda()
    prob = torch.empty((1, 2, 512, 512), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    dt, per = timed_steps(torch, lambda: net.forward(img, prob, stream), steps, warmup)
    dt /= steps
    net.close()
    # 2 f_in k^2 f_out w_out^2 over the table's convolutions and the up step
    gflop = 2e-9 * (3 * 9 * 64 * 690 ** 2 + 64 * 9 * 64 * 688 ** 2 + 64 * 36 * 128 * 339 ** 2 + 128 * 16 * 128 * (332 ** 2 + 318 ** 2)
                    + 128 * 64 * 512 * 258 ** 2 + 512 * 256 * 258 ** 2 + 256 * 128 * 516 ** 2 + 192 * 9 * 128 * 514 ** 2
                    + 128 * 9 * 64 * 512 ** 2 + 64 * 2 * 512 ** 2)
    return {"ms_per_step": round(dt * 1e3, 4), "events": per, "labelled_pixels_per_s": round(512 * 512 / dt, 1),
            "gflop": round(gflop, 1), "tflops": round(gflop / dt / 1e3, 1), "frac_of_mfma_peak": round(gflop / dt / 1e3 / PEAK_TFLOPS[dtype], 4)}


def measure_unet_train(torch, B, S, which, steps, warmup, dtype="f32"):
    """One training step (forward, masked softmax loss, backward, SGD) of the U-Net (572^2 -> 388^2) or the
    USK-Net (692^2 -> 512^2) of the paper's tables, labels masked by inverse frequency; dtype = storage type of
    activations and error maps."""
    import numpy as np
    if which == "unet":
        params, names = S.unet_params(1, 2, 1005, depth=4, base=64), S.unet_param_names(4)
        net, c_in, size, out = B.UNet(1, 2, depth=4, base_ch=64, dtype=dtype), 1, 572, 388
    else:
        params, names = S.usknet_params(3, 2, 1006, base=64), S.USKNET_PARAM_NAMES
        net, c_in, size, out = B.USKNet(3, 2, base_ch=64, dtype=dtype), 3, 692, 512
    for i, name in enumerate(names):
        net.set_weights(i, *params[name])
    net.plan(1, size, size, training=True)
    img = torch.from_numpy(np.stack([S.em_like_image(size, size, 1010 + c) for c in range(c_in)])[None].copy()).cuda()
    lab = torch.from_numpy(S.mask_labels_by_frequency(S.binary_labels(1, out, out, 1011), 2, 1012)).cuda()
    prob = torch.empty((1, 2, out, out), dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        net.forward(img, prob, stream)
        net.backward(lab, loss, stream)
        net.sgd_step(1e-3, 0.9, 0.0, stream)
    dt, per = timed_steps(torch, step, steps, warmup)
    dt /= steps
    final = float(loss.item())
    net.close()
    return {"ms_per_step": round(dt * 1e3, 3), "events": per, "labelled_pixels_per_s": round(out * out / dt, 1), "loss_after": round(final, 4)}


def measure_paper_sknet(torch, B, S, steps, warmup, dtype="f32"):
    """The paper's own SK network (Section 3.3.2: 3 x 229^2 after padding -> 2 x 128^2; its inner product
    is a k = 10, d = 8 convolution 192 -> 1024, 644 of the 695 GFLOP): the workload of the
    paper's label-throughput and layer-efficiency tables."""
    layers = S.paper_sknet_layers()
    ws, bs = S.he_normal_weights(layers, 3, 1003)
    net = B.SKNet(layers, 3, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    net.plan(1, 128, 128, pad=True)
    img = torch.from_numpy(S.uniform_image(1, 3, 128, 128, 12)).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    dt, per = timed_steps(torch, lambda: net.forward(img, prob, stream), steps, warmup)
    dt /= steps
    ip1 = [i for i in range(net.num_steps()) if net.step_name(i).startswith("conv6_k10")][0]
    ip1_ms = net.time_step(ip1, 3, stream)
    name = net.step_name(ip1)
    net.close()
    return {"ms_per_step": round(dt * 1e3, 3), "events": per, "pixels_per_s": round(128 * 128 / dt, 1),
            "forward_tflops": round(694.6 / dt / 1e3, 1), name + "_ms": round(ip1_ms, 3),
            name + "_tflops": round(644.23 / ip1_ms, 1),
            name + "_frac_of_mfma_peak": round(644.23 / ip1_ms / PEAK_TFLOPS[dtype], 4),
            "paper_pixels_per_s": {"W9100 OpenCL": 59513, "GTX 980 CUDA": 85460}}


def measure_sknet3d(torch, B, S, steps, warmup, dtype="f32"):
    """3-D SK net forward (Section 5.2.2): the Algorithm-1 conversion of an 18^3 sliding-window net
    (conv k3, pool, conv k3, pool, inner products 128 and 64; context 17) on a stack of 81 synthetic
    145 x 145 sections -> 64 x 128 x 128 labelled voxels, fp32 or 16-bit storage."""
    import numpy as np
    layers = S.sknet3d_layers(classes=2)
    ws, bs = S.he_normal_weights3d(layers, 1, 1100)
    net = B.SKNet3D(layers, 1, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    dz, h, w = 81, 145, 145
    net.plan(dz, h, w)
    shapes = net.infer_shapes(dz, h, w)
    vol = torch.from_numpy(np.ascontiguousarray(S.em_like_volume(dz, h, w, 1101).transpose(1, 0, 2, 3))).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    dt, per = timed_steps(torch, lambda: net.forward(vol, prob, stream), steps, warmup)
    dt /= steps
    net.close()
    gflop, f_in = 0.0, 1
    for lay, (c, d_, h_, w_) in zip(layers, shapes[1:]):
        if lay["type"] == "conv":
            gflop += 2e-9 * f_in * lay["k"] ** 3 * c * d_ * h_ * w_       # Section 5.5's count with k^3 taps
            f_in = c
    voxels = shapes[-1][1] * shapes[-1][2] * shapes[-1][3]
    return {"ms_per_step": round(dt * 1e3, 4), "events": per, "labelled_voxels_per_s": round(voxels / dt, 1),
            "gflop": round(gflop, 1), "tflops": round(gflop / dt / 1e3, 1)}


def measure_sknet3d_train(torch, B, S, steps, warmup, dtype="f32"):
    """One training step of the 3-D SK net of measure_sknet3d on the same volume: forward on a training plan,
    masked softmax loss, backward, SGD; dtype = storage type of activations and error maps."""
    import numpy as np
    layers = S.sknet3d_layers(classes=2)
    ws, bs = S.he_normal_weights3d(layers, 1, 1100)
    net = B.SKNet3D(layers, 1, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    dz, h, w = 81, 145, 145
    net.plan(dz, h, w, training=True)
    od, _, oh, ow = net.out_shape()
    vol = torch.from_numpy(np.ascontiguousarray(S.em_like_volume(dz, h, w, 1101).transpose(1, 0, 2, 3))).cuda()
    lab = S.binary_labels(od, oh, ow, 1102)
    labels = torch.from_numpy(S.mask_labels_by_frequency(lab, 2, 1103)).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    loss = torch.empty((), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        net.forward(vol, prob, stream)
        net.backward(labels, loss, stream)
        net.sgd_step(1e-3, 0.9, 0.0, stream)

    dt, per = timed_steps(torch, step, steps, warmup)
    dt /= steps
    final = float(loss.cpu())
    net.close()
    return {"ms_per_step": round(dt * 1e3, 3), "events": per, "labelled_voxels_per_s": round(od * oh * ow / dt, 1), "loss_after": round(final, 4)}


def measured_peaks(torch, B):
    """What this GPU sustains on a bare MFMA issue loop and on a streaming copy (not the method)."""
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)   # 1 GiB each
    dst = torch.empty_like(src)
    peaks = {"mfma_f32_tflops": round(B.sk_probe_mfma("f32", 100000), 1),
             "mfma_bf16_tflops": round(B.sk_probe_mfma("bf16", 100000), 1),
             "mfma_f16_tflops": round(B.sk_probe_mfma("f16", 100000), 1),
             # same loop, every MFMA with hashed operands of its own: the rate under the power limit
             "mfma_f32_tflops_varied_operands": round(B.sk_probe_mfma("f32", 100000, varied=True), 1),
             "mfma_bf16_tflops_varied_operands": round(B.sk_probe_mfma("bf16", 100000, varied=True), 1),
             "mfma_f16_tflops_varied_operands": round(B.sk_probe_mfma("f16", 100000, varied=True), 1),
             "copy_gbs_1gib": round(B.sk_probe_copy(src, dst, 10), 1)}
    del src, dst
    torch.cuda.empty_cache()
    return peaks


def cpu_baselines(S, r):
    """The fp64 oracle as it stands, timed on this machine's host cores on bounded samples of the benchmark workloads."""
    import numpy as np
    from oracle import layers as OL, nets as ON

    def timed(fn, budget, most):
        reps, t = 0, 0.0
        while t < budget and reps < most:
            t0 = time.perf_counter()
            fn()
            t += time.perf_counter() - t0
            reps += 1
        return reps, t

    threads = OL.num_threads()
    layers, ws, bs, img = r["layers"], r["ws"], r["bs"], r["img"]
    reps, t = timed(lambda: ON.sknet_forward(img, layers, ws, bs), 8.0, 40)
    main = {"value": round(512 * 512 * reps / t, 1), "unit": "pixels/s", "cores": threads, "kind": "oracle",
            "sample": "%d full forward pass(es) of the same 512x512 workload, fp64 C oracle, OpenMP over output rows" % reps}
    more = {}
    OL.set_num_threads(1)
    reps, t = timed(lambda: ON.sknet_forward(img, layers, ws, bs), 3.0, 1)
    more["c2_forward_single_thread"] = {"value": round(512 * 512 * reps / t, 1), "unit": "pixels/s", "cores": 1,
                                        "sample": "%d full forward pass of the 512x512 workload" % reps}
    OL.set_num_threads(threads)
    labels = S.binary_labels(1, 512, 512, 2004)
    ow, ob = [x.astype(np.float64) for x in ws], [x.astype(np.float64) for x in bs]

    def train():
        _, acts, ams = ON.sknet_forward(img, layers, ow, ob, keep=True)
        ON.sknet_backward(layers, ow, acts, ams, labels)
    reps, t = timed(train, 3.0, 1)
    more["c4_forward_backward"] = {"value": round(512 * 512 * reps / t, 1), "unit": "pixels/s", "cores": threads,
                                   "sample": "%d forward + backward pass of the 512x512 training workload (no SGD step: it is 0.1 MFLOP)" % reps}
    img3 = S.em_like_batch(1, 1024, 1024, 3)
    reps, t = timed(lambda: ON.sknet_forward(img3, layers, ws, bs), 3.0, 1)
    more["c3_forward"] = {"value": round(1024 * 1024 * reps / t, 1), "unit": "pixels/s", "cores": threads,
                          "sample": "1 of the 8 images of the 8x1024x1024 workload (the images are independent: the rate is that of all 8)"}
    params = {k: (a.astype(np.float64), b.astype(np.float64)) for k, (a, b) in S.unet_params(1, 2, 1005, depth=4, base=64).items()}
    uimg = S.em_like_image(572, 572, 1006)[None, None].astype(np.float64)
    reps, t = timed(lambda: ON.unet_forward(uimg, params, depth=4), 3.0, 1)
    more["c5_unet_forward"] = {"value": round(388 * 388 * reps / t, 1), "unit": "labelled pixels/s", "cores": threads,
                               "sample": "1 full U-Net forward pass, 572^2 -> 388^2 (300.9 GFLOP in fp64)"}
    return main, more


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", choices=["c2", "c3", "c4", "c3train", "c5", "c5bf16", "usk", "uskbf16", "papersk", "paperskbf16", "sk3d", "sk3dbf16", "sk3dtrain",
                                           "unettrain", "usktrain", "unettrainbf16", "usktrainbf16", "sk3dtrainbf16", "copy"], default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import sk_synth as S
    from paper_1509_03371_amd import binding as B

    torch.cuda.set_device(0)
    table = traffic_table()
    out = {"metric": METRIC, "unit": "pixels/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic"}

    if args.workload == "copy":
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        gbs = B.sk_probe_copy(src, dst, max(1, args.steps))
        print(json.dumps({"metric": "streaming copy", "value": round(gbs, 1), "unit": "GB/s (read + written)",
                          "bytes_read_per_launch": src.numel() * 4, "bytes_written_per_launch": src.numel() * 4,
                          "launches": max(1, args.steps) + 1, "kernel": "stream_copy_kernel"}))
        return

    if args.workload in ("c5", "c5bf16"):
        dt = "f32" if args.workload == "c5" else "bf16"
        r = measure_unet(torch, B, S, dt, args.steps, args.warmup)
        out.update({"value": r["labelled_pixels_per_s"], "ms_per_step": r["ms_per_step"], "ms_per_step_events": r["events"], "dtype": dt,
                    "config": {"workload": "U-Net forward 1x1x572x572 -> 2x388x388, %s (BASELINE configs[4])" % dt,
                               "global_batch": 1, "parallelism": "single GPU"},
                    "roofline": r["roofline"], "forward_tflops": r["tflops"]})
        print(json.dumps(out))
        return

    if args.workload in ("unettrain", "usktrain", "unettrainbf16", "usktrainbf16"):
        wdt = "bf16" if args.workload.endswith("bf16") else "f32"
        r = measure_unet_train(torch, B, S, "unet" if args.workload.startswith("unet") else "usk", args.steps, args.warmup, wdt)
        out.update({"value": r["labelled_pixels_per_s"], "ms_per_step": r["ms_per_step"], "ms_per_step_events": r["events"], "dtype": wdt,
                    "config": {"workload": ("U-Net 572^2 -> 388^2" if args.workload.startswith("unet") else "USK-Net 692^2 -> 512^2")
                                           + " training step (forward, masked softmax loss, backward, SGD), " + wdt,
                               "global_batch": 1, "parallelism": "single GPU"}, "roofline": None, "detail": r})
        print(json.dumps(out))
        return

    if args.workload in ("usk", "uskbf16", "papersk", "paperskbf16", "sk3d", "sk3dbf16", "sk3dtrain", "sk3dtrainbf16"):
        wdt = "bf16" if args.workload.endswith("bf16") else "f32"
        if args.workload in ("sk3dtrain", "sk3dtrainbf16"):
            r = measure_sknet3d_train(torch, B, S, args.steps, args.warmup, wdt)
            px, what = r["labelled_voxels_per_s"], "3-D SK net training step, 81x145x145 -> 64x128x128 labels, %s: forward, masked softmax loss, backward, SGD; value = labelled voxels per second" % wdt
        elif args.workload in ("sk3d", "sk3dbf16"):
            r = measure_sknet3d(torch, B, S, args.steps, args.warmup, wdt)
            px, what = r["labelled_voxels_per_s"], "3-D SK net forward, 81x145x145 -> 2x64x128x128 (context 17), %s; value = labelled voxels per second" % wdt
        elif args.workload in ("usk", "uskbf16"):
            r = measure_usknet(torch, B, S, args.steps, args.warmup, wdt)
            px, what = r["labelled_pixels_per_s"], "USK-Net forward 1x3x692x692 -> 2x512x512, %s (the paper's USK configuration table)" % wdt
        else:
            r = measure_paper_sknet(torch, B, S, args.steps, args.warmup, wdt)
            px, what = r["pixels_per_s"], "the paper's SK-Net forward, 3x128x128 -> 2x128x128 (padded to 229), %s" % wdt
        out.update({"value": px, "ms_per_step": r["ms_per_step"], "ms_per_step_events": r["events"], "dtype": wdt,
                    "config": {"workload": what, "global_batch": 1, "parallelism": "single GPU"}, "roofline": None, "detail": r})
        print(json.dumps(out))
        return

    r = None
    if args.workload in ("c2", "c3"):
        dtype, n, H, seed = ("f32", 1, 512, 2) if args.workload == "c2" else ("bf16", 8, 1024, 3)
        r = measure_forward(torch, B, S, dtype, n, H, H, args.steps, args.warmup, seed)
        out.update({
            "value": round(r["pixels_per_s"], 1), "ms_per_step": round(r["ms_per_step"], 4), "ms_per_step_events": r["events"], "dtype": dtype,
            "config": {"workload": "SK-Net forward, %dx1x%dx%d %s image(s), %s (BASELINE configs[%d])"
                                   % (n, H, H, "fp32" if dtype == "f32" else dtype, NET_DESC, 1 if args.workload == "c2" else 2),
                       "global_batch": n, "parallelism": "single GPU"},
            "roofline": forward_roofline(r, dtype, table, args.workload + "_conv"),
            "forward_tflops": round(r["forward_tflops"], 2),
            "pool_gbs": None if r["pool_gbs"] is None else round(r["pool_gbs"], 1),
            "pool_frac_of_hbm_peak": None if r["pool_gbs"] is None else round(r["pool_gbs"] / HBM_PEAK_GBS, 4),
            "step_ms": r["step_ms"],
            "measured_peaks": measured_peaks(torch, B),
        })
    else:
        n, H = (1, 512) if args.workload == "c4" else (8, 1024)
        rt = measure_train(torch, B, S, "bf16", n, H, H, args.steps, args.warmup, 2 if n == 1 else 3)
        out.update({
            "value": round(rt["pixels_per_s"], 1), "ms_per_step": round(rt["ms_per_step"], 4), "ms_per_step_events": rt["events"], "dtype": "bf16",
            "config": {"workload": "SK-Net training step, %dx1x%dx%d bf16: forward, softmax loss, backward, SGD (head and loss one kernel per direction); " % (n, H, H)
                                   + NET_DESC + (" (BASELINE configs[3])" if n == 1 else " (configs[3]'s step on configs[2]'s batch)"),
                       "global_batch": n, "parallelism": "single GPU"},
            "roofline": train_roofline(rt, "bf16", table, args.workload + "_wgrad"), "parts_ms": rt["parts_ms"],
        })
        sm = measure_softmax_kernels(torch, B, S, "bf16", n, H, H)
        hb = out["roofline"]["hbm_bound_kernels"]
        hb.update({"softmax_gbs": sm["softmax_gbs"], "softmax_loss_gbs": sm["softmax_loss_gbs"], "softmax_ms": sm["softmax_ms"],
                   "softmax_loss_ms": sm["softmax_loss_ms"],
                   "softmax_note": "stand-alone kernels of a layer-by-layer plan (mode 1) on the same images; the timed step has them inside the head kernels"})
        hb["frac"].update({"softmax_gbs": round(sm["softmax_gbs"] / HBM_PEAK_GBS, 4) if sm["softmax_gbs"] else None,
                           "softmax_loss_gbs": round(sm["softmax_loss_gbs"] / HBM_PEAK_GBS, 4)})

    if args.workload == "c2" and not args.no_extras:
        extras = {}
        r3 = measure_forward(torch, B, S, "bf16", 8, 1024, 1024, 10, 3, 3, kernel_iters=5)
        extras["c3_bf16_forward_8x1024"] = {
            "pixels_per_s": round(r3["pixels_per_s"], 1), "ms_per_step": round(r3["ms_per_step"], 4), "ms_per_step_events": r3["events"],
            "roofline": forward_roofline(r3, "bf16", table, "c3_conv"),
            "forward_tflops": round(r3["forward_tflops"], 1),
            "pool_gbs": None if r3["pool_gbs"] is None else round(r3["pool_gbs"], 1), "step_ms": r3["step_ms"]}
        rt = measure_train(torch, B, S, "bf16", 1, 512, 512, 20, 3, 2)
        extras["c4_bf16_train_512"] = {"pixels_per_s": round(rt["pixels_per_s"], 1), "ms_per_step": round(rt["ms_per_step"], 4),
                                       "ms_per_step_events": rt["events"], "roofline": train_roofline(rt, "bf16", table, "c4_wgrad"),
                                       "parts_ms": rt["parts_ms"]}
        rt = measure_train(torch, B, S, "f32", 1, 512, 512, 10, 3, 2, detail=False)
        extras["c4_as_f32_train_512"] = {"pixels_per_s": round(rt["pixels_per_s"], 1), "ms_per_step": round(rt["ms_per_step"], 4)}
        rt = measure_train(torch, B, S, "bf16", 8, 1024, 1024, 5, 2, 3, kernel_iters=3)
        extras["c3train_bf16_train_8x1024"] = {"pixels_per_s": round(rt["pixels_per_s"], 1), "ms_per_step": round(rt["ms_per_step"], 4),
                                               "ms_per_step_events": rt["events"], "roofline": train_roofline(rt, "bf16", table, "c3train_wgrad"),
                                               "parts_ms": rt["parts_ms"]}
        for name, dt in (("c5_unet_572_f32", "f32"), ("c5_unet_572_bf16", "bf16")):
            extras[name] = measure_unet(torch, B, S, dt, 10, 3)
        extras["paper_sknet_128_f32"] = measure_paper_sknet(torch, B, S, 5, 2)
        extras["paper_sknet_128_bf16"] = measure_paper_sknet(torch, B, S, 5, 2, "bf16")
        extras["usknet_692_f32_forward"] = measure_usknet(torch, B, S, 5, 2)
        extras["usknet_692_bf16_forward"] = measure_usknet(torch, B, S, 5, 2, "bf16")
        extras["sknet3d_81x145x145_f32_forward"] = measure_sknet3d(torch, B, S, 5, 2)
        extras["sknet3d_81x145x145_bf16_forward"] = measure_sknet3d(torch, B, S, 5, 2, "bf16")
        extras["sknet3d_81x145x145_f32_train_step"] = measure_sknet3d_train(torch, B, S, 3, 1)
        extras["sknet3d_81x145x145_bf16_train_step"] = measure_sknet3d_train(torch, B, S, 3, 1, "bf16")
        extras["unet_572_f32_train_step"] = measure_unet_train(torch, B, S, "unet", 3, 1)
        extras["usknet_692_f32_train_step"] = measure_unet_train(torch, B, S, "usk", 3, 1)
        extras["unet_572_bf16_train_step"] = measure_unet_train(torch, B, S, "unet", 3, 1, "bf16")
        extras["usknet_692_bf16_train_step"] = measure_unet_train(torch, B, S, "usk", 3, 1, "bf16")
        out["extras"] = extras

    if args.workload == "c2" and not args.no_cpu_baseline:
        out["cpu_baseline"], out["cpu_baseline_more"] = cpu_baselines(S, r)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
