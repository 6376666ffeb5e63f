"""Benchmark of the SK-Net hot path on one MI355X.  Prints ONE JSON line.

Default workload (BASELINE configs[1], the one the headline metric is quoted on): SK-Net forward on
one 1x1x512x512 fp32 image -- mirror padding, four stages of [conv k4 -> 48 maps + ReLU, max pool
k2 s1] at kernel strides 1/2/4/8, 1x1 conv 48 -> 200 + ReLU, 1x1 conv 200 -> 2, per-pixel softmax.
A step is one such pass over one synthetic image that is resident in HBM before the timed region.

--workload c3 : the same net in bf16 (fp32 accumulate) on 8 images of 1024x1024 (configs[2])
--workload c4 : one bf16 training step at 512x512 (configs[3]): forward, softmax loss, backward, SGD
--workload c5 / c5bf16 : U-Net forward on one 572x572 image (configs[4]) in fp32 / bf16
--workload sk3d / sk3dtrain : 3-D SK net on a stack of 81 sections of 145x145 (Section 5.2.2), fp32: forward / training step
--workload copy : only the streaming-copy probe on 2 x 1 GiB (the known-size kernel that the HBM
                  byte counters of a profiler run are calibrated against)
The default run also appends short c3 / c4 measurements under "extras" (skip with --no-extras).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0}   # MI355X dense MFMA peaks
HBM_PEAK_GBS = 8000.0
METRIC = "labelled pixels/sec SK-Net fwd (and fwd+bwd) 1 GPU; conv % MFMA peak"
# Bytes moved beyond L2 per launch of the dominant kernel (average of its three launches per pass),
# from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by what the same counters
# read for stream_copy_kernel on 1 GiB (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0); the runs and their
# figures are in profiles/sknet_c{2,3}_forward_hbm_traffic_pmc.txt and
# profiles/stream_copy_1gib_pmc_calibration.txt.  KiB: (fetch x 2, write).
TRAFFIC_KIB = {"c2": (2.0 * (35765.2 + 34265.0 + 30821.7) / 3, (78827.5 + 71135.3 + 58340.2) / 3),
               "c3": (2.0 * (479830.4 + 473130.7 + 454601.8) / 3, (870701.7 + 846215.4 + 798768.0) / 3)}


def build_net(B, S, dtype, n, H, W, training):
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    net = B.SKNet(layers, 1, 2, dtype=dtype)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    net.plan(n, H, W, pad=True, training=training)
    return net, layers, ws, bs


def images(S, n, H, W, first_seed):
    return S.em_like_batch(n, H, W, first_seed)


def measure_forward(torch, B, S, dtype, n, H, W, steps, warmup, first_seed, kernel_iters=20):
    net, layers, ws, bs = build_net(B, S, dtype, n, H, W, False)
    img = images(S, n, H, W, first_seed)
    timg = torch.from_numpy(img).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        net.forward(timg, prob, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.forward(timg, prob, stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3

    # per-kernel durations: HIP events recorded on the same stream, inside the library
    shapes = net.infer_shapes(H, W)
    esize = 4 if dtype == "f32" else 2
    step_ms, conv_flops, conv_ms, total_flops = {}, 0.0, 0.0, 0.0
    conv_bytes, conv_launches = 0.0, 0
    pool_bytes, pool_ms = 0.0, 0.0
    f_in_of = {}
    f_in = 1
    for li, l in enumerate(layers):
        f_in_of[li] = f_in
        if l["type"] == "conv":
            f_in = l["f_out"]
    import re
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
            fl = 2.0 * f_in_of[li] * l["k"] ** 2 * l["f_out"] * ho * wo * n
            total_flops += fl
            if f_in_of[li] == 48 and l["f_out"] == 48:      # the dominant kernel: 48 -> 48, k4, dilated
                conv_flops += fl
                conv_ms += ms
                hi, wi = shapes[li][1:]
                conv_bytes += esize * n * 48.0 * (hi * wi + ho * wo)   # every input and output element once
                conv_launches += 1
        else:                                         # pool as a layer of its own: one element read + one written
            pool_bytes += 2.0 * esize * n * c * ho * wo
            pool_ms += ms
    for li, l in enumerate(layers):                   # the 1x1 convolutions of a fused head
        if l["type"] == "conv" and not any(k.startswith("conv%d_" % li) for k in step_ms):
            c, ho, wo = shapes[li + 1]
            total_flops += 2.0 * f_in_of[li] * l["k"] ** 2 * l["f_out"] * ho * wo * n
    res = {
        "ms_per_step": ms_per_step, "pixels_per_s": n * H * W * steps / dt, "step_ms": step_ms,
        "conv_tflops": conv_flops / (conv_ms * 1e-3) / 1e12, "forward_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "pool_gbs": (pool_bytes / (pool_ms * 1e-3) / 1e9) if pool_ms > 0 else None, "conv_alg_bytes": conv_bytes / max(conv_launches, 1), "layers": layers, "ws": ws, "bs": bs, "img": img,
    }
    net.close()
    return res


def measure_train(torch, B, S, dtype, n, H, W, steps, warmup, first_seed):
    net, layers, ws, bs = build_net(B, S, dtype, n, H, W, True)
    timg = torch.from_numpy(images(S, n, H, W, first_seed)).cuda()
    labels = torch.from_numpy(S.binary_labels(n, H, W, 2004)).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def one():
        net.forward(timg, prob, stream)
        net.backward(labels, loss, stream)
        net.sgd_step(0.01, stream=stream)

    for _ in range(warmup):
        one()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    net.close()
    return {"pixels_per_s": n * H * W * steps / dt, "ms_per_step": dt / steps * 1e3, "steps": steps}


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
    for _ in range(warmup):
        net.forward(img, prob, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.forward(img, prob, stream)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    net.close()
    gflop = 300.9            # 1-channel input; the paper's table (3 channels) sums to 301.6
    return {"ms_per_step": round(dt * 1e3, 4), "labelled_pixels_per_s": round(388 * 388 / dt, 1),
            "tflops": round(gflop / dt / 1e3, 1)}


def measure_usknet(torch, B, S, steps, warmup, dtype="f32"):
    """USK-Net forward of the paper's USK configuration table (3 x 692^2 -> 2 x 512^2)."""
    params = S.usknet_params(3, 2, 1006, base=64)
    net = B.USKNet(3, 2, base_ch=64, dtype=dtype)
    for i, name in enumerate(S.USKNET_PARAM_NAMES):
        net.set_weights(i, *params[name])
    net.plan(1, 692, 692)
    import numpy as np
    img = torch.from_numpy(np.stack([S.em_like_image(692, 692, 1007 + c) for c in range(3)])[None].copy()).cuda()
    prob = torch.empty((1, 2, 512, 512), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        net.forward(img, prob, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.forward(img, prob, stream)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    net.close()
    # 2 f_in k^2 f_out w_out^2 over the table's convolutions and the up step
    gflop = 2e-9 * (3 * 9 * 64 * 690 ** 2 + 64 * 9 * 64 * 688 ** 2 + 64 * 36 * 128 * 339 ** 2 + 128 * 16 * 128 * (332 ** 2 + 318 ** 2)
                    + 128 * 64 * 512 * 258 ** 2 + 512 * 256 * 258 ** 2 + 256 * 128 * 516 ** 2 + 192 * 9 * 128 * 514 ** 2
                    + 128 * 9 * 64 * 512 ** 2 + 64 * 2 * 512 ** 2)
    return {"ms_per_step": round(dt * 1e3, 4), "labelled_pixels_per_s": round(512 * 512 / dt, 1),
            "gflop": round(gflop, 1), "tflops": round(gflop / dt / 1e3, 1)}


def measure_unet_train(torch, B, S, which, steps, warmup):
    """One training step (forward, masked softmax loss, backward, SGD) of the U-Net (572^2 -> 388^2) or the
    USK-Net (692^2 -> 512^2) of the paper's tables, fp32, labels masked by inverse frequency."""
    import numpy as np
    if which == "unet":
        params, names = S.unet_params(1, 2, 1005, depth=4, base=64), S.unet_param_names(4)
        net, c_in, size, out = B.UNet(1, 2, depth=4, base_ch=64), 1, 572, 388
    else:
        params, names = S.usknet_params(3, 2, 1006, base=64), S.USKNET_PARAM_NAMES
        net, c_in, size, out = B.USKNet(3, 2, base_ch=64), 3, 692, 512
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
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    final = float(loss.item())
    net.close()
    return {"ms_per_step": round(dt * 1e3, 3), "labelled_pixels_per_s": round(out * out / dt, 1), "loss_after": round(final, 4)}


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
    for _ in range(warmup):
        net.forward(img, prob, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.forward(img, prob, stream)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    ip1_ms = net.time_step(7, 3, stream)               # pad, 6 layers, then the k10 d8 convolution
    name = net.step_name(7)
    net.close()
    return {"ms_per_step": round(dt * 1e3, 3), "pixels_per_s": round(128 * 128 / dt, 1),
            "forward_tflops": round(694.6 / dt / 1e3, 1), name + "_ms": round(ip1_ms, 3),
            name + "_tflops": round(644.23 / ip1_ms, 1),
            name + "_frac_of_mfma_peak": round(644.23 / ip1_ms / PEAK_TFLOPS[dtype], 4),
            "paper_pixels_per_s": {"W9100 OpenCL": 59513, "GTX 980 CUDA": 85460}}


def measure_sknet3d(torch, B, S, steps, warmup):
    """3-D SK net forward (Section 5.2.2): the Algorithm-1 conversion of an 18^3 sliding-window net
    (conv k3, pool, conv k3, pool, inner products 128 and 64; context 17) on a stack of 81 synthetic
    145 x 145 sections -> 64 x 128 x 128 labelled voxels, fp32."""
    import numpy as np
    layers = S.sknet3d_layers(classes=2)
    ws, bs = S.he_normal_weights3d(layers, 1, 1100)
    net = B.SKNet3D(layers, 1, 2)
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    dz, h, w = 81, 145, 145
    net.plan(dz, h, w)
    shapes = net.infer_shapes(dz, h, w)
    vol = torch.from_numpy(np.ascontiguousarray(S.em_like_volume(dz, h, w, 1101).transpose(1, 0, 2, 3))).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        net.forward(vol, prob, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.forward(vol, prob, stream)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    net.close()
    gflop, f_in = 0.0, 1
    for lay, (c, d_, h_, w_) in zip(layers, shapes[1:]):
        if lay["type"] == "conv":
            gflop += 2e-9 * f_in * lay["k"] ** 3 * c * d_ * h_ * w_       # Section 5.5's count with k^3 taps
            f_in = c
    voxels = shapes[-1][1] * shapes[-1][2] * shapes[-1][3]
    return {"ms_per_step": round(dt * 1e3, 4), "labelled_voxels_per_s": round(voxels / dt, 1),
            "gflop": round(gflop, 1), "tflops": round(gflop / dt / 1e3, 1)}


def measure_sknet3d_train(torch, B, S, steps, warmup):
    """One training step of the 3-D SK net of measure_sknet3d on the same volume: forward on a training plan,
    masked softmax loss, backward, SGD."""
    import numpy as np
    layers = S.sknet3d_layers(classes=2)
    ws, bs = S.he_normal_weights3d(layers, 1, 1100)
    net = B.SKNet3D(layers, 1, 2)
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

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    final = float(loss.cpu())
    net.close()
    return {"ms_per_step": round(dt * 1e3, 3), "labelled_voxels_per_s": round(od * oh * ow / dt, 1), "loss_after": round(final, 4)}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", choices=["c2", "c3", "c4", "c5", "c5bf16", "usk", "uskbf16", "papersk", "paperskbf16", "sk3d", "sk3dtrain", "unettrain", "usktrain",
                                           "copy"], default="c2")
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
    net_desc = "4x[conv k4 48 + ReLU, pool k2] d=1/2/4/8, 1x1 48->200 + ReLU, 1x1 200->2, softmax"
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
        out.update({"value": r["labelled_pixels_per_s"], "ms_per_step": r["ms_per_step"], "dtype": dt,
                    "config": {"workload": "U-Net forward 1x1x572x572 -> 2x388x388, %s (BASELINE configs[4])" % dt,
                               "global_batch": 1, "parallelism": "single GPU"},
                    "roofline": None, "forward_tflops": r["tflops"]})
        print(json.dumps(out))
        return

    if args.workload in ("unettrain", "usktrain"):
        r = measure_unet_train(torch, B, S, "unet" if args.workload == "unettrain" else "usk", args.steps, args.warmup)
        out.update({"value": r["labelled_pixels_per_s"], "ms_per_step": r["ms_per_step"], "dtype": "f32",
                    "config": {"workload": ("U-Net 572^2 -> 388^2" if args.workload == "unettrain" else "USK-Net 692^2 -> 512^2")
                                           + " training step (forward, masked softmax loss, backward, SGD), fp32",
                               "global_batch": 1, "parallelism": "single GPU"}, "roofline": None, "detail": r})
        print(json.dumps(out))
        return

    if args.workload in ("usk", "uskbf16", "papersk", "paperskbf16", "sk3d", "sk3dtrain"):
        wdt = "bf16" if args.workload.endswith("bf16") else "f32"
        if args.workload == "sk3dtrain":
            r = measure_sknet3d_train(torch, B, S, args.steps, args.warmup)
            px, what = r["labelled_voxels_per_s"], "3-D SK net training step, 81x145x145 -> 64x128x128 labels, fp32: forward, masked softmax loss, backward, SGD; value = labelled voxels per second"
        elif args.workload == "sk3d":
            r = measure_sknet3d(torch, B, S, args.steps, args.warmup)
            px, what = r["labelled_voxels_per_s"], "3-D SK net forward, 81x145x145 -> 2x64x128x128 (context 17), fp32; value = labelled voxels per second"
        elif args.workload in ("usk", "uskbf16"):
            r = measure_usknet(torch, B, S, args.steps, args.warmup, wdt)
            px, what = r["labelled_pixels_per_s"], "USK-Net forward 1x3x692x692 -> 2x512x512, %s (the paper's USK configuration table)" % wdt
        else:
            r = measure_paper_sknet(torch, B, S, args.steps, args.warmup, wdt)
            px, what = r["pixels_per_s"], "the paper's SK-Net forward, 3x128x128 -> 2x128x128 (padded to 229), %s" % wdt
        out.update({"value": px, "ms_per_step": r["ms_per_step"], "dtype": wdt,
                    "config": {"workload": what, "global_batch": 1, "parallelism": "single GPU"}, "roofline": None, "detail": r})
        print(json.dumps(out))
        return

    if args.workload in ("c2", "c3"):
        dtype, n, H, seed = ("f32", 1, 512, 2) if args.workload == "c2" else ("bf16", 8, 1024, 3)
        r = measure_forward(torch, B, S, dtype, n, H, H, args.steps, args.warmup, seed)
        peak = PEAK_TFLOPS[dtype]
        out.update({
            "value": round(r["pixels_per_s"], 1), "ms_per_step": round(r["ms_per_step"], 4), "dtype": dtype,
            "config": {"workload": "SK-Net forward, %dx1x%dx%d %s image(s), %s (BASELINE configs[%d])"
                                   % (n, H, H, "fp32" if dtype == "f32" else dtype, net_desc, 1 if args.workload == "c2" else 2),
                       "global_batch": n, "parallelism": "single GPU"},
            "roofline": {"bound": "mfma", "achieved": round(r["conv_tflops"], 2), "peak": peak, "unit": "TFLOP/s",
                         "frac": round(r["conv_tflops"] / peak, 4),
                         "traffic": int(sum(TRAFFIC_KIB[args.workload]) * 1024),
                         "traffic_unit": "bytes beyond L2 per launch (read + written), from profiles/",
                         "algorithmic_bytes": int(r["conv_alg_bytes"]),
                         "kernel": "48->48 k4 SK convolutions at d=2,4,8 (%s)"
                                   % ("conv_f32_pf_kernel<3,1,4,4,2,false,4>" if dtype == "f32" else "conv_h_ring_kernel<bf16,4,3,MAP4,8,false,3,true,4>")},
            "forward_tflops": round(r["forward_tflops"], 2),
            "pool_gbs": None if r["pool_gbs"] is None else round(r["pool_gbs"], 1),
            "pool_frac_of_hbm_peak": None if r["pool_gbs"] is None else round(r["pool_gbs"] / HBM_PEAK_GBS, 4),
            "step_ms": r["step_ms"],
            "measured_peaks": measured_peaks(torch, B),
        })
    else:
        r = measure_train(torch, B, S, "bf16", 1, 512, 512, args.steps, args.warmup, 2)
        out.update({
            "value": round(r["pixels_per_s"], 1), "ms_per_step": round(r["ms_per_step"], 4), "dtype": "bf16",
            "config": {"workload": "SK-Net training step, 1x1x512x512 bf16: forward, softmax loss, backward, SGD; "
                                   + net_desc + " (BASELINE configs[3])", "global_batch": 1, "parallelism": "single GPU"},
            "roofline": None,
        })

    if args.workload == "c2" and not args.no_extras:
        extras = {}
        r3 = measure_forward(torch, B, S, "bf16", 8, 1024, 1024, 10, 3, 3, kernel_iters=5)
        extras["c3_bf16_forward_8x1024"] = {
            "pixels_per_s": round(r3["pixels_per_s"], 1), "ms_per_step": round(r3["ms_per_step"], 4),
            "conv_tflops": round(r3["conv_tflops"], 1), "conv_frac_of_bf16_mfma_peak": round(r3["conv_tflops"] / 2500.0, 4),
            "pool_gbs": None if r3["pool_gbs"] is None else round(r3["pool_gbs"], 1),
            "pool_frac_of_hbm_peak": None if r3["pool_gbs"] is None else round(r3["pool_gbs"] / HBM_PEAK_GBS, 4),
            "step_ms": r3["step_ms"]}
        for name, dt in (("c4_bf16_train_512", "bf16"), ("c4_as_f32_train_512", "f32")):
            rt = measure_train(torch, B, S, dt, 1, 512, 512, 20, 3, 2)
            extras[name] = {"pixels_per_s": round(rt["pixels_per_s"], 1), "ms_per_step": round(rt["ms_per_step"], 4)}
        for name, dt in (("c5_unet_572_f32", "f32"), ("c5_unet_572_bf16", "bf16")):
            extras[name] = measure_unet(torch, B, S, dt, 10, 3)
        extras["paper_sknet_128_f32"] = measure_paper_sknet(torch, B, S, 5, 2)
        extras["paper_sknet_128_bf16"] = measure_paper_sknet(torch, B, S, 5, 2, "bf16")
        extras["usknet_692_f32_forward"] = measure_usknet(torch, B, S, 5, 2)
        extras["usknet_692_bf16_forward"] = measure_usknet(torch, B, S, 5, 2, "bf16")
        extras["sknet3d_81x145x145_f32_forward"] = measure_sknet3d(torch, B, S, 5, 2)
        extras["sknet3d_81x145x145_f32_train_step"] = measure_sknet3d_train(torch, B, S, 3, 1)
        extras["unet_572_f32_train_step"] = measure_unet_train(torch, B, S, "unet", 3, 1)
        extras["usknet_692_f32_train_step"] = measure_unet_train(torch, B, S, "usk", 3, 1)
        out["extras"] = extras

    if args.workload == "c2" and not args.no_cpu_baseline:
        from oracle import nets as ON
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 40:
            t0 = time.perf_counter()
            ON.sknet_forward(r["img"], r["layers"], r["ws"], r["bs"])
            t_cpu += time.perf_counter() - t0
            reps += 1
        out["cpu_baseline"] = {"value": round(512 * 512 * reps / t_cpu, 1), "unit": "pixels/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "kind": "oracle",
                               "sample": "%d full forward pass(es) of the same 512x512 workload, fp64 C oracle with OpenMP" % reps}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
