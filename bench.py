"""Benchmark of the SK-Net hot path on one MI355X.

Workload (BASELINE config 2): SK-Net forward on one 1x1x512x512 fp32 image -- mirror padding,
four stages of [conv k4 -> 48 maps + ReLU, max pool k2 s1] at kernel strides 1/2/4/8, 1x1 conv
48 -> 200 + ReLU, 1x1 conv 200 -> 2, per-pixel softmax.  A step is one such pass; the image is
resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_FP32_PEAK_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
HBM_PEAK_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--size", type=int, default=512, help="image side (512 = BASELINE config 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-train", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import sk_synth as S
    from paper_1509_03371_amd import binding as B

    torch.cuda.set_device(0)
    H = W = args.size
    layers = S.sknet_layers()
    ws, bs = S.he_normal_weights(layers, 1, 1001)
    img = S.em_like_batch(1, H, W, 2)
    net = B.SKNet(layers, 1, 2, dtype="f32")
    for i, (w, b) in enumerate(zip(ws, bs)):
        net.set_weights(i, w, b)
    net.plan(1, H, W, pad=True, training=False)
    timg = torch.from_numpy(img).cuda()
    prob = torch.empty(net.out_shape(), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        net.forward(timg, prob, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        net.forward(timg, prob, stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    px_per_s = H * W * args.steps / dt

    # per-kernel durations, HIP events on the same stream (inside the library)
    shapes = net.infer_shapes(H, W)
    step_ms, conv_flops, conv_ms = {}, 0.0, 0.0
    total_flops = 0.0
    f_in = 1
    for step in range(net.num_steps()):
        ms = net.time_step(step, 20, stream)
        name = net.step_name(step)
        step_ms[name] = round(ms, 5)
        if 1 <= step <= len(layers) and layers[step - 1]["type"] == "conv":
            l = layers[step - 1]
            c, ho, wo = shapes[step]
            fl = 2.0 * f_in * l["k"] ** 2 * l["f_out"] * ho * wo
            total_flops += fl
            if f_in == 48 and l["f_out"] == 48:      # the dominant kernel: 48 -> 48, k4, dilated
                conv_flops += fl
                conv_ms += ms
            f_in = l["f_out"]
    achieved = conv_flops / (conv_ms * 1e-3) / 1e12

    out = {
        "metric": "labelled pixels/sec SK-Net fwd (and fwd+bwd) 1 GPU; conv % MFMA peak",
        "value": round(px_per_s, 1), "unit": "pixels/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "SK-Net forward, 1x1x%dx%d fp32 image, 4x[conv k4 48 + ReLU, pool k2] d=1/2/4/8, "
                               "1x1 48->200 + ReLU, 1x1 200->2, softmax (BASELINE configs[1])" % (H, W),
                   "global_batch": 1, "parallelism": "single GPU"},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_FP32_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / MFMA_FP32_PEAK_TFLOPS, 4), "traffic": None,
                     "kernel": "conv_f32_kernel<3,2> (48->48 k4 convs at d=2,4,8)"},
        "forward_tflops": round(total_flops / (ms_per_step * 1e-3) / 1e12, 2),
        "step_ms": step_ms,
    }

    if not args.no_train:
        tnet = B.SKNet(layers, 1, 2, dtype="f32")
        for i, (w, b) in enumerate(zip(ws, bs)):
            tnet.set_weights(i, w, b)
        tnet.plan(1, H, W, pad=True, training=True)
        labels = torch.from_numpy(S.binary_labels(1, H, W, 2004)).cuda()
        loss = torch.empty(1, dtype=torch.float32, device="cuda")
        tsteps = max(1, args.steps // 2)
        for _ in range(max(1, args.warmup // 2)):
            tnet.forward(timg, prob, stream); tnet.backward(labels, loss, stream); tnet.sgd_step(0.0, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(tsteps):
            tnet.forward(timg, prob, stream)
            tnet.backward(labels, loss, stream)
            tnet.sgd_step(0.0, stream=stream)      # lr 0 keeps the weights (and the timings) stationary
        torch.cuda.synchronize()
        tdt = time.perf_counter() - t0
        out["train"] = {"workload": "forward + softmax loss + backward + SGD, same net and image, fp32",
                        "pixels_per_s": round(H * W * tsteps / tdt, 1), "ms_per_step": round(tdt / tsteps * 1e3, 4),
                        "steps": tsteps}
        tnet.close()

    if not args.no_cpu_baseline:
        from oracle import nets as ON
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 4:
            t0 = time.perf_counter()
            ON.sknet_forward(img, layers, ws, bs)
            t_cpu += time.perf_counter() - t0
            reps += 1
        out["cpu_baseline"] = {"value": round(H * W * reps / t_cpu, 1), "unit": "pixels/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "kind": "oracle",
                               "sample": "%d full forward pass(es) of the same %dx%d workload, fp64 C oracle with OpenMP" % (reps, H, W)}
    net.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
