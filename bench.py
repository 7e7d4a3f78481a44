#!/usr/bin/env python3
"""Throughput of the whole-image MPCNN training pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--no-cpu-baseline]

One step = one pass of the whole hot path (forward + backward of every layer, all
kernels of the C ABI call mpcnn_seg_backward; plus mpcnn_sgd_step for the workload
that trains) over one batch of seeded synthetic images already resident in HBM.
Prints ONE JSON line: training pixels/s (valid output pixels = patches per second),
the roofline figures of the dominant kernel (timed live with HIP events recorded on
the launch stream by the library's profile hooks), and the fp64 patch-by-patch oracle
timed on the host cores of this machine on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"mfma": (157.3, "TFLOP/s"), "hbm": (8000.0, "GB/s")}   # MI355X: fp32 MFMA, HBM3E


def read_traffic(path, kernel):
    """HBM bytes per launch of `kernel` as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (two runs, scaled by a copy of known size); None if no such measurement is committed."""
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 2 and f[0] == kernel:
                return float(f[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="workload index (default: the metric's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernels", action="store_true", help="also print the per-kernel table to stderr")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of known size (to scale rocprofv3's FETCH_SIZE / "
                         "WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not "
              "supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_1302_1690_amd import mpcnn, workloads as wl

    if args.copy_calibration:
        n = 256 * 1024 * 1024 // 4                    # 256 MiB read + 256 MiB written per copy
        src = torch.rand(n, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 4 * n, "copy_bytes_written": 4 * n, "copies": 5}))
        return 0

    cfg = wl.CONFIGS[args.config]
    img, lab = wl.make_inputs(cfg)
    params = wl.make_params(cfg)
    net = mpcnn.Net(cfg.layers, cfg.in_channels, cfg.patch,
                    dtype=mpcnn.BF16 if cfg.dtype == "bf16" else mpcnn.F32)
    net.set_params(params)
    d_img = torch.from_numpy(img).cuda()
    d_lab = torch.from_numpy(lab).cuda()
    probs = torch.empty((cfg.batch, cfg.n_classes, cfg.out_h, cfg.out_w), dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    ws = net.alloc_workspace(cfg.batch, cfg.height, cfg.width, True)
    do_sgd = cfg.sgd_steps > 0
    grad_scale = 1.0 / cfg.valid_pixels          # lr applies to the mean per-pixel loss

    def step():
        net.seg_backward(d_img, d_lab, None, probs, loss, ws=ws)
        if do_sgd:
            net.sgd_step(cfg.lr, grad_scale)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    value = cfg.valid_pixels * args.steps / dt
    final_loss = float(loss.item())

    # ---- per-kernel durations: same steps again with HIP events around every launch
    if do_sgd:
        net.set_params(params)
    net.profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    stats = net.profile_read()
    net.profile_enable(False)
    by_name = {}
    for s in stats:
        if s["launches"] == 0:
            continue
        k = by_name.setdefault(s["name"], dict(ms=0.0, launches=0, flops=0.0, bytes=0.0, steps=set()))
        k["ms"] += s["ms_total"]
        k["launches"] += s["launches"]
        k["flops"] += s["flops"] * s["launches"]
        k["bytes"] += s["bytes"] * s["launches"]
        k["steps"].add(s["step"])
    dom_name = max(by_name, key=lambda n: by_name[n]["ms"])
    dom = by_name[dom_name]
    bound = "mfma" if "mfma" in dom_name else "hbm"
    peak, unit = PEAK[bound]
    if bound == "mfma" and cfg.dtype == "bf16":
        peak = 2500.0   # bf16 storage multiplies on the bf16 matrix instruction (fp32 accumulation)
    work = dom["flops"] if bound == "mfma" else dom["bytes"]
    achieved = work / (dom["ms"] * 1e-3) / (1e12 if bound == "mfma" else 1e9)
    traffic = read_traffic(os.path.join(ROOT, "profiles", "traffic_%s.txt" % cfg.name), dom_name)
    roofline = {"bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic, "kernel": dom_name,
                "avg_launch_us": round(1e3 * dom["ms"] / dom["launches"], 2),
                "launches_per_step": dom["launches"] // args.steps,
                "share_of_step": round(dom["ms"] / args.steps / ms_per_step, 3)}
    if args.kernels:
        tot = sum(v["ms"] for v in by_name.values())
        for n, v in sorted(by_name.items(), key=lambda kv: -kv[1]["ms"]):
            tf = v["flops"] / (v["ms"] * 1e-3) / 1e12 if v["ms"] > 0 else 0
            gb = v["bytes"] / (v["ms"] * 1e-3) / 1e9 if v["ms"] > 0 else 0
            print("%-20s %3d launches/step %8.1f us/step %5.1f%%  %7.2f TFLOP/s %8.1f GB/s" % (
                n, v["launches"] // args.steps, 1e3 * v["ms"] / args.steps, 100 * v["ms"] / tot, tf, gb),
                file=sys.stderr)
        for s in sorted(stats, key=lambda s: -s["ms_total"]):
            if s["launches"]:
                us = 1e3 * s["ms_total"] / s["launches"]
                print("  %-20s layer %2d  %8.1f us  %7.2f TFLOP/s %8.1f GB/s" % (
                    s["name"], s["layer"], us, s["flops"] / us / 1e6, s["bytes"] / us / 1e3), file=sys.stderr)

    # ---- deployment forward of the same images (mirrored borders, output as large as the image;
    # outside the timed training steps): seconds per image, the unit the paper quotes for it
    net.seg_forward_same(d_img)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_fwd = max(5, args.steps // 2)
    for _ in range(n_fwd):
        net.seg_forward_same(d_img)
    torch.cuda.synchronize()
    fwd_ms_per_image = 1e3 * (time.perf_counter() - t0) / (n_fwd * cfg.batch)

    # ---- the oracle on the host cores, bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_sample = {0: 2209, 1: 32768, 2: 32768, 3: 2048, 4: 2048}[args.config]   # about 10 s of the oracle on 16 threads
        sel = wl.sample_pixels(cfg, n_sample, 4242)
        t0 = time.perf_counter()
        oracle.run(cfg.layers, cfg.in_channels, cfg.patch, params.astype(np.float64),
                   img.astype(np.float64), lab, sel=sel, want_grads=True)
        cdt = time.perf_counter() - t0
        cpu = {"value": round(sel.size / cdt, 2), "unit": "pixels/s", "cores": oracle.threads(),
               "kind": "oracle", "sample": "%d seeded output pixels of %s, fp64 patch-by-patch forward+backward, "
               "%.1f s" % (sel.size, cfg.name, cdt)}

    out = {
        "metric": "training pixels/sec (fwd+bwd, whole image) on 1 MI355X",
        "value": round(value, 1), "unit": "pixels/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "height": cfg.height, "width": cfg.width,
                   "patch": cfg.patch, "valid_pixels_per_step": cfg.valid_pixels,
                   "storage": cfg.dtype,
                   "step": "fwd+bwd" + ("+sgd" if do_sgd else ""), "loss": final_loss},
        "roofline": roofline, "cpu_baseline": cpu,
        "deploy_forward": {"ms_per_image": round(fwd_ms_per_image, 4), "output": "%dx%d" % (cfg.height, cfg.width),
                           "borders": "mirrored"},
    }
    print(json.dumps(out))
    net.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
