#!/usr/bin/env python3
"""Throughput of the whole-image MPCNN training pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--only-headline]
                    [--no-cpu-baseline] [--kernels]

One step = one pass of the whole hot path (forward + backward of every layer, all
kernels of the C ABI call mpcnn_seg_backward; plus mpcnn_sgd_step for the workload
that trains) over one batch of seeded synthetic images already resident in HBM.

Prints ONE JSON line.  The headline (`value`, `ms_per_step`, `roofline`, `cpu_baseline`) is
the largest fp32 workload, cfg3_deep78_1024, timed over exactly K steps after W warm-up
steps.  `other_workloads` carries the other benchmark configurations, each with its own
step time, pixels/s and rooflines: cfg1_steel44_256, cfg2_steel44_8x512_sgd (as stated: 10 x
forward + backward + SGD step - the ten steps are the measurement, after one warm-up pass of
ten steps from the same parameters) and cfg4_deep78_rgb_2x2048_bf16 (bf16 storage).

Every workload reports two roofline entries, both from per-launch HIP events recorded on
the launch stream by the library's profile hooks over a repeat of the timed steps:
  `roofline`      the dominant matrix-core launch site family (conv forward, data gradient or
                  weight gradient): algorithmic flops / time against the MFMA peak of the
                  instruction that family runs on (fp32 157.3 TFLOP/s, bf16 2500 TFLOP/s);
  `roofline_hbm`  the max-filter and routing passes: algorithmic bytes / time against 8 TB/s.
`cpu_baseline` is the fp64 patch-by-patch oracle timed on this machine's host cores on a bounded
sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA = 157.3      # TFLOP/s, MI355X dense fp32 matrix
PEAK_BF16_MFMA = 2500.0     # TFLOP/s, dense bf16 matrix
PEAK_HBM = 8000.0           # GB/s, HBM3E
HEADLINE = 3
# pixels the oracle is timed on (about 10 s on 16 threads for the headline, a few seconds for the rest)
ORACLE_SAMPLE = {0: 2209, 1: 8192, 2: 8192, 3: 1536, 4: 384}
MATRIX_SITES = ("conv_fwd", "conv_dgrad", "wgrad")


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


def rooflines(stats, steps, ms_per_step, workload):
    """The two roofline entries from the per-site records of `steps` profiled steps."""
    by_name = {}
    for s in stats:
        if s["launches"] == 0:
            continue
        k = by_name.setdefault(s["name"], dict(ms=0.0, launches=0, flops=0.0, bytes=0.0))
        k["ms"] += s["ms_total"]
        k["launches"] += s["launches"]
        k["flops"] += s["flops"] * s["launches"]
        k["bytes"] += s["bytes"] * s["launches"]
    matrix = {n: v for n, v in by_name.items() if n.startswith(MATRIX_SITES) and n.endswith(("_mfma", "_bm"))}
    out = {}
    if matrix:
        name = max(matrix, key=lambda n: matrix[n]["ms"])
        dom = matrix[name]
        peak = PEAK_BF16_MFMA if name.endswith("_bm") else PEAK_FP32_MFMA
        achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        out["roofline"] = {
            "bound": "mfma", "achieved": round(achieved, 3), "peak": peak, "unit": "TFLOP/s",
            "frac": round(achieved / peak, 4),
            "traffic": read_traffic(os.path.join(ROOT, "profiles", "traffic_%s.txt" % workload), name),
            "kernel": name, "avg_launch_us": round(1e3 * dom["ms"] / dom["launches"], 2),
            "launches_per_step": dom["launches"] // steps,
            "share_of_step": round(dom["ms"] / steps / ms_per_step, 3),
            "all_matrix_sites": {n: {"achieved": round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2),
                                     "frac": round(v["flops"] / (v["ms"] * 1e-3) / 1e12 /
                                                   (PEAK_BF16_MFMA if n.endswith("_bm") else PEAK_FP32_MFMA), 4),
                                     "us_per_step": round(1e3 * v["ms"] / steps, 1)}
                                 for n, v in sorted(matrix.items())},
        }
    pool = {n: by_name[n] for n in ("maxfilter_fwd", "maxfilter_bwd") if n in by_name}
    if pool:
        ms = sum(v["ms"] for v in pool.values())
        byts = sum(v["bytes"] for v in pool.values())
        traffic = [read_traffic(os.path.join(ROOT, "profiles", "traffic_%s.txt" % workload), n) for n in pool]
        out["roofline_hbm"] = {
            "bound": "hbm", "achieved": round(byts / (ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM, "unit": "GB/s",
            "frac": round(byts / (ms * 1e-3) / 1e9 / PEAK_HBM, 4),
            "kernels": {n: {"achieved": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1),
                            "frac": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9 / PEAK_HBM, 4),
                            "avg_launch_us": round(1e3 * v["ms"] / v["launches"], 2),
                            "algorithmic_bytes_per_launch": round(v["bytes"] / v["launches"]),
                            "traffic": t}
                        for (n, v), t in zip(pool.items(), traffic)},
            "launches_per_step": sum(v["launches"] for v in pool.values()) // steps,
            "share_of_step": round(ms / steps / ms_per_step, 3),
        }
    return out, by_name


def run_workload(index, steps, warmup, cpu_baseline, kernels, deploy, graph=False):
    import numpy as np
    import torch
    from paper_1302_1690_amd import mpcnn, workloads as wl

    cfg = wl.CONFIGS[index]
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

    for _ in range(warmup):
        step()
    if do_sgd:
        net.set_params(params)                   # the measured steps start from the same parameters
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / steps
    final_loss = float(loss.item())

    # ---- per-kernel durations: the same steps again with HIP events around every launch
    if do_sgd:
        net.set_params(params)
    net.profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    stats = net.profile_read()
    net.profile_enable(False)
    roofs, by_name = rooflines(stats, steps, ms_per_step, cfg.name)
    if kernels:
        tot = sum(v["ms"] for v in by_name.values())
        print("---- %s: %.3f ms per step" % (cfg.name, ms_per_step), file=sys.stderr)
        for n, v in sorted(by_name.items(), key=lambda kv: -kv[1]["ms"]):
            tf = v["flops"] / (v["ms"] * 1e-3) / 1e12 if v["ms"] > 0 else 0
            gb = v["bytes"] / (v["ms"] * 1e-3) / 1e9 if v["ms"] > 0 else 0
            print("%-20s %3d launches/step %8.1f us/step %5.1f%%  %7.2f TFLOP/s %8.1f GB/s" % (
                n, v["launches"] // steps, 1e3 * v["ms"] / steps, 100 * v["ms"] / tot, tf, gb), file=sys.stderr)
        for s in sorted(stats, key=lambda s: -s["ms_total"]):
            if s["launches"]:
                us = 1e3 * s["ms_total"] / s["launches"]
                print("  %-20s layer %2d  %8.1f us  %7.2f TFLOP/s %8.1f GB/s" % (
                    s["name"], s["layer"], us, s["flops"] / us / 1e6, s["bytes"] / us / 1e3), file=sys.stderr)

    out = {
        "workload": cfg.name, "value": round(cfg.valid_pixels * steps / dt, 1), "unit": "pixels/s",
        "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "config": {"workload": cfg.name, "batch": cfg.batch, "height": cfg.height, "width": cfg.width,
                   "patch": cfg.patch, "valid_pixels_per_step": cfg.valid_pixels, "storage": cfg.dtype,
                   "step": "fwd+bwd" + ("+sgd(lr %g on the mean loss)" % cfg.lr if do_sgd else ""),
                   "loss": final_loss},
    }
    out.update(roofs)

    # ---- the same step recorded once into a HIP graph and replayed (the step only launches kernels on the
    # stream it is given): what the launches' host side costs, reported beside the eager figure
    if graph:
        if do_sgd:
            net.set_params(params)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                               # (weight packs brought up to date outside the recording when nothing updates them)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step()
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        out["graph_replay_ms_per_step"] = round(1e3 * (time.perf_counter() - t0) / steps, 4)
        del g

    # ---- deployment forward of the same images (mirrored borders, output as large as the image;
    # outside the timed training steps): milliseconds per image, the unit the paper quotes for it
    if deploy:
        net.seg_forward_same(d_img)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_fwd = max(5, steps // 2)
        for _ in range(n_fwd):
            net.seg_forward_same(d_img)
        torch.cuda.synchronize()
        out["deploy_forward"] = {"ms_per_image": round(1e3 * (time.perf_counter() - t0) / (n_fwd * cfg.batch), 4),
                                 "output": "%dx%d" % (cfg.height, cfg.width), "borders": "mirrored"}
    net.close()
    del ws, probs, d_img, d_lab
    torch.cuda.empty_cache()

    # ---- the oracle on the host cores, bounded sample of the same workload
    if cpu_baseline:
        import oracle
        sel = wl.sample_pixels(cfg, ORACLE_SAMPLE[index], 4242)
        t0 = time.perf_counter()
        oracle.run(cfg.layers, cfg.in_channels, cfg.patch, params.astype(np.float64),
                   img.astype(np.float64), lab, sel=sel, want_grads=True)
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(sel.size / cdt, 2), "unit": "pixels/s", "cores": oracle.threads(),
                               "kind": "oracle",
                               "sample": "%d seeded output pixels of %s, fp64 patch-by-patch forward+backward, "
                                         "%.1f s" % (sel.size, cfg.name, cdt)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=HEADLINE, help="headline workload index (default: the largest fp32 one)")
    ap.add_argument("--only-headline", action="store_true", help="skip the other workloads")
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

    import torch
    from paper_1302_1690_amd import workloads as wl

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

    cpu = not args.no_cpu_baseline
    head = run_workload(args.config, args.steps, args.warmup, cpu, args.kernels, deploy=True, graph=not args.only_headline)
    others = []
    if not args.only_headline:
        for idx in (1, 2, 4, 3):
            if idx == args.config:
                continue
            cfg = wl.CONFIGS[idx]
            if cfg.sgd_steps > 0:
                k, w = cfg.sgd_steps, cfg.sgd_steps   # the ten steps are the measurement, after one warm-up pass
            elif idx == 4:
                k, w = max(3, min(args.steps, 5)), 2  # 40 ms steps: a handful
            elif idx == 1:
                k, w = max(args.steps, 50), max(args.warmup, 5)
            else:
                k, w = args.steps, args.warmup
            others.append(run_workload(idx, k, w, cpu, args.kernels, deploy=(idx == 1), graph=True))

    out = {
        "metric": "training pixels/sec (fwd+bwd, whole image) on 1 MI355X",
        "value": head["value"], "unit": "pixels/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"],
        "roofline": head.get("roofline"), "roofline_hbm": head.get("roofline_hbm"),
        "cpu_baseline": head.get("cpu_baseline"),
        "deploy_forward": head.get("deploy_forward"),
        "graph_replay_ms_per_step": head.get("graph_replay_ms_per_step"),
        "other_workloads": others,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
