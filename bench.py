#!/usr/bin/env python3
"""Benchmark of the scattering hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one forward transform (S0, S1, S2) of the whole batch of the headline
workload: Scattering2D, J=3, L=8, 128 RGB images of 256x256 (384 planes), synthetic
1/f^2 Gaussian fields, inputs and outputs resident in HBM.  Prints ONE JSON line:
throughput in images/s, the roofline of the kernel that takes the most time (timed live
with HIP events inside the library on the stream it launches on), and the fp64 CPU
oracle timed on this machine's host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
ALU_PEAK_TFLOPS = 157.3        # MI355X fp32 vector peak (256 CUs x 4 SIMD x 16 lanes x 2 x 2.4 GHz)
WORKLOAD = 2                   # index into workloads.CONFIGS: 2-D J=3 L=8 256x256, 128x3 planes
# committed rocprofv3 counter summaries, profiles/hbm_traffic_<tag>.txt, per workload index
TRAFFIC_TAGS = {0: "2d_J2_L8_32x32_b4", 1: "2d_J2_L8_32x32_b3072", 2: "2d_J3_L8_256x256_b384",
                3: "2d_J4_L8_512x512_b32", 4: "1d_J6_Q8_65536_b64", 5: "3d_J2_L3_64x64x64_b16"}


def cpu_baseline(planes, dims, J, LQ, channels, budget_s=20.0, grad=None):
    """Time the oracle (single process, numpy FFTs are single threaded) on as many planes
    of the workload as fit in about budget_s seconds.  With `grad` (dL/dS for every plane)
    the oracle's backward pass is timed instead of its forward pass."""
    import oracle
    if dims == 3:
        from oracle import harmonic3d
        bank = harmonic3d.bank_3d(planes.shape[-3:], J, LQ)
        if grad is not None:
            run = lambda x: harmonic3d.harmonic_scattering3d_backward(x, grad[:len(x)], J, LQ, bank=bank)
        else:
            run = lambda x: harmonic3d.harmonic_scattering3d(x, J, LQ, bank=bank)
    elif dims == 2 and grad is not None:
        n_r, n_c = planes.shape[-2:]
        bank = oracle.bank_2d(n_r, n_c, J, LQ)
        run = lambda x: oracle.scattering2d_backward(x, grad[:len(x)], J, LQ, bank=bank)
    elif grad is not None:
        bank = oracle.bank_1d(planes.shape[-1], J, LQ)
        run = lambda x: oracle.scattering1d_backward(x, grad[:len(x)], J, LQ, bank=bank)
    elif dims == 2:
        n_r, n_c = planes.shape[-2:]
        bank = oracle.bank_2d(n_r, n_c, J, LQ)     # built once, like the GPU plan; not timed
        run = lambda x: oracle.scattering2d(x, J, LQ, bank=bank)
    else:
        bank = oracle.bank_1d(planes.shape[-1], J, LQ)
        run = lambda x: oracle.scattering1d(x, J, LQ, bank=bank)
    t0 = time.perf_counter()
    run(planes[:1])
    one = time.perf_counter() - t0
    n = int(max(1, min(len(planes), budget_s / max(one, 1e-6))))
    t0 = time.perf_counter()
    run(planes[:n])
    dt = time.perf_counter() - t0
    return {"value": n / dt / channels, "unit": "images/s", "cores": 1, "kind": "oracle",
            "sample": "%d of %d planes (%d-channel images), fp64 numpy %s, filter bank "
                      "prebuilt, %.1f s" % (n, len(planes), channels,
                                            "backward pass (forward recomputed inside)"
                                            if grad is not None else "cascade", dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cpu-seconds", type=float, default=20.0,
                    help="CPU time budget of the oracle baseline (0 disables it)")
    ap.add_argument("--workload", type=int, default=WORKLOAD,
                    help="index of the configuration to run (default 2 = the headline one; "
                         "0, 1, 3, 4 are the other parity configurations, 5 the 3-D solid "
                         "harmonic transform of 16 volumes of 64^3, J=2, L=3)")
    ap.add_argument("--backward", action="store_true",
                    help="time the backward pass (gradient with respect to the input of a "
                         "seeded random dL/dS; recomputes the forward cascade inside) instead "
                         "of the forward transform")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known "
                         "traffic, to calibrate profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (planes are independent, so more GPUs would "
              "just split the batch); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_1812_11214_amd as scat
    from paper_1812_11214_amd import workloads

    wl = args.workload
    cfg = workloads.config(wl)
    P = workloads.num_planes(wl)
    C = cfg["channels"]
    x_host = workloads.planes(wl)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    x = torch.from_numpy(x_host).cuda()
    plan = scat.Scattering(cfg["shape"], cfg["J"], cfg["LQ"])
    out = torch.empty((P, plan.K) + plan.out_shape, dtype=torch.float32, device="cuda")
    g_host = None
    if args.backward:
        g_host = np.random.default_rng(181211214).standard_normal(
            tuple(out.shape), dtype=np.float32)
        g = torch.from_numpy(g_host).cuda()
        gin = torch.empty_like(x)
        step = lambda: plan.backward(x, g, grad_in=gin)
    else:
        step = lambda: plan.forward(x, out=out)

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()

    if args.copy_probe:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        b.copy_(a)                    # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b

    # which kernel takes the most time? (one untimed forward with every launch bracketed)
    plan.timing_begin(None)
    step()
    torch.cuda.synchronize()
    table = plan.timing_end()
    dominant = max(table, key=lambda k: table[k]["ms"])

    # timed region: K steps, the dominant kernel's launches bracketed by HIP events
    plan.timing_begin(dominant)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record()
    for _ in range(args.steps):
        step()
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dom = plan.timing_end()[dominant]
    ms_per_step = start.elapsed_time(stop) / args.steps

    # sanity: the output is finite and S0 of a zero-mean unit-variance field is small
    chk = (gin if args.backward else out)[:2].float().cpu().numpy()
    assert np.isfinite(chk).all()

    avg_ms = dom["ms"] / dom["launches"]
    bytes_per_launch = dom["alg_bytes"] / dom["launches"]
    flops_per_launch = dom["model_flops"] / dom["launches"]
    achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
    # HBM bytes per launch of every kernel from the committed rocprofv3 counter summary
    # (FETCH_SIZE and WRITE_SIZE runs of this same command, scaled by a plain copy)
    per_kernel = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s%s.txt"
                         % (TRAFFIC_TAGS.get(wl, "none"), "_backward" if args.backward else ""))
    if os.path.exists(tpath):
        with open(tpath) as f:
            for line in f:
                cols = line.rstrip("\n").split("\t")
                if not line.startswith("#") and len(cols) == 5:
                    per_kernel[cols[0]] = float(cols[4])
    traffic = per_kernel.get(dominant)
    # whole step: measured HBM bytes of all its launches over the measured step time
    pipeline = None
    if per_kernel and all(k in per_kernel for k in table):
        step_bytes = sum(per_kernel[k] * table[k]["launches"] for k in table)
        rate = step_bytes / (ms_per_step * 1e-3) / 1e9
        pipeline = {"hbm_bytes_per_step": step_bytes, "achieved": rate, "unit": "GB/s",
                    "frac": rate / HBM_PEAK_GBS,
                    "alg_bytes_per_step": sum(v["alg_bytes"] for v in table.values())}
    model_tflops = flops_per_launch / (avg_ms * 1e-3) / 1e12
    # the roofline that bounds this kernel: the larger of the time its least traffic needs
    # at the HBM peak and the time its model flops need at the fp32 vector peak
    hbm_bound = bytes_per_launch / (HBM_PEAK_GBS * 1e9) >= flops_per_launch / (ALU_PEAK_TFLOPS * 1e12)
    if hbm_bound:
        roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS}
    else:
        roofline = {"bound": "alu", "kernel": dominant, "achieved": model_tflops,
                    "peak": ALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": model_tflops / ALU_PEAK_TFLOPS}
    roofline.update({"traffic": traffic, "avg_launch_ms": avg_ms,
                     "launches_timed": dom["launches"],
                     "alg_bytes_per_launch": bytes_per_launch, "alg_gbs": achieved,
                     "model_tflops": model_tflops,
                     "share_of_step": dom["ms"] / args.steps / ms_per_step})
    # whole step against the fp32 vector peak with the 5 n log2 n flop model
    step_flops = sum(v["model_flops"] for v in table.values())
    step_tflops = step_flops / (ms_per_step * 1e-3) / 1e12
    pipeline_alu = {"model_flops_per_step": step_flops, "achieved": step_tflops,
                    "unit": "TFLOP/s", "peak": ALU_PEAK_TFLOPS,
                    "frac": step_tflops / ALU_PEAK_TFLOPS}

    images_per_s = (P / C) / (ms_per_step * 1e-3)
    result = {
        "metric": ("scattering backward pass (gradient wrt the input, forward recomputed) "
                   "images/sec on 1 MI355X (%s)" % cfg["name"] if args.backward else
                   "Scattering2D J=3 L=8 256x256 images/sec on 1 MI355X; % HBM roofline"
                   if wl == WORKLOAD else "scattering images/sec on 1 MI355X (%s)" % cfg["name"]),
        "value": images_per_s, "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg["name"], "planes_per_step": P, "channels": C,
                   "J": cfg["J"], "LQ": cfg["LQ"], "shape": list(cfg["shape"]), "max_order": 2,
                   "coefficients": plan.K},
        "planes_per_s": P / (ms_per_step * 1e-3),
        "wall_ms_per_step": wall / args.steps * 1e3,
        "roofline": roofline,
        "pipeline_hbm": pipeline,
        "pipeline_alu": pipeline_alu,
        "kernel_table_ms": {k: round(v["ms"], 4) for k, v in table.items()},
    }
    plan.close()
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(x_host, cfg["dims"], cfg["J"], cfg["LQ"], C,
                                              args.cpu_seconds, grad=g_host)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
