#!/usr/bin/env python3
"""Benchmark of the scattering hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one forward transform (S0, S1, S2) of the whole batch of the headline
workload: Scattering2D, J=3, L=8, 128 RGB images of 256x256 (384 planes), synthetic
1/f^2 Gaussian fields, inputs and outputs resident in HBM.  Prints ONE JSON line:
throughput in images/s; `roofline`, the fraction of the binding roofline (fp32 vector ALUs:
the path's algorithmic bytes need far less time at the HBM peak than its model flops at the
ALU peak) reached by the kernel that takes the most time, timed live with HIP events inside
the library on the stream it launches on; `step`, the same for the whole step together with
the algorithmic and the measured HBM traffic and their ratio; and the fp64 CPU oracle timed
on this machine's host cores on a bounded sample of the same workload.
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
TRAFFIC_TAGS = {1: "2d_J2_L8_32x32_b3072", 2: "2d_J3_L8_256x256_b384",
                3: "2d_J4_L8_512x512_b32", 4: "1d_J6_Q8_65536_b64", 5: "3d_J2_L3_64x64x64_b16"}
# Algorithmic work per plane of the forward transform, per workload index: model flops
# (5 n log2 n for every transform of the cascade taken as a full complex one, plus the
# pointwise products, folds and moduli) and bytes (input + output + filter tables / planes).
MODEL_MFLOP_PER_PLANE = {0: 2.50 + 0.52, 1: 2.50 + 0.52, 2: 332.2 + 60.0, 3: 1587.7 + 342.0,
                         4: 296.0 + 43.5}
ALG_BYTES_PER_PLANE = {0: 4096 + 20736 + 17664, 1: 4096 + 20736 + 23, 2: 262144 + 888832 + 18645,
                       3: 1048576 + 1708032 + 1239552, 4: 262144 + 692224 + 237000}


def oracle_worker(wl, start, count, t_start):
    """One process of the all-cores leg (`bench.py --oracle-worker wl start count t_start`):
    builds the filter bank and its planes untimed, waits for the common start time, runs the
    forward oracle and prints when it started and finished (time.time())."""
    import oracle
    from paper_1812_11214_amd import workloads
    cfg = workloads.config(wl)
    x = workloads.planes(wl, count, start)
    if cfg["dims"] == 2:
        bank = oracle.bank_2d(cfg["shape"][0], cfg["shape"][1], cfg["J"], cfg["LQ"])
        run = lambda v: oracle.scattering2d(v, cfg["J"], cfg["LQ"], bank=bank)
    else:
        bank = oracle.bank_1d(cfg["shape"][0], cfg["J"], cfg["LQ"])
        run = lambda v: oracle.scattering1d(v, cfg["J"], cfg["LQ"], bank=bank)
    run(x[:1])
    ready = time.time()
    while time.time() < t_start:
        time.sleep(0.001)
    t0 = time.time()
    run(x)
    print("%.6f %.6f %.6f" % (ready, t0, time.time()), flush=True)


def cpu_all_cores(wl, total_planes, channels, per_plane_s, budget_s):
    """The forward oracle on one worker process per host core this process may run on (at most
    16), each with its own planes of the workload (planes are independent; numpy's FFT is
    single threaded).  The workers start together; throughput = planes / (last end - start)."""
    import subprocess
    cores = min(len(os.sched_getaffinity(0)), 16)
    per = int(max(1, min(total_planes // cores, budget_s / max(per_plane_s, 1e-6))))
    setup_s = 20.0 + 3.0 * per_plane_s           # imports, bank, planes, one warm-up plane
    t_start = time.time() + setup_s
    env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1")
    procs = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--oracle-worker",
                               str(wl), str(i * per), str(per), repr(t_start)],
                              stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, env=env)
             for i in range(cores)]
    ends, late = [], 0
    try:
        for pr in procs:
            outp, _ = pr.communicate(timeout=setup_s + 6.0 * per * per_plane_s + 60.0)
            ready, t0, t1 = (float(v) for v in outp.split())
            late += ready > t_start
            ends.append(t1)
    except Exception:
        for pr in procs:
            if pr.poll() is None:
                pr.kill()
        return None
    dt = max(ends) - t_start
    return {"value": cores * per / dt / channels, "unit": "images/s", "cores": cores,
            "sample": "%d planes on each of %d worker processes, started together, %.1f s%s"
                      % (per, cores, dt, " (%d workers were late)" % late if late else "")}


def cpu_baseline(planes, dims, J, LQ, channels, budget_s=20.0, grad=None, wl=None):
    """Time the oracle on as many planes of the workload as fit in about budget_s seconds:
    one process on one core (numpy's FFT is single threaded) and, for the forward pass of the
    1-D and 2-D cascades, a pool of processes on all host cores.  With `grad` (dL/dS for every
    plane) the oracle's backward pass is timed instead of its forward pass."""
    import oracle
    pool_leg = grad is None and dims in (1, 2) and wl is not None
    if pool_leg:
        budget_s *= 0.4               # the rest goes to the all-cores leg
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
    single = {"value": n / dt / channels, "unit": "images/s", "cores": 1, "kind": "oracle",
              "sample": "%d of %d planes (%d-channel images), fp64 numpy %s, filter bank "
                        "prebuilt, %.1f s" % (n, len(planes), channels,
                                              "backward pass (forward recomputed inside)"
                                              if grad is not None else "cascade", dt)}
    if not pool_leg:
        return single
    allc = cpu_all_cores(wl, len(planes), channels, dt / n, budget_s * 1.5)
    if allc is None:
        return single
    return {"value": allc["value"], "unit": "images/s", "cores": allc["cores"], "kind": "oracle",
            "sample": "fp64 numpy cascade, filter bank prebuilt, %d-channel images: %s"
                      % (channels, allc["sample"]),
            "single_core": single}


def main():
    if len(sys.argv) == 6 and sys.argv[1] == "--oracle-worker":
        oracle_worker(int(sys.argv[2]), int(sys.argv[3]), int(sys.argv[4]), float(sys.argv[5]))
        return
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
    ap.add_argument("--pass-kernels", action="store_true",
                    help="2-D 256x256 / 128x128 plans: row and column passes over the whole batch "
                         "(SCAT_PLAN_PASS_KERNELS) instead of the default walk of the tree with "
                         "one workgroup per node")
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
    plan = scat.Scattering(cfg["shape"], cfg["J"], cfg["LQ"], node_kernels=not args.pass_kernels)
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
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dom = plan.timing_end()[dominant]
    ms_per_step = marks[0].elapsed_time(marks[-1]) / args.steps
    each = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))

    # sanity: the output is finite and S0 of a zero-mean unit-variance field is small
    chk = (gin if args.backward else out)[:2].float().cpu().numpy()
    assert np.isfinite(chk).all()

    avg_ms = dom["ms"] / dom["launches"]
    bytes_per_launch = dom["alg_bytes"] / dom["launches"]
    flops_per_launch = dom["model_flops"] / dom["launches"]
    # HBM bytes per launch of every kernel from the committed rocprofv3 counter summary
    # (FETCH_SIZE and WRITE_SIZE runs of this same command, scaled by a plain copy)
    per_kernel = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s%s%s.txt"
                         % (TRAFFIC_TAGS.get(wl, "none"), "_backward" if args.backward else "",
                            "_pass_kernels" if args.pass_kernels else ""))
    if os.path.exists(tpath):
        with open(tpath) as f:
            for line in f:
                cols = line.rstrip("\n").split("\t")
                if not line.startswith("#") and len(cols) == 5:
                    per_kernel[cols[0]] = float(cols[4])
    traffic = per_kernel.get(dominant)
    measured_step_bytes = None
    if per_kernel and all(k in per_kernel for k in table):
        measured_step_bytes = sum(per_kernel[k] * table[k]["launches"] for k in table)

    # ---- the dominant kernel against the roofline that binds it.  Its work: the model flops
    # of the transforms and pointwise steps it performs (5 n log2 n per transform; the
    # library's per-launch figure) and, as HBM bytes, what of the path's inputs, outputs and
    # tables it touches; everything else it moves is intermediate traffic, not work.
    model_tflops = flops_per_launch / (avg_ms * 1e-3) / 1e12
    t_alu = flops_per_launch / (ALU_PEAK_TFLOPS * 1e12)
    roofline = {"bound": "alu", "kernel": dominant, "achieved": model_tflops,
                "peak": ALU_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": model_tflops / ALU_PEAK_TFLOPS,
                "traffic": traffic, "avg_launch_ms": avg_ms, "launches_timed": dom["launches"],
                "model_flops_per_launch": flops_per_launch,
                "share_of_step": dom["ms"] / args.steps / ms_per_step,
                # the kernel's own least I/O (intermediates included) over its time: how fast
                # the pass moves data, NOT a fraction of any roofline of the path
                "pass_io_bytes_per_launch": bytes_per_launch,
                "pass_io_gbs": bytes_per_launch / (avg_ms * 1e-3) / 1e9}

    # ---- the whole step: model flops and algorithmic bytes (input + output + tables) of the
    # workload against the two peaks; the binding roofline is the one that needs more time
    t_step = ms_per_step * 1e-3
    if not args.backward and wl in MODEL_MFLOP_PER_PLANE:
        step_flops = MODEL_MFLOP_PER_PLANE[wl] * 1e6 * P
        alg_bytes = float(ALG_BYTES_PER_PLANE[wl]) * P
    else:  # no tabulated figure: the library's own sums (flops) and plain input + output
        step_flops = sum(v["model_flops"] for v in table.values())
        alg_bytes = float(x.numel() * 4 + out.numel() * 4) * (2 if args.backward else 1)
    t_alu_step = step_flops / (ALU_PEAK_TFLOPS * 1e12)
    t_hbm_step = alg_bytes / (HBM_PEAK_GBS * 1e9)
    step_info = {
        "model_flops": step_flops, "model_tflops": step_flops / t_step / 1e12,
        "frac_alu": t_alu_step / t_step,
        "alg_bytes": alg_bytes, "alg_gbs": alg_bytes / t_step / 1e9,
        "hbm_alg_frac": t_hbm_step / t_step,
        "binding": "alu" if t_alu_step >= t_hbm_step else "hbm",
        "frac_binding": max(t_alu_step, t_hbm_step) / t_step,
        "measured_hbm_bytes": measured_step_bytes,
        "measured_hbm_gbs": measured_step_bytes / t_step / 1e9 if measured_step_bytes else None,
        "measured_hbm_frac": (measured_step_bytes / t_step / 1e9 / HBM_PEAK_GBS
                              if measured_step_bytes else None),
        "traffic_amplification": measured_step_bytes / alg_bytes if measured_step_bytes else None,
        "library_model_flops": sum(v["model_flops"] for v in table.values()),
        "ms_median": each[len(each) // 2], "ms_min": each[0], "ms_max": each[-1],
    }

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
                   "coefficients": plan.K,
                   "schedule": "pass_kernels" if args.pass_kernels else "default"},
        "planes_per_s": P / (ms_per_step * 1e-3),
        "wall_ms_per_step": wall / args.steps * 1e3,
        "roofline": roofline,
        "step": step_info,
        "kernel_table_ms": {k: round(v["ms"], 4) for k, v in table.items()},
    }
    plan.close()
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(x_host, cfg["dims"], cfg["J"], cfg["LQ"], C,
                                              args.cpu_seconds, grad=g_host, wl=wl)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
