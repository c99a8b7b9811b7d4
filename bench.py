#!/usr/bin/env python3
"""Benchmark of the adjoint-stencil hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--all] [--no-cpu-baseline]

A step is one call of sadj_adjoint_wave3d (core region + remainder regions) on the
headline workload: 3-D variable-coefficient wave stencil, 25-point star (radius 4),
512^3 grid, fp64, u_bar accumulated, inputs already resident in HBM.  Prints ONE
JSON line.  `value` = grid points of u_bar updated per second (Gpoints/s).

roofline: HBM-bound.  achieved = algorithmic bytes per call / mean kernel time
measured with HIP events on the launch stream; algorithmic bytes = read c and r_bar
once on the primal interior, read and write u_bar once on the whole grid
(16 N + 16 |I| bytes in fp64).  peak = 8000 GB/s (MI355X HBM3E).

cpu_baseline: the CPU oracle (scatter adjoint, one core, gcc -O2) timed on the
leading z-planes of the same arrays (about 15 s of work, at most the whole grid).

With --all the same JSON line carries an "others" object with the remaining
workloads (fp32, radius 1, primal, 2-D, Burgers, 1-D), each timed the same way.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "adjoint stencil Gpoints/s + % of peak HBM GB/s, 3D wave r=4 512^3 fp64"


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for ln in fh:
                if ln.startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def interior_points(shape, radius):
    n = 1
    for s in shape:
        n *= s - 2 * radius
    return n


def wave_adjoint_bytes(shape, radius, esize, with_prev=False):
    N = int(np.prod(shape))
    I = interior_points(shape, radius)
    b = 2 * esize * N + 2 * esize * I
    if with_prev:
        b += 2 * esize * I
    return b


def time_calls(fn, steps, warmup):
    """Returns (wall ms per step, mean HIP-event ms per call).  Events are recorded
    on torch's current stream, which is the stream the binding launches on."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        starts[i].record()
        fn()
        stops[i].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ev = [s.elapsed_time(e) for s, e in zip(starts, stops)]
    return (t1 - t0) * 1e3 / steps, float(np.mean(ev)), float(np.min(ev))


def read_traffic(name):
    """HBM bytes per launch derived from rocprofv3 --pmc runs, kept as text under
    profiles/ (line 'traffic_bytes_per_launch: N'); None when not recorded."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as fh:
            for ln in fh:
                if ln.startswith("traffic_bytes_per_launch:"):
                    return float(ln.split(":", 1)[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--all", action="store_true", help="also time the other workloads")
    ap.add_argument("--remainder-study", action="store_true",
                    help="also time the three remainder strategies of the 3-D adjoint")
    ap.add_argument("--paper-sizes", action="store_true",
                    help="also time the paper's own two experiments (1000^3 wave step, 10^9-cell Burgers step; "
                         "needs about 35 GB of device memory)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--size", type=int, default=512, help="grid edge of the headline workload")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed region run one plain device copy of a whole array (the known-size "
                         "reference that calibrates rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the hot path is a single-GPU kernel "
              "library and no multi-GPU figure is produced); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import inputs
    import paper_1907_02818_amd as sadj

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sadj.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    n = args.size
    shape = (n, n, n)
    R = 4
    d = inputs.config_inputs("wave3d_r4", shape=shape, fields=("c", "r_bar", "u_bar"))
    c, rb, ub = (torch.from_numpy(d[k]).to(dev) for k in ("c", "r_bar", "u_bar"))
    torch.cuda.synchronize()

    wall_ms, ev_ms, ev_min = time_calls(lambda: sadj.sadj_adjoint_wave3d(R, c, rb, ub), args.steps, args.warmup)
    N = n ** 3
    alg_bytes = wave_adjoint_bytes(shape, R, 8)
    achieved = alg_bytes / (ev_ms * 1e-3) / 1e9
    out = {
        "metric": METRIC,
        "value": N / (wall_ms * 1e-3) / 1e9,
        "unit": "Gpoints/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "wave3d adjoint, 25-point star r=4, %d^3, fp64, u_bar only" % n,
                   "variant": sadj.get_option("wave3d.variant"),
                   "zchunk": sadj.get_option("wave3d.zchunk")},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": read_traffic("adjoint_wave3d_r4_f64_512_pmc.txt") if n == 512 else None,
                     "kernel_ms_mean": ev_ms, "kernel_ms_min": ev_min, "algorithmic_bytes": alg_bytes},
    }

    # the paper's own timings of the same method (Section 4, performance tables), with their
    # hardware: context only, another machine, another stencil radius and grid; `--paper-sizes`
    # times these two workloads here
    out["paper_context"] = {
        "wave_7pt_1000^3_gather_adjoint_best_s": {"Xeon E5-2650 v4, 12 threads": 1.322396, "Xeon Phi 7210, 64 threads": 1.286821},
        "wave_7pt_1000^3_primal_best_s": {"Xeon E5-2650 v4, 12 threads": 0.897188, "Xeon Phi 7210, 32 threads": 0.843320},
        "burgers_1e9_gather_adjoint_best_s": {"Xeon E5-2650 v4, 12 threads": 1.535777, "Xeon Phi 7210, 128 threads": 0.756979},
        "burgers_1e9_primal_best_s": {"Xeon E5-2650 v4, 12 threads": 0.555659, "Xeon Phi 7210, 128 threads": 0.502064},
    }

    others = {}

    def add(name, fn, points, nbytes, dtype):
        w, e, emin = time_calls(fn, max(5, args.steps // 4), max(3, args.warmup // 4))
        others[name] = {"Gpoints/s": points / (w * 1e-3) / 1e9, "ms": w, "kernel_ms_mean": e,
                        "GB/s": nbytes / (e * 1e-3) / 1e9, "frac": nbytes / (e * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "dtype": dtype}

    # fp32 run of the same workload (same draws rounded to float)
    c32, rb32, ub32 = c.float(), rb.float(), ub.float()
    add("wave3d_r4_f32_adjoint", lambda: sadj.sadj_adjoint_wave3d(R, c32, rb32, ub32), N,
        wave_adjoint_bytes(shape, R, 4), "f32")
    del c32, rb32, ub32

    if args.remainder_study:
        # Section 3.3.4's alternatives on the GPU: 0 guarded only where needed (default),
        # 1 guarded everywhere ("zero padding"), 2 core and remainder as separate dispatches
        for rad in (4, 1):
            for strat in (0, 1, 2):
                sadj.set_option("wave3d.remainder", strat)
                add("remainder_strategy%d_r%d_f64_adjoint" % (strat, rad),
                    lambda: sadj.sadj_adjoint_wave3d(rad, c, rb, ub), N, wave_adjoint_bytes(shape, rad, 8), "f64")
        sadj.set_option("wave3d.remainder", 0)
        # Section 3.5: terms added in the order and rounding of the sequential scatter
        sadj.set_option("wave3d.order", 1)
        for rad in (4, 1):
            add("scatter_order_r%d_f64_adjoint" % rad, lambda: sadj.sadj_adjoint_wave3d(rad, c, rb, ub), N,
                wave_adjoint_bytes(shape, rad, 8), "f64")
        sadj.set_option("wave3d.order", 0)
        # contrast: the conventional scatter with atomic updates (not the method)
        for rad in (4, 1):
            add("atomic_scatter_r%d_f64_adjoint" % rad, lambda: sadj.sadj_adjoint_wave3d_atomic_scatter(rad, c, rb, ub),
                N, wave_adjoint_bytes(shape, rad, 8), "f64")

    if args.all:
        upb = torch.from_numpy(inputs.config_inputs("wave3d_r4", shape=shape, fields=("u_prev_bar",))["u_prev_bar"]).to(dev)
        add("wave3d_r4_f64_adjoint_with_u_prev_bar", lambda: sadj.sadj_adjoint_wave3d(R, c, rb, ub, upb), N,
            wave_adjoint_bytes(shape, R, 8, True), "f64")
        # reverse sweep of a time loop: per step read c and lam_a on I, read+write lam_b, write lam_p
        ksteps = 6
        I4 = interior_points(shape, R)
        add("wave3d_r4_f64_adjoint_steps_per_step", lambda: sadj.sadj_adjoint_wave3d_steps(R, ksteps, c, rb, ub, upb),
            N * ksteps, ksteps * (16 * I4 + 16 * N + 8 * N), "f64")
        others["wave3d_r4_f64_adjoint_steps_per_step"]["ms"] /= ksteps
        others["wave3d_r4_f64_adjoint_steps_per_step"]["kernel_ms_mean"] /= ksteps
        # primal: reads u, u_prev, c, writes r (u_bar/u_prev_bar buffers reused as u/u_prev)
        r = torch.empty_like(ub)
        I = interior_points(shape, R)
        add("wave3d_r4_f64_primal", lambda: sadj.sadj_primal_wave3d(R, ub, upb, c, r), N, 8 * N + 24 * I, "f64")
        add("wave3d_r1_f64_adjoint", lambda: sadj.sadj_adjoint_wave3d(1, c, rb, ub), N,
            wave_adjoint_bytes(shape, 1, 8), "f64")
        add("wave3d_r1_f64_primal", lambda: sadj.sadj_primal_wave3d(1, ub, upb, c, r), N,
            8 * N + 24 * interior_points(shape, 1), "f64")
        for rad in (2, 3):
            add("wave3d_r%d_f64_adjoint" % rad, lambda: sadj.sadj_adjoint_wave3d(rad, c, rb, ub), N,
                wave_adjoint_bytes(shape, rad, 8), "f64")
        # dense 3x3x3 box stencil with asymmetric weights (27 terms), same grid
        wbox = [[[0.1 * (i + 3 * j + 9 * k) - 1.0 for i in range(3)] for j in range(3)] for k in range(3)]
        add("box3d_f64_adjoint", lambda: sadj.sadj_adjoint_box(wbox, c, rb, ub), N,
            wave_adjoint_bytes(shape, 1, 8), "f64")
        add("box3d_f64_primal", lambda: sadj.sadj_primal_box(wbox, ub, c, r), N,
            8 * N + 16 * interior_points(shape, 1), "f64")
        # general star of radius 4 with an asymmetric weight table (25 free weights)
        wstar = [0.3] + [0.05 * (i % 7) - 0.12 for i in range(24)]
        add("star3d_r4_f64_adjoint", lambda: sadj.sadj_adjoint_star3d(4, wstar, c, rb, ub), N,
            wave_adjoint_bytes(shape, 4, 8), "f64")
        add("star3d_r4_f64_primal", lambda: sadj.sadj_primal_star3d(4, wstar, ub, c, r), N,
            8 * N + 16 * interior_points(shape, 4), "f64")
        del upb, r
        # 2-D 8192^2
        s2 = (8192, 8192)
        c2, rb2, ub2 = (t.reshape(-1)[: s2[0] * s2[1]].reshape(s2) for t in (c, rb, ub))
        add("wave2d_f64_adjoint", lambda: sadj.sadj_adjoint_wave2d(c2, rb2, ub2), s2[0] * s2[1],
            wave_adjoint_bytes(s2, 1, 8), "f64")
        r2 = torch.empty_like(ub2)
        add("wave2d_f64_primal", lambda: sadj.sadj_primal_wave2d(ub2, rb2, c2, r2), s2[0] * s2[1],
            8 * s2[0] * s2[1] + 24 * interior_points(s2, 1), "f64")
        wbox2 = [[0.1 * (i + 3 * j) - 0.4 for i in range(3)] for j in range(3)]
        add("box2d_f64_adjoint", lambda: sadj.sadj_adjoint_box(wbox2, c2, rb2, ub2), s2[0] * s2[1],
            wave_adjoint_bytes(s2, 1, 8), "f64")
        del r2
        # Burgers 2^24, rotating three buffer sets so the arrays do not stay in the 256 MB last-level cache
        nb = 1 << 24
        sets = [tuple(t.reshape(-1)[k * nb:(k + 1) * nb] for t in (rb, c, ub)) for k in range(3)]
        state = {"i": 0}

        def burg():
            u_, r_, b_ = sets[state["i"] % 3]
            state["i"] += 1
            sadj.sadj_adjoint_burgers1d(0.1, 0.05, u_, r_, b_)
        add("burgers1d_f64_adjoint", burg, nb, 32 * nb, "f64")
        # reverse sweep over stored Burgers states: per step read u^t and lam, write lam (24 B/pt)
        ks = 12
        states = torch.rand(ks + 1, nb, device=dev, dtype=torch.float64)
        la, lb = torch.rand(nb, device=dev, dtype=torch.float64), torch.zeros(nb, device=dev, dtype=torch.float64)
        add("burgers1d_f64_adjoint_steps_per_step", lambda: sadj.sadj_adjoint_burgers1d_steps(0.1, 0.05, ks, ks, states, la, lb),
            nb * ks, 32 * nb + (ks - 1) * 24 * nb, "f64")
        others["burgers1d_f64_adjoint_steps_per_step"]["ms"] /= ks
        others["burgers1d_f64_adjoint_steps_per_step"]["kernel_ms_mean"] /= ks
        del states, la, lb
        sadj.set_option("stencil1d.functor", 1)      # same stencil through the generic functor kernel
        add("burgers1d_f64_adjoint_functor", burg, nb, 32 * nb, "f64")
        sadj.set_option("stencil1d.functor", 0)

        def burg_primal():
            u_, r_, b_ = sets[state["i"] % 3]
            state["i"] += 1
            sadj.sadj_primal_burgers1d(0.1, 0.05, u_, b_)
        add("burgers1d_f64_primal", burg_primal, nb, 16 * nb, "f64")
        n1 = 4096
        c1, rb1, ub1 = (t.reshape(-1)[:n1] for t in (c, rb, ub))
        add("wave1d_f64_adjoint_n4096_latency", lambda: sadj.sadj_adjoint_wave1d(c1, rb1, ub1), n1, 32 * n1, "f64")
        # the same call recorded 100 times into a HIP graph: the launch-bound size without host launch cost
        per_graph = 100
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            sadj.sadj_adjoint_wave1d(c1, rb1, ub1)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(per_graph):
                sadj.sadj_adjoint_wave1d(c1, rb1, ub1)
        add("wave1d_f64_adjoint_n4096_in_hip_graph_per_call", graph.replay, n1 * per_graph, 32 * n1 * per_graph, "f64")
        for key in ("ms", "kernel_ms_mean"):
            others["wave1d_f64_adjoint_n4096_in_hip_graph_per_call"][key] /= per_graph
    if args.paper_sizes:
        # The paper's experiments (Section 4.1: one step of the 7-point wave solver on 1000^3;
        # Section 4.2: one Burgers step on 10^9 cells), fp64, synthetic values.  The paper's
        # best gather-adjoint and primal times are quoted as context with their hardware
        # (one 12-core Xeon E5-2650 v4 socket; Xeon Phi 7210); they are not a baseline for `value`.
        s3 = (1000, 1000, 1000)
        N3 = s3[0] * s3[1] * s3[2]
        gen = torch.Generator(device=dev)
        gen.manual_seed(1907)
        cw = torch.rand(s3, generator=gen, device=dev, dtype=torch.float64) * 0.09 + 0.01
        a1, a2, a3 = (torch.rand(s3, generator=gen, device=dev, dtype=torch.float64) * 2 - 1 for _ in range(3))

        def add_paper(name, fn, points, nbytes, paper):
            add(name, fn, points, nbytes, "f64")
            others[name]["paper_context"] = dict(paper, note="the paper's timing on its own hardware; context only")
            others[name]["paper_context"]["time_ratio_paper_over_here"] = paper["seconds_best"] / (others[name]["ms"] * 1e-3)

        add_paper("paper_wave3d_7pt_1000^3_f64_adjoint_u_bar_and_u_prev_bar",
                  lambda: sadj.sadj_adjoint_wave3d(1, cw, a1, a2, a3), N3, wave_adjoint_bytes(s3, 1, 8, True),
                  {"seconds_best": 1.322396, "hardware": "Xeon E5-2650 v4, 12 threads",
                   "seconds_best_other": 1.286821, "hardware_other": "Xeon Phi 7210, 64 threads"})
        add_paper("paper_wave3d_7pt_1000^3_f64_primal",
                  lambda: sadj.sadj_primal_wave3d(1, a2, a3, cw, a1), N3, 8 * N3 + 24 * interior_points(s3, 1),
                  {"seconds_best": 0.897188, "hardware": "Xeon E5-2650 v4, 12 threads",
                   "seconds_best_other": 0.843320, "hardware_other": "Xeon Phi 7210, 32 threads"})
        ub1d, rb1d, ubar1d, r1d = (t.reshape(-1) for t in (a1, a2, a3, cw))
        add_paper("paper_burgers1d_1e9_f64_adjoint",
                  lambda: sadj.sadj_adjoint_burgers1d(0.1, 0.05, ub1d, rb1d, ubar1d), N3, 32 * N3,
                  {"seconds_best": 1.535777, "hardware": "Xeon E5-2650 v4, 12 threads",
                   "seconds_best_other": 0.756979, "hardware_other": "Xeon Phi 7210, 128 threads"})
        add_paper("paper_burgers1d_1e9_f64_primal",
                  lambda: sadj.sadj_primal_burgers1d(0.1, 0.05, ub1d, r1d), N3, 16 * N3,
                  {"seconds_best": 0.555659, "hardware": "Xeon E5-2650 v4, 12 threads",
                   "seconds_best_other": 0.502064, "hardware_other": "Xeon Phi 7210, 128 threads"})
        del cw, a1, a2, a3, ub1d, rb1d, ubar1d, r1d
    out["others"] = others
    if args.copy_probe:
        ub.copy_(c)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()

        def run_oracle(nzs):
            sl = (slice(0, nzs),)
            t0 = time.perf_counter()
            oracle.wave_adjoint(d["c"][sl], d["r_bar"][sl], d["u_bar"][sl], R)
            return time.perf_counter() - t0

        probe = min(n, 32)
        rate = probe / run_oracle(probe)                 # planes per second on this host
        nzs = int(min(n, max(probe, rate * 15.0)))      # about 15 s of CPU work, at most the whole grid
        dt = run_oracle(nzs)
        out["cpu_baseline"] = {"value": nzs * n * n / dt / 1e9, "unit": "Gpoints/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d z-planes of the same %d^3 arrays (%d x %d x %d grid), one run, "
                                         "%.1f s" % (nzs, n, n, n, nzs, dt),
                               "host_cpus": os.cpu_count(), "host_cpu_model": cpu_model()}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
