#!/usr/bin/env python3
"""Benchmark of the adjoint-stencil hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--all] [--only NAME] [--no-cpu-baseline]

A step is one call of sadj_adjoint_wave3d (core region + remainder regions) on the
headline workload: 3-D variable-coefficient wave stencil, 25-point star (radius 4),
512^3 grid, fp64, u_bar accumulated, inputs already resident in HBM.  Prints ONE
JSON line.  `value` = grid points of u_bar updated per second (Gpoints/s).

Timing protocol.  After a load step from idle the GPU's firmware lowers the shader
clock for some 20 ms (2.43 -> about 1.5 GHz, restored in steps; the memory clock stays
put), and a kernel that is not purely memory-bound runs up to 20 % slower meanwhile.
Every timed leg is therefore preceded by a disclosed SETTLE phase: the call is launched
in groups of ten until the per-launch times of a group agree within 1 % (its slowest
and fastest launch set aside) and the group's mean is within 1 % of the previous
group's (at most `--settle-cap` launches).
Then come the W warm-up and the K timed steps exactly as the flags say; nothing inside
the timed region differs from a run without the settle phase.  The JSON carries
`settle_launches` and the mean of the first (unsettled) launches next to the timed mean.

roofline: HBM-bound.  achieved = algorithmic bytes per call / mean kernel time
measured with HIP events on the launch stream; algorithmic bytes = read c and r_bar
once on the primal interior, read and write u_bar once on the whole grid
(16 N + 16 |I| bytes in fp64).  peak = 8000 GB/s (MI355X HBM3E).  stream_ceiling =
what the library's plain streaming kernel with the same mix of streams (two arrays
read, one read and written, no halo) reaches in the same process.

cpu_baseline: the CPU oracle (scatter adjoint, one core, gcc -O2) on the same arrays,
median of three runs.

`others` carries the remaining workloads of the benchmark definition (fp32, with
u_prev_bar, primal, radius 1, 2-D, Burgers, 1-D), each timed the same way; --all adds
the further stencil families, --only NAME times a single workload (for profiling).
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
HEADLINE = "wave3d_r4_f64_adjoint"


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


def read_traffic(workload):
    """HBM bytes per launch from the rocprofv3 --pmc summary profiles/<workload>_pmc.txt
    (lines 'traffic_bytes_per_launch: N' and 'library_sources_sha256: H').  Returns
    (bytes or None, note): the value is reported only if the summary was taken from the
    sources this library was built from."""
    path = os.path.join(ROOT, "profiles", workload + "_pmc.txt")
    val = sha = None
    try:
        with open(path) as fh:
            for ln in fh:
                if ln.startswith("traffic_bytes_per_launch:"):
                    val = float(ln.split(":", 1)[1])
                elif ln.startswith("library_sources_sha256:"):
                    sha = ln.split(":", 1)[1].strip()
    except OSError:
        return None, "no counter summary recorded for this workload"
    if val is None:
        return None, "summary holds no traffic line"
    from paper_1907_02818_amd.profile_summary import library_sources_sha256
    if sha != library_sources_sha256():
        return None, "recorded summary profiles/%s_pmc.txt is from other kernel sources (stale)" % workload
    return val, "recorded: profiles/%s_pmc.txt, same kernel sources (sha256 %s)" % (workload, sha[:12])


class Timer:
    def __init__(self, settle_cap):
        self.settle_cap = settle_cap

    def settle(self, fn):
        """Launch in groups of ten until the clocks have settled (see module docstring).
        Returns (launches done, mean ms of the first up to 25 launches, settled?)."""
        import torch
        group, tol = 10, 0.01
        done, first, prev_mean, ok = 0, [], None, False
        while done < self.settle_cap:
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(group + 1)]
            ev[0].record()
            for i in range(group):
                fn()
                ev[i + 1].record()
            torch.cuda.synchronize()
            t = [ev[i].elapsed_time(ev[i + 1]) for i in range(group)]
            done += group
            if len(first) < 25:
                first.extend(t[: 25 - len(first)])
            mean = float(np.mean(t))
            mid = sorted(t)[1:-1]                     # one outlier on either side is tolerated
            if mid[-1] <= mid[0] * (1 + tol) and prev_mean is not None and abs(mean - prev_mean) <= tol * prev_mean:
                ok = True
                break
            prev_mean = mean
        return done, (float(np.mean(first)) if first else None), ok

    def time_calls(self, fn, steps, warmup):
        """Returns a dict: wall ms per step, mean / min HIP-event ms per call (events are
        recorded on torch's current stream, the stream the binding launches on), and the
        settle phase's figures."""
        import torch
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        settle_launches, first_ms, settled = self.settle(fn) if self.settle_cap > 0 else (0, None, False)
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            starts[i].record()
            fn()
            stops[i].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ev = [s.elapsed_time(e) for s, e in zip(starts, stops)]
        return {"wall_ms": (t1 - t0) * 1e3 / steps, "ev_mean": float(np.mean(ev)), "ev_min": float(np.min(ev)),
                "settle_launches": settle_launches, "settled": settled, "unsettled_first_ms": first_ms}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--all", action="store_true", help="also time the further stencil families and modes")
    ap.add_argument("--only", default=None, help="time this one workload only (a key of `others`, or the headline)")
    ap.add_argument("--remainder-study", action="store_true",
                    help="also time the three remainder strategies of the 3-D adjoint")
    ap.add_argument("--paper-sizes", action="store_true",
                    help="also time the paper's own two experiments (1000^3 wave step, 10^9-cell Burgers step; "
                         "needs about 35 GB of device memory)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--settle-cap", type=int, default=300,
                    help="upper limit of launches in the settle phase before each timed leg (0 = no settle phase)")
    ap.add_argument("--size", type=int, default=512, help="grid edge of the headline workload")
    ap.add_argument("--size2d", type=int, default=8192, help="grid edge of the 2-D workloads (views of the 3-D arrays: "
                    "size2d^2 may not exceed size^3)")
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
    timer = Timer(args.settle_cap)

    n = args.size
    shape = (n, n, n)
    R = 4
    N = n ** 3
    d = inputs.config_inputs("wave3d_r4", shape=shape, fields=("c", "r_bar", "u_bar"))
    c, rb, ub = (torch.from_numpy(d[k]).to(dev) for k in ("c", "r_bar", "u_bar"))
    torch.cuda.synchronize()

    others = {}
    steps_o, warm_o = max(5, args.steps // 4), max(3, args.warmup // 4)

    def add(name, fn, points, nbytes, dtype, per=1, steps=None, warmup=None):
        """Time one further workload; `per` = inner steps one call performs.  One untimed
        call first, so that arrays the workload creates on first use exist."""
        fn()
        torch.cuda.synchronize()
        t = timer.time_calls(fn, steps or steps_o, warmup or warm_o)
        gbs = nbytes / (t["ev_mean"] * 1e-3) / 1e9
        traffic, tnote = read_traffic(name) if n == 512 else (None, "")
        others[name] = {"Gpoints/s": points / (t["wall_ms"] * 1e-3) / 1e9, "ms": t["wall_ms"] / per,
                        "kernel_ms_mean": t["ev_mean"] / per, "kernel_ms_min": t["ev_min"] / per,
                        "GB/s": gbs, "frac": gbs / HBM_PEAK_GBS, "dtype": dtype,
                        "algorithmic_bytes": nbytes // per,
                        "settle_launches": t["settle_launches"], "settled": t["settled"],
                        "kernel_ms_unsettled_first25": (t["unsettled_first_ms"] / per) if t["unsettled_first_ms"] else None}
        if traffic is not None:
            others[name]["traffic"] = traffic
            others[name]["traffic_source"] = tnote
        return others[name]

    # ---------------------------------------------------------------- workload table
    # Arrays of the further workloads are views of / conversions from the headline's
    # seeded arrays (values do not change a streaming kernel's speed).
    lazy = {}

    def get(key, make):
        if key not in lazy:
            lazy[key] = make()
        return lazy[key]

    def upb():
        return get("upb", lambda: torch.from_numpy(
            inputs.config_inputs("wave3d_r4", shape=shape, fields=("u_prev_bar",))["u_prev_bar"]).to(dev))

    def rbuf():
        return get("r", lambda: torch.empty_like(ub))

    def r2d():
        return get("r2d", lambda: rbuf().reshape(-1)[: s2[0] * s2[1]].reshape(s2))

    def f32set():
        return get("f32", lambda: (c.float(), rb.float(), ub.float()))

    s2 = (args.size2d, args.size2d)
    if s2[0] * s2[1] > N or s2[0] < 3:
        print("bench.py: --size2d %d does not fit the %d^3 arrays" % (args.size2d, n), file=sys.stderr)
        sys.exit(2)
    nb = 1 << 24
    n1 = 4096

    def views2d():
        return get("v2d", lambda: tuple(t.reshape(-1)[: s2[0] * s2[1]].reshape(s2) for t in (c, rb, ub)))

    def views1d():
        return get("v1d", lambda: tuple(t.reshape(-1)[:n1] for t in (c, rb, ub)))

    burg_state = {"i": 0}

    def burg_sets():
        # three rotating buffer sets so that the 128 MiB arrays do not stay in the 256 MB last-level cache
        return get("burg", lambda: [tuple(t.reshape(-1)[k * nb:(k + 1) * nb] for t in (rb, c, ub)) for k in range(3)])

    def burg_adj():
        u_, r_, b_ = burg_sets()[burg_state["i"] % 3]
        burg_state["i"] += 1
        sadj.sadj_adjoint_burgers1d(0.1, 0.05, u_, r_, b_)

    def burg_pri():
        u_, r_, b_ = burg_sets()[burg_state["i"] % 3]
        burg_state["i"] += 1
        sadj.sadj_primal_burgers1d(0.1, 0.05, u_, b_)

    I4, I1 = interior_points(shape, 4), interior_points(shape, 1)
    table = {
        # the benchmark definition's five configurations and the forms the paper differentiates
        "wave3d_r4_f32_adjoint": lambda: add("wave3d_r4_f32_adjoint", lambda: sadj.sadj_adjoint_wave3d(R, *f32set()), N,
                                             wave_adjoint_bytes(shape, R, 4), "f32"),
        "wave3d_r4_f64_adjoint_with_u_prev_bar": lambda: add(
            "wave3d_r4_f64_adjoint_with_u_prev_bar", lambda: sadj.sadj_adjoint_wave3d(R, c, rb, ub, upb()), N,
            wave_adjoint_bytes(shape, R, 8, True), "f64"),
        "wave3d_r4_f64_primal": lambda: add("wave3d_r4_f64_primal", lambda: sadj.sadj_primal_wave3d(R, ub, upb(), c, rbuf()),
                                            N, 8 * N + 24 * I4, "f64"),
        "wave3d_r1_f64_adjoint": lambda: add("wave3d_r1_f64_adjoint", lambda: sadj.sadj_adjoint_wave3d(1, c, rb, ub), N,
                                             wave_adjoint_bytes(shape, 1, 8), "f64"),
        "wave3d_r1_f64_adjoint_with_u_prev_bar": lambda: add(
            "wave3d_r1_f64_adjoint_with_u_prev_bar", lambda: sadj.sadj_adjoint_wave3d(1, c, rb, ub, upb()), N,
            wave_adjoint_bytes(shape, 1, 8, True), "f64"),
        "wave2d_f64_adjoint": lambda: add("wave2d_f64_adjoint", lambda: sadj.sadj_adjoint_wave2d(*views2d()),
                                          s2[0] * s2[1], wave_adjoint_bytes(s2, 1, 8), "f64"),
        "burgers1d_f64_adjoint": lambda: add("burgers1d_f64_adjoint", burg_adj, nb, 32 * nb, "f64"),
        "wave1d_f64_adjoint_n4096_latency": lambda: add(
            "wave1d_f64_adjoint_n4096_latency",
            lambda: sadj.sadj_adjoint_wave1d(*views1d()), n1, 32 * n1, "f64"),
    }
    default_names = list(table)

    def more():
        wbox = [[[0.1 * (i + 3 * j + 9 * k) - 1.0 for i in range(3)] for j in range(3)] for k in range(3)]
        wbox2 = [[0.1 * (i + 3 * j) - 0.4 for i in range(3)] for j in range(3)]
        wstar = [0.3] + [0.05 * (i % 7) - 0.12 for i in range(24)]
        ksteps = 6
        t = {
            # reverse sweep of a time loop: per step read c and lam_a on I, read+write lam_b, write lam_p
            "wave3d_r4_f64_adjoint_steps_per_step": lambda: add(
                "wave3d_r4_f64_adjoint_steps_per_step", lambda: sadj.sadj_adjoint_wave3d_steps(R, ksteps, c, rb, ub, upb()),
                N * ksteps, ksteps * (16 * I4 + 16 * N + 8 * N), "f64", per=ksteps),
            "wave3d_r1_f64_primal": lambda: add("wave3d_r1_f64_primal", lambda: sadj.sadj_primal_wave3d(1, ub, upb(), c, rbuf()),
                                                N, 8 * N + 24 * I1, "f64"),
            "wave3d_r2_f64_adjoint": lambda: add("wave3d_r2_f64_adjoint", lambda: sadj.sadj_adjoint_wave3d(2, c, rb, ub), N,
                                                 wave_adjoint_bytes(shape, 2, 8), "f64"),
            "wave3d_r3_f64_adjoint": lambda: add("wave3d_r3_f64_adjoint", lambda: sadj.sadj_adjoint_wave3d(3, c, rb, ub), N,
                                                 wave_adjoint_bytes(shape, 3, 8), "f64"),
            # dense 3x3x3 box stencil with asymmetric weights (27 terms), same grid
            "box3d_f64_adjoint": lambda: add("box3d_f64_adjoint", lambda: sadj.sadj_adjoint_box(wbox, c, rb, ub), N,
                                             wave_adjoint_bytes(shape, 1, 8), "f64"),
            "box3d_f64_primal": lambda: add("box3d_f64_primal", lambda: sadj.sadj_primal_box(wbox, ub, c, rbuf()), N,
                                            8 * N + 16 * I1, "f64"),
            # general star of radius 4 with an asymmetric weight table (25 free weights)
            "star3d_r4_f64_adjoint": lambda: add("star3d_r4_f64_adjoint", lambda: sadj.sadj_adjoint_star3d(4, wstar, c, rb, ub),
                                                 N, wave_adjoint_bytes(shape, 4, 8), "f64"),
            "star3d_r4_f64_primal": lambda: add("star3d_r4_f64_primal", lambda: sadj.sadj_primal_star3d(4, wstar, ub, c, rbuf()),
                                                N, 8 * N + 16 * I4, "f64"),
            "star3d_r1_f64_adjoint": lambda: add("star3d_r1_f64_adjoint", lambda: sadj.sadj_adjoint_star3d(1, wstar[:7], c, rb, ub),
                                                 N, wave_adjoint_bytes(shape, 1, 8), "f64"),
            "star3d_r1_f64_primal": lambda: add("star3d_r1_f64_primal", lambda: sadj.sadj_primal_star3d(1, wstar[:7], ub, c, rbuf()),
                                                N, 8 * N + 16 * I1, "f64"),
            "wave2d_f64_primal": lambda: add(
                "wave2d_f64_primal",
                lambda: sadj.sadj_primal_wave2d(views2d()[2], views2d()[1], views2d()[0], r2d()),
                s2[0] * s2[1], 8 * s2[0] * s2[1] + 24 * interior_points(s2, 1), "f64"),
            "box2d_f64_adjoint": lambda: add("box2d_f64_adjoint", lambda: sadj.sadj_adjoint_box(wbox2, *views2d()),
                                             s2[0] * s2[1], wave_adjoint_bytes(s2, 1, 8), "f64"),
            "burgers1d_f64_primal": lambda: add("burgers1d_f64_primal", burg_pri, nb, 16 * nb, "f64"),
        }
        return t

    if args.all or (args.only and args.only not in table and args.only != HEADLINE):
        table.update(more())

    def burgers_steps_leg():
        # Reverse sweep over stored Burgers states.  Step by step: per step read u^t and lam, write
        # lam (24 B/pt; the first step accumulates: 32).  The same 24 B/pt are the yardstick for the
        # fused sweep (runs of five assigned steps per pass: lam read and written once per five
        # states), whose fraction may therefore exceed what one pass per step could reach.
        ks = 16
        states = torch.rand(ks + 1, nb, device=dev, dtype=torch.float64) - 0.5
        la, lb = torch.rand(nb, device=dev, dtype=torch.float64), torch.zeros(nb, device=dev, dtype=torch.float64)
        per_step_bytes = 32 * nb + (ks - 1) * 24 * nb
        sadj.set_option("burgers1d.fuse", 1)
        add("burgers1d_f64_adjoint_steps_per_step", lambda: sadj.sadj_adjoint_burgers1d_steps(0.1, 0.05, ks, ks, states, la, lb),
            nb * ks, per_step_bytes, "f64", per=ks)
        sadj.set_option("burgers1d.fuse", 0)
        o = add("burgers1d_f64_adjoint_steps_fused_per_step",
                lambda: sadj.sadj_adjoint_burgers1d_steps(0.1, 0.05, ks, ks, states, la, lb), nb * ks, per_step_bytes, "f64", per=ks)
        o["note"] = ("fraction is against the step-by-step compulsory bytes (24 B/pt/step); the fused passes themselves move "
                     "(16 + 8*5)/5 = 11.2 B/pt/step plus 6.7 % recomputed window overlap")

    # reverse sweep of a time loop of 7-point wave steps, 25 steps per call: one kernel per step, or with
    # pairs of steps fused (step 0 alone, then 12 pairs); both priced at the step-by-step bytes
    wave_ks = 25
    wave_step_bytes = 16 * I1 + 24 * N

    def wave_steps_leg():
        add("wave3d_r1_f64_adjoint_steps_per_step", lambda: sadj.sadj_adjoint_wave3d_steps(1, wave_ks, c, rb, ub, upb()),
            N * wave_ks, wave_ks * wave_step_bytes, "f64", per=wave_ks)

    def wave_steps_fused_leg():
        work = get("work", lambda: torch.empty_like(c))
        o = add("wave3d_r1_f64_adjoint_steps_fused_per_step",
                lambda: sadj.sadj_adjoint_wave3d_steps_fused(1, wave_ks, c, rb, ub, upb(), work), N * wave_ks,
                wave_ks * wave_step_bytes, "f64", per=wave_ks)
        o["kernel_algorithmic_bytes"] = 24 * I1 + 16 * N
        if "traffic" in o:                       # the recorded counters are those of one launch of the pair kernel
            o["kernel_traffic"] = o.pop("traffic")
        o["note"] = ("fraction is against the step-by-step compulsory bytes (40 B/pt/step); a call is one single step and 12 "
                     "launches of the pair kernel, each of which moves kernel_algorithmic_bytes for two steps "
                     "(a, b, c read on I, two results written)")

    def functor_leg():
        sadj.set_option("stencil1d.functor", 1)      # same stencil through the generic functor kernel
        add("burgers1d_f64_adjoint_functor", burg_adj, nb, 32 * nb, "f64")
        sadj.set_option("stencil1d.functor", 0)

    def graph_leg():
        # the n = 4096 call recorded 100 times into a HIP graph: the launch-bound size without host launch cost
        c1, rb1, ub1 = views1d()
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
        add("wave1d_f64_adjoint_n4096_in_hip_graph_per_call", graph.replay, n1 * per_graph, 32 * n1 * per_graph, "f64",
            per=per_graph)

    def star_functor_leg(name, fn, nbytes):
        # the same 7-point star through the generic functor kernels (include/sadj_stencil_star.hpp)
        def leg():
            sadj.set_option("star3d.functor", 1)
            try:
                add(name, fn, N, nbytes, "f64")
            finally:
                sadj.set_option("star3d.functor", 0)
        return leg

    w7 = [0.3] + [0.05 * (i % 7) - 0.12 for i in range(6)]
    if args.all or args.only in ("star3d_r1_f64_adjoint_functor", "star3d_r1_f64_primal_functor"):
        table["star3d_r1_f64_adjoint_functor"] = star_functor_leg(
            "star3d_r1_f64_adjoint_functor", lambda: sadj.sadj_adjoint_star3d(1, w7, c, rb, ub), wave_adjoint_bytes(shape, 1, 8))
        table["star3d_r1_f64_primal_functor"] = star_functor_leg(
            "star3d_r1_f64_primal_functor", lambda: sadj.sadj_primal_star3d(1, w7, ub, c, rbuf()), 8 * N + 16 * I1)
    if args.all or args.only in ("burgers1d_f64_adjoint_steps_per_step", "burgers1d_f64_adjoint_steps_fused_per_step"):
        table["burgers1d_f64_adjoint_steps_per_step"] = burgers_steps_leg
        table["burgers1d_f64_adjoint_steps_fused_per_step"] = burgers_steps_leg
    table["wave3d_r1_f64_adjoint_steps_per_step"] = wave_steps_leg
    table["wave3d_r1_f64_adjoint_steps_fused_per_step"] = wave_steps_fused_leg
    default_names += ["wave3d_r1_f64_adjoint_steps_per_step", "wave3d_r1_f64_adjoint_steps_fused_per_step"]
    if args.all:
        del table["burgers1d_f64_adjoint_steps_fused_per_step"]
        table["burgers1d_f64_adjoint_functor"] = functor_leg
        table["wave1d_f64_adjoint_n4096_in_hip_graph_per_call"] = graph_leg

    # ---------------------------------------------------------------- headline
    out = {"metric": METRIC, "unit": "Gpoints/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
           "size": n, "size2d": args.size2d}
    props = torch.cuda.get_device_properties(dev)
    out["device"] = {"name": props.name, "compute_units": props.multi_processor_count,
                     "memory_GiB": round(props.total_memory / 2 ** 30, 1), "library": sadj.version()}
    if args.only is None or args.only == HEADLINE:
        t = timer.time_calls(lambda: sadj.sadj_adjoint_wave3d(R, c, rb, ub), args.steps, args.warmup)
        alg_bytes = wave_adjoint_bytes(shape, R, 8)
        achieved = alg_bytes / (t["ev_mean"] * 1e-3) / 1e9
        traffic, tnote = read_traffic(HEADLINE) if n == 512 else (None, "recorded for 512^3 only")
        out.update({
            "value": N / (t["wall_ms"] * 1e-3) / 1e9,
            "ms_per_step": t["wall_ms"],
            "config": {"workload": "wave3d adjoint, 25-point star r=4, %d^3, fp64, u_bar only" % n,
                       "variant": sadj.get_option("wave3d.variant"),
                       "zchunk": sadj.get_option("wave3d.zchunk")},
            "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": tnote,
                         "kernel_ms_mean": t["ev_mean"], "kernel_ms_min": t["ev_min"], "algorithmic_bytes": alg_bytes},
            "settle": {"launches": t["settle_launches"], "settled": t["settled"], "cap": args.settle_cap,
                       "kernel_ms_unsettled_first25": t["unsettled_first_ms"],
                       "rule": "groups of 10 launches until the times of a group agree within 1 % (slowest and fastest "
                               "set aside) and the group mean is within 1 % of the previous group's; then the W warm-up "
                               "and K timed steps as flagged",
                       "why": "after a load step from idle the shader clock drops from 2.43 to about 1.5 GHz for some "
                              "20 ms (memory clock unchanged); the first launches of a process run up to 20 % slower"},
        })
    else:
        out.update({"value": None, "ms_per_step": None, "config": {"workload": "only " + args.only}})

    # the paper's own timings of the same method (Section 4, performance tables), with their
    # hardware: context only, another machine, another stencil radius and grid; `--paper-sizes`
    # times these two workloads here
    out["paper_context"] = {
        "wave_7pt_1000^3_gather_adjoint_best_s": {"Xeon E5-2650 v4, 12 threads": 1.322396, "Xeon Phi 7210, 64 threads": 1.286821},
        "wave_7pt_1000^3_primal_best_s": {"Xeon E5-2650 v4, 12 threads": 0.897188, "Xeon Phi 7210, 32 threads": 0.843320},
        "burgers_1e9_gather_adjoint_best_s": {"Xeon E5-2650 v4, 12 threads": 1.535777, "Xeon Phi 7210, 128 threads": 0.756979},
        "burgers_1e9_primal_best_s": {"Xeon E5-2650 v4, 12 threads": 0.555659, "Xeon Phi 7210, 128 threads": 0.502064},
    }

    # ---------------------------------------------------------------- streaming ceiling
    def stream_ceiling(dtype_name):
        a_, b_, o_ = ((c, rb, ub) if dtype_name == "f64" else f32set())
        a_, b_, o_ = (t.reshape(-1) for t in (a_, b_, o_))
        esize = 8 if dtype_name == "f64" else 4
        best = None
        for shp in (0, 1, 2):
            t = timer.time_calls(lambda: sadj.sadj_stream_probe(shp, a_, b_, o_), steps_o, warm_o)
            gbs = 4 * esize * N / (t["ev_mean"] * 1e-3) / 1e9
            if best is None or gbs > best["GB/s"]:
                best = {"GB/s": gbs, "kernel_ms_mean": t["ev_mean"], "shape": shp, "bytes": 4 * esize * N,
                        "what": "out[i] += a[i]*b[i] over the same %d^3 %s arrays (sadj_stream_probe), best of three launch shapes"
                                % (n, dtype_name)}
        return best

    if args.only is None:
        sc = stream_ceiling("f64")
        out["roofline"]["stream_ceiling"] = sc
        out["roofline"]["frac_of_ceiling"] = out["roofline"]["achieved"] / sc["GB/s"]
        names = list(table) if args.all else default_names
        for name in names:
            table[name]()
            if name == "wave3d_r4_f32_adjoint":
                sc32 = stream_ceiling("f32")
                others[name]["stream_ceiling"] = sc32
                others[name]["frac_of_ceiling"] = others[name]["GB/s"] / sc32["GB/s"]
                lazy.pop("f32", None)
        for name, o in others.items():
            if o["dtype"] == "f64" and "latency" not in name and "graph" not in name:
                o["frac_of_ceiling"] = o["GB/s"] / sc["GB/s"]
    elif args.only != HEADLINE:
        if args.only not in table:
            print("bench.py: unknown workload %r; known: %s" % (args.only, ", ".join([HEADLINE] + sorted(table))), file=sys.stderr)
            sys.exit(2)
        table[args.only]()

    if args.remainder_study:
        # Section 3.3.4's alternatives on the GPU: 0 guarded only where needed (default),
        # 1 guarded everywhere ("zero padding"), 2 core and remainder as separate dispatches
        for rad in (4, 3, 2, 1):
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

    lazy.clear()
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
        # reverse sweep of a time loop of such steps (the paper notes that solvers take many, Section 4): 25 steps per
        # call, one kernel per step, then with pairs of steps fused (step 0 alone, then 12 pairs)
        a4 = torch.empty_like(a1)
        ks3, step3 = 25, 16 * interior_points(s3, 1) + 24 * N3
        add("paper_wave3d_7pt_1000^3_f64_adjoint_steps_per_step", lambda: sadj.sadj_adjoint_wave3d_steps(1, ks3, cw, a1, a2, a3),
            N3 * ks3, ks3 * step3, "f64", per=ks3)
        add("paper_wave3d_7pt_1000^3_f64_adjoint_steps_fused_per_step",
            lambda: sadj.sadj_adjoint_wave3d_steps_fused(1, ks3, cw, a1, a2, a3, a4), N3 * ks3, ks3 * step3, "f64", per=ks3)
        del a4
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
        src = torch.ones(1 << 27, device=dev, dtype=torch.float64)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                   # exactly 1 GiB read and 1 GiB written
        torch.cuda.synchronize()

    if not args.no_cpu_baseline and args.only is None:
        import oracle
        oracle.build()

        def run_oracle(nzs):
            sl = (slice(0, nzs),)
            t0 = time.perf_counter()
            oracle.wave_adjoint(d["c"][sl], d["r_bar"][sl], d["u_bar"][sl], R)
            return time.perf_counter() - t0

        probe = min(n, 32)
        rate = probe / run_oracle(probe)                 # planes per second on this host
        nzs = int(min(n, max(probe, rate * 8.0)))       # about 8 s of CPU work per run, at most the whole grid
        runs = sorted(run_oracle(nzs) for _ in range(3))
        dt = runs[1]
        out["cpu_baseline"] = {"value": nzs * n * n / dt / 1e9, "unit": "Gpoints/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d z-planes of the same %d^3 arrays (%d x %d x %d grid), median of 3 runs "
                                         "(%.1f / %.1f / %.1f s)" % (nzs, n, n, n, nzs, runs[0], runs[1], runs[2]),
                               "host_cpus": os.cpu_count(), "host_cpu_model": cpu_model()}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
