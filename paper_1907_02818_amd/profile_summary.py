"""Turn rocprofv3 output of `bench.py --only WORKLOAD` runs into the short text summaries
kept under profiles/.

    python -m paper_1907_02818_amd.profile_summary WORKLOAD DIR

DIR holds what three rocprofv3 runs of the same workload wrote (csv output, `-o p`):

    DIR/stats/   rocprofv3 --kernel-trace --stats -d DIR/stats -o p --output-format csv -- \
                     python3 bench.py --only WORKLOAD --steps 50 --warmup 5 --no-cpu-baseline
    DIR/fetch/   rocprofv3 --pmc FETCH_SIZE --kernel-trace -d DIR/fetch -o p --output-format csv -- \
                     python3 bench.py --only WORKLOAD --steps 5 --warmup 2 --settle-cap 0 --no-cpu-baseline --copy-probe
    DIR/write/   the same with WRITE_SIZE
    DIR/stats.json   stdout of the first run (bench.py's JSON line: algorithmic bytes of the workload)

and, optionally, DIR/sq/ from a run with SQ_* counters.  With `--all DIR` instead of a workload
it writes profiles/all_workloads_stats.txt from DIR/stats/ and DIR/stats.json of a
`bench.py --all --remainder-study` run under rocprofv3 --kernel-trace --stats.  Writes profiles/WORKLOAD_stats.txt
and profiles/WORKLOAD_pmc.txt.  The counters are calibrated on the run's last dispatch, the
plain device copy of one 1 GiB array that `--copy-probe` appends (2^30 bytes read, 2^30
written).  The pmc summary records a hash of the kernel sources, so that bench.py reports its
traffic figure only for a library built from the same sources.

This module only reads files; it starts no profiler and no GPU work.
"""
from __future__ import annotations

import csv
import glob
import hashlib
import json
import os
import statistics
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
GIB = 1 << 30


def library_sources_sha256() -> str:
    """Hash of the kernel sources and headers libsadj.so is built from."""
    h = hashlib.sha256()
    files = []
    for d in (os.path.join(HERE, "csrc"), os.path.join(ROOT, "include")):
        for name in sorted(os.listdir(d)):
            if name.endswith((".hip", ".hpp")):          # kernel sources; sadj.h holds declarations only
                files.append(os.path.join(d, name))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def _rows(pattern):
    files = sorted(glob.glob(pattern, recursive=True))
    if not files:
        raise FileNotFoundError(pattern)
    with open(files[0], newline="") as fh:
        return list(csv.DictReader(fh))


def _short(name):
    return name.split("(")[0].replace("void ", "")


def _is_ours(name):
    return "sadj::" in name


def _bench_json(path):
    with open(path) as fh:
        for ln in reversed(fh.read().splitlines()):
            ln = ln.strip()
            if ln.startswith("{"):
                return json.loads(ln)
    raise ValueError("no JSON line in " + path)


def _workload_figures(js, workload):
    if workload in js.get("others", {}):
        o = js["others"][workload]
        if "kernel_algorithmic_bytes" in o:          # a call launches several kernels: bytes of the dominant kernel's launch
            return int(o["kernel_algorithmic_bytes"]), None, o.get("settle_launches")
        return int(o["algorithmic_bytes"]), o["kernel_ms_mean"], o.get("settle_launches")
    r = js["roofline"]
    return int(r["algorithmic_bytes"]), r["kernel_ms_mean"], js.get("settle", {}).get("launches")


def summarise(workload, d):
    js = _bench_json(os.path.join(d, "stats.json"))
    alg, bench_ms, settle = _workload_figures(js, workload)
    steps, warmup = js["steps"], js["warmup"]
    if workload in js.get("others", {}):            # bench.py times the further workloads with a quarter of the steps
        steps, warmup = max(5, steps // 4), max(3, warmup // 4)
    flag_steps, flag_warmup = js["steps"], js["warmup"]
    only = ("--only %s " % workload + ("--size %d " % js["size"] if js.get("size", 512) != 512 else "")
            + ("--size2d %d " % js["size2d"] if js.get("size2d", 8192) != 8192 else ""))
    cmd_stats = ("rocprofv3 --kernel-trace --stats -d DIR/stats -o p --output-format csv -- python3 bench.py "
                 + only + "--steps %d --warmup %d --no-cpu-baseline" % (flag_steps, flag_warmup))
    cmd_pmc = ("rocprofv3 --pmc %s --kernel-trace -d DIR/%s -o p --output-format csv -- python3 bench.py "
               + only + "--steps 5 --warmup 2 --settle-cap 0 --no-cpu-baseline --copy-probe")

    # ---- kernel trace: the library kernel with the largest total time is the workload's kernel
    trace = _rows(os.path.join(d, "stats", "**", "*kernel_trace.csv"))
    per = {}
    for r in trace:
        if _is_ours(r["Kernel_Name"]):
            per.setdefault(r["Kernel_Name"], []).append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r))
    if not per:
        raise ValueError("no libsadj kernel in the trace")
    kname = max(per, key=lambda k: sum(e - s for s, e, _ in per[k]))
    launches = sorted(per[kname])
    dur = [(e - s) / 1e3 for s, e, _ in launches]
    timed = dur[-steps:] if len(dur) >= steps else dur
    first = launches[0][2]
    lines = ["rocprofv3 kernel-trace summary: bench.py workload %s" % workload,
             "command (from the repository root, on one MI355X; DIR is any scratch directory):",
             "  " + cmd_stats, "",
             "kernel: %s" % _short(kname),
             "workgroups %d x %s threads, LDS %s B per workgroup, %s VGPRs" % (
                 int(first["Grid_Size_X"]) // max(1, int(first["Workgroup_Size_X"])), first["Workgroup_Size_X"],
                 first["LDS_Block_Size"], first.get("VGPR_Count", "?")),
             "launches in the run: %d (one untimed first call where the workload is not the headline, settle phase %s, "
             "warm-up %d, timed %d; one kernel per call unless noted)" % (len(dur), settle, warmup, steps),
             "all launches:        avg %.1f us, min %.1f us, max %.1f us" % (statistics.mean(dur), min(dur), max(dur)),
             "first 25 launches:   avg %.1f us (shader clock still settling after the load step)" % statistics.mean(dur[:25]),
             "the %d timed launches: avg %.1f us, min %.1f us, max %.1f us" % (
                 len(timed), statistics.mean(timed), min(timed), max(timed)),
             ("bench.py's own HIP-event mean for the same launches: %.1f us" % (bench_ms * 1e3)) if bench_ms is not None else
             "(a call of this workload launches several kernels; bench.py times calls, this summary the dominant kernel)",
             "algorithmic bytes per launch: %d" % alg,
             "=> achieved %.0f GB/s = %.1f %% of 8000 GB/s (timed launches)" % (
                 alg / statistics.mean(timed) / 1e3, alg / statistics.mean(timed) / 1e3 / 80), ""]
    stats = _rows(os.path.join(d, "stats", "**", "*kernel_stats.csv"))
    lines.append("%-86s %6s %10s %10s %10s %7s" % ("rocprofv3 --stats, top kernels", "calls", "avg_us", "min_us", "max_us", "pct"))
    for r in stats[:5]:
        lines.append("%-86s %6s %10.1f %10.1f %10.1f %7s" % (_short(r["Name"])[:86], r["Calls"], float(r["AverageNs"]) / 1e3,
                                                               float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, r["Percentage"]))
    stats_txt = "\n".join(lines) + "\n"

    # ---- counters
    def pmc(sub, ctr):
        rs = _rows(os.path.join(d, sub, "**", "*counter_collection.csv"))
        k = [float(r["Counter_Value"]) for r in rs if r["Kernel_Name"] == kname and r["Counter_Name"] == ctr]
        cp = [float(r["Counter_Value"]) for r in rs if "copyBuffer" in r["Kernel_Name"] and r["Counter_Name"] == ctr]
        if not k or not cp:
            raise ValueError("counter %s: kernel or calibration copy missing in %s" % (ctr, sub))
        return k, cp[-1]

    fk, fcopy = pmc("fetch", "FETCH_SIZE")
    wk, wcopy = pmc("write", "WRITE_SIZE")
    fscale, wscale = (GIB / 1024) / fcopy, (GIB / 1024) / wcopy      # true KiB per counter unit
    fbytes = statistics.mean(fk) * fscale * 1024
    wbytes = statistics.mean(wk) * wscale * 1024
    sha = library_sources_sha256()
    lines = ["rocprofv3 --pmc summary: HBM-side traffic of bench.py workload %s" % workload,
             "commands (one counter per run; DIR is any scratch directory):",
             "  " + cmd_pmc % ("FETCH_SIZE", "fetch"),
             "  " + cmd_pmc % ("WRITE_SIZE", "write"), "",
             "kernel: %s" % _short(kname),
             "calibration: the last dispatch of each run is a plain device copy of one 512^3 fp64 array (1 GiB read, 1 GiB written)",
             "  FETCH_SIZE of the copy: %.1f  -> scale %.4f (true KiB per counter unit)" % (fcopy, fscale),
             "  WRITE_SIZE of the copy: %.1f  -> scale %.4f" % (wcopy, wscale),
             "mean over %d / %d dispatches of the kernel:" % (len(fk), len(wk)),
             "  FETCH_SIZE %.1f  -> %.0f bytes read" % (statistics.mean(fk), fbytes),
             "  WRITE_SIZE %.1f  -> %.0f bytes written" % (statistics.mean(wk), wbytes),
             "  total %.0f bytes per launch = %.3f x the algorithmic %d bytes" % (fbytes + wbytes, (fbytes + wbytes) / alg, alg),
             "traffic_bytes_per_launch: %.0f" % (fbytes + wbytes),
             "library_sources_sha256: %s" % sha]
    sq_dir = os.path.join(d, "sq")
    if os.path.isdir(sq_dir):
        acc = {}
        for r in _rows(os.path.join(sq_dir, "**", "*counter_collection.csv")):
            if r["Kernel_Name"] == kname:
                acc.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
        if acc:
            m = {k: statistics.mean(v) for k, v in acc.items()}
            lines += ["", "further counters of the same kernel (a run of its own, mean per dispatch):",
                      "  rocprofv3 --pmc " + " ".join(sorted(m)) + " --kernel-trace -d DIR/sq -o p --output-format csv -- python3 bench.py "
                      + only + "--steps 5 --warmup 2 --settle-cap 0 --no-cpu-baseline",
                      "  " + ", ".join("%s %.4g" % (k, v) for k, v in sorted(m.items()))]
            if m.get("SQ_WAVE_CYCLES") and "SQ_WAIT_INST_ANY" in m:
                lines.append("  wave-cycles spent waiting for an instruction to complete: %.0f %%"
                             % (100 * m["SQ_WAIT_INST_ANY"] / m["SQ_WAVE_CYCLES"]))
            if m.get("SQ_ACTIVE_INST_LDS") and "SQ_LDS_BANK_CONFLICT" in m:
                lines.append("  LDS bank-conflict cycles per active LDS cycle: %.3f"
                             % (m["SQ_LDS_BANK_CONFLICT"] / m["SQ_ACTIVE_INST_LDS"]))
            if m.get("SQ_INSTS_VALU") and m.get("SQ_INSTS_LDS"):
                lines.append("  vector ALU instructions per LDS instruction: %.1f" % (m["SQ_INSTS_VALU"] / m["SQ_INSTS_LDS"]))
    pmc_txt = "\n".join(lines) + "\n"
    return stats_txt, pmc_txt


def summarise_all(d):
    """Summary of a `bench.py --all --remainder-study` run under rocprofv3 --kernel-trace --stats:
    DIR/stats/ (csv) and DIR/stats.json (bench.py's JSON line)."""
    js = _bench_json(os.path.join(d, "stats.json"))
    lines = ["rocprofv3 kernel-trace summary of every benchmark workload, one MI355X",
             "command (from the repository root; DIR is any scratch directory):",
             "  rocprofv3 --kernel-trace --stats -d DIR/stats -o p --output-format csv -- python3 bench.py --all "
             "--remainder-study --steps %d --warmup %d --no-cpu-baseline" % (js["steps"], js["warmup"]), "",
             "bench.py's figures (HIP-event mean of the timed calls after the settle phase; fraction of 8000 GB/s on",
             "algorithmic bytes; per step where a call performs several steps):", "",
             "%-52s %10s %9s %8s" % ("workload", "ms", "GB/s", "% peak")]
    rows = [(HEADLINE, js["roofline"]["kernel_ms_mean"], js["roofline"]["achieved"], js["roofline"]["frac"])]
    rows += [(k, v["kernel_ms_mean"], v["GB/s"], v["frac"]) for k, v in js["others"].items()]
    for k, ms, gbs, frac in rows:
        lines.append("%-52s %10.4f %9.0f %8.1f" % (k, ms, gbs, 100 * frac))
    sc = js["roofline"].get("stream_ceiling")
    if sc:
        lines.append("%-52s %10.4f %9.0f %8.1f" % ("streaming ceiling (out += a*b, same arrays)", sc["kernel_ms_mean"], sc["GB/s"], sc["GB/s"] / 80))
    stats = _rows(os.path.join(d, "stats", "**", "*kernel_stats.csv"))
    lines += ["", "rocprofv3 --stats, library kernels (avg over ALL launches of a kernel, settle and warm-up included):", "",
              "%-100s %6s %10s %10s" % ("kernel", "calls", "avg_us", "min_us")]
    for r in stats:
        if _is_ours(r["Name"]):
            lines.append("%-100s %6s %10.1f %10.1f" % (_short(r["Name"])[:100], r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3))
    return "\n".join(lines) + "\n"


HEADLINE = "wave3d_r4_f64_adjoint"


def main(argv):
    if len(argv) == 3 and argv[1] == "--all":
        txt = summarise_all(argv[2])
        with open(os.path.join(ROOT, "profiles", "all_workloads_stats.txt"), "w") as fh:
            fh.write(txt)
        sys.stdout.write(txt)
        return 0
    if len(argv) != 3:
        print(__doc__, file=sys.stderr)
        return 2
    workload, d = argv[1], argv[2]
    stats_txt, pmc_txt = summarise(workload, d)
    out = os.path.join(ROOT, "profiles")
    os.makedirs(out, exist_ok=True)
    js = _bench_json(os.path.join(d, "stats.json"))
    size, size2d = js.get("size", 512), js.get("size2d", 8192)
    if size != 512:
        workload += "_%d" % size                       # 3-D workloads at another grid edge (bench.py --size)
    if size2d != 8192 and "2d" in workload:
        workload += "_%d" % size2d                     # 2-D workloads at another grid edge (bench.py --size2d)
    with open(os.path.join(out, workload + "_stats.txt"), "w") as fh:
        fh.write(stats_txt)
    with open(os.path.join(out, workload + "_pmc.txt"), "w") as fh:
        fh.write(pmc_txt)
    sys.stdout.write(stats_txt + "\n" + pmc_txt)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
