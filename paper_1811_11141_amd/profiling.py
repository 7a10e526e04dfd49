"""rocprofv3 runs of bench.py and the short summaries under profiles/ made from them.

    python3 -m paper_1811_11141_amd.profiling run [all|traces|counters] [variant]
                                                         on the MI355X machine: the rocprofv3 runs below, raw
                                                         output under $MGWFBP_PROFILE_RAW (default
                                                         profile_raw/ in the repository)
    python3 -m paper_1811_11141_amd.profiling summarise  anywhere: that raw output -> profiles/*.md and
                                                         profiles/traffic.json (what bench.py reports
                                                         as roofline.traffic)

Two kinds of run, never combined: kernel traces (`--kernel-trace --stats`: per-kernel durations) and
counter runs (`--pmc FETCH_SIZE`, then `--pmc WRITE_SIZE`: HBM bytes per dispatch).  Every run
profiles `python3 bench.py ...` itself (the program comes straight after `--`).  The counter runs use
bench.py's --extras 1, which also launches the library's plain copy probe: its bytes are known, so
the same run calibrates the counters (FETCH_SIZE counts in units that need a factor, see the
summaries).
"""
from __future__ import annotations

import collections
import csv
import json
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
RAW = os.path.abspath(os.environ.get("MGWFBP_PROFILE_RAW", os.path.join(ROOT, "profile_raw")))
PROFILES = os.path.join(ROOT, "profiles")
QUIET = "--extras 0 --others 0 --cpu-baseline 0"

WORKLOADS = {   # tag -> (bench.py workload arguments, description, N, P)
    "resnet50_n8": ("", "ResNet-50-shaped gradient set, N = 8", 8, 25_557_032),
    "googlenet_n8": ("--workload googlenet", "GoogLeNet-shaped gradient set, N = 8", 8, 13_378_280),
    "vgg16_n16": ("--workload vgg16", "VGG-16-shaped gradient set, N = 16", 16, 138_357_544),
}
UNITS = {"fused": lambda n: n + 1, "step": lambda n: n + 5, "step_without_out": lambda n: n + 4,
         "pack": lambda n: 2 * n, "reduce": lambda n: n + 1, "unpack": lambda n: 2, "pack_reduce": lambda n: n + 1,
         "unpack_only": lambda n: 2, "unpack_update": lambda n: 6, "unpack_update_without_out": lambda n: 5,
         "gated_all_arrived": lambda n: n + 1}
# variant -> (summary file stem, regex of the kernel's name in rocprofv3's output)
KERNELS = {"fused": ("k_fused", r"k_fused<\d+, \d+, false"), "step": ("k_fused_update", r"k_fused<\d+, \d+, true"),
           "pack": ("k_pack", r"k_pack<"), "reduce": ("k_reduce", r"k_reduce<"), "unpack": ("k_unpack", r"k_unpack<false"),
           "unpack_update": ("k_unpack_update", r"k_unpack<true"),
           "gated_all_arrived": ("k_fused_gated", r"k_fused_gated<\d+, false")}
TRACES = [("resnet50_n8", v, 100) for v in ("fused", "step", "pack", "reduce", "unpack", "unpack_update",
                                            "gated_all_arrived")] + \
         [("googlenet_n8", v, 100) for v in ("fused", "step", "pack", "unpack", "unpack_update")] + \
         [("vgg16_n16", v, 30) for v in ("fused", "step")]
COUNTER_RUNS = [("resnet50_n8", 16), ("googlenet_n8", 16), ("vgg16_n16", 6)]


def bench_args(wl_tag: str, variant: str, steps: int) -> str:
    wl_args = WORKLOADS[wl_tag][0]
    return " ".join(x for x in (wl_args, f"--variant {variant}" if variant != "fused" else "",
                                f"--steps {steps} --warmup {max(3, steps // 10)}", QUIET) if x)


def counter_args(wl_tag: str, steps: int) -> str:
    # counters are collected one kernel at a time: the signal kernels of per_group_gated could not run beside
    # the launch that waits for them (it would give up), so that form is left out
    return " ".join(x for x in (WORKLOADS[wl_tag][0], f"--steps {steps} --warmup 3 --extras 1 --skip per_group_gated "
                                                      "--others 0 --cpu-baseline 0") if x)


def short(name: str) -> str:
    n = name.replace("void ", "").replace("mgwfbp::(anonymous namespace)::", "").split("(")[0]
    return n if len(n) < 90 else n[:87] + "..."


# ---- on the GPU machine --------------------------------------------------------------------------

def _rocprof(flags: list, out_dir: str, args: str, limit_s: int) -> None:
    os.makedirs(out_dir, exist_ok=True)
    cmd = ["rocprofv3", *flags, "-d", out_dir, "-o", "p", "--output-format", "csv", "--",
           "python3", os.path.join(ROOT, "bench.py"), *args.split()]
    print("[profiling]", " ".join(cmd), flush=True)
    env = dict(os.environ, TMPDIR="/tmp")
    with open(os.path.join(out_dir, "run.log"), "w") as log:
        res = subprocess.run(["timeout", "-s", "KILL", str(limit_s), *cmd], cwd="/tmp", env=env, stdout=log,
                             stderr=subprocess.STDOUT)
    if res.returncode != 0:
        raise SystemExit(f"rocprofv3 run failed ({res.returncode}): see {out_dir}/run.log")


def _find(out_dir: str, suffix: str) -> str:
    for base, _, files in os.walk(out_dir):
        for f in files:
            if f.endswith(suffix):
                return os.path.join(base, f)
    raise SystemExit(f"no *{suffix} under {out_dir}")


def _aggregate_counters(out_dir: str) -> None:
    """counter_collection.csv (one row per dispatch and counter) -> counters.csv (one row per kernel,
    grid size and counter: dispatches, average, minimum, maximum)."""
    agg = collections.defaultdict(list)
    with open(_find(out_dir, "counter_collection.csv")) as f:
        for r in csv.DictReader(f):
            agg[(r["Kernel_Name"], r["Grid_Size"], r["Counter_Name"])].append(float(r["Counter_Value"]))
    with open(os.path.join(out_dir, "counters.csv"), "w", newline="") as f:
        wr = csv.writer(f)
        wr.writerow(["Kernel_Name", "Grid_Size", "Counter_Name", "Dispatches", "Average", "Min", "Max"])
        for k, v in sorted(agg.items()):
            wr.writerow([*k, len(v), sum(v) / len(v), min(v), max(v)])


def _prune(out_dir: str) -> None:
    """Keep the small tables only: raw traces and databases stay on the box."""
    for base, _, files in os.walk(out_dir):
        for f in files:
            p = os.path.join(base, f)
            if f in ("counters.csv", "run.log", "bench_line.json") or f.endswith("kernel_stats.csv"):
                continue
            os.remove(p)


def run(part: str = "all", only: str = "") -> None:
    for wl_tag, variant, steps in (TRACES if part in ("all", "traces") else []):
        if only and variant != only:
            continue
        out = os.path.join(RAW, f"trace_{wl_tag}_{variant}")
        args = bench_args(wl_tag, variant, steps)
        # the unprofiled figure of the same command on the same box, for comparison
        res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args.split()], capture_output=True,
                             text=True, timeout=600)
        os.makedirs(out, exist_ok=True)
        with open(os.path.join(out, "bench_line.json"), "w") as f:
            f.write(([l for l in res.stdout.splitlines() if l.startswith("{")] or ["{}"])[-1])
        _rocprof(["--kernel-trace", "--stats"], out, args, 300)
        _find(out, "kernel_stats.csv")
        _prune(out)
        print(f"[profiling] trace {wl_tag} {variant} done", flush=True)
    for wl_tag, steps in (COUNTER_RUNS if part in ("all", "counters") else []):
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            out = os.path.join(RAW, f"pmc_{wl_tag}_{counter}")
            _rocprof(["--pmc", counter], out, counter_args(wl_tag, steps), 420)
            _aggregate_counters(out)
            _prune(out)
            print(f"[profiling] counters {wl_tag} {counter} done", flush=True)


# ---- anywhere ----------------------------------------------------------------------------------

def _trace_summary(wl_tag: str, variant: str, steps: int) -> None:
    out = os.path.join(RAW, f"trace_{wl_tag}_{variant}")
    _, desc, n, p = WORKLOADS[wl_tag]
    stem, pattern = KERNELS[variant]
    rows = list(csv.DictReader(open(_find(out, "kernel_stats.csv"))))
    alg = 4 * UNITS[variant](n) * p
    text = [f"# rocprofv3 kernel trace: {stem} ({variant}), {desc}, optimal plan, whole plan in one launch", "",
            "Command (from /tmp with TMPDIR=/tmp on the MI355X box; `python3 -m paper_1811_11141_amd.profiling run`",
            "issues it):", "",
            "    rocprofv3 --kernel-trace --stats -d <out> -o p --output-format csv -- \\",
            f"        python3 bench.py {bench_args(wl_tag, variant, steps)}", "",
            "p_kernel_stats.csv, top rows (ns):", "",
            "| kernel | calls | total | average | % | min | max | stddev |", "|---|---|---|---|---|---|---|---|"]
    main = None
    for r in rows[:5]:
        text.append(f"| {short(r['Name'])} | {r['Calls']} | {r['TotalDurationNs']} | {float(r['AverageNs']):.0f} | "
                    f"{r['Percentage']} | {r['MinNs']} | {r['MaxNs']} | {float(r['StdDev']):.0f} |")
    for r in rows:
        if re.search(pattern, r["Name"]) and (main is None or int(r["TotalDurationNs"]) > int(main["TotalDurationNs"])):
            main = r
    if main is None:
        raise SystemExit(f"{out}: no kernel matches {pattern}")
    avg, mn = float(main["AverageNs"]) / 1e3, float(main["MinNs"]) / 1e3
    kind = "Algorithmic" if variant in ("fused", "step", "gated_all_arrived") else "Actual"
    text += ["", f"{short(main['Name'])}: {main['Calls']} launches, average {avg:.1f} us, minimum {mn:.1f} us.",
             f"{kind} bytes per launch {alg:,} -> {alg / avg / 1e3:.0f} GB/s = {alg / avg / 1e3 / 80:.1f} % of 8 TB/s at the "
             f"average ({alg / mn / 1e3:.0f} GB/s = {alg / mn / 1e3 / 80:.1f} % at the minimum).", ""]
    try:
        line = json.load(open(os.path.join(out, "bench_line.json")))
        rf = line["roofline"]
        text += ["The same command without the profiler, just before, on the same box (bench.py, HIP-event brackets):",
                 f"{rf['kernel_avg_us']} us per launch on average, minimum {rf['kernel_min_us']} us, "
                 f"roofline.frac {rf['frac']}, whole-job value {line['value']} GB/s.", ""]
    except (OSError, ValueError, KeyError):
        pass
    with open(os.path.join(PROFILES, f"{stem}_{wl_tag}_kernel_trace.md"), "w") as f:
        f.write("\n".join(text))


def _counter_table(wl_tag: str, counter: str) -> dict:
    rows = list(csv.DictReader(open(os.path.join(RAW, f"pmc_{wl_tag}_{counter}", "counters.csv"))))
    return {(r["Kernel_Name"], int(r["Grid_Size"])): r for r in rows if r["Counter_Name"] == counter}


def _traffic_summary(wl_tag: str, steps: int) -> dict:
    _, desc, n, p = WORKLOADS[wl_tag]
    fetch, write = _counter_table(wl_tag, "FETCH_SIZE"), _counter_table(wl_tag, "WRITE_SIZE")

    def pick(pattern):          # whole-plan launches: the most frequent of the large grids that match
        keys = [k for k in fetch if re.search(pattern, k[0]) and k in write and k[1] >= 128 * 2048]
        return max(keys, key=lambda k: (int(fetch[k]["Dispatches"]), k[1])) if keys else None

    cal = pick(r"k_probe_copy")
    if cal is None:
        raise SystemExit(f"{wl_tag}: the counter runs hold no copy probe to calibrate with")
    n_probe = (n * p + 3) // 4 * 4
    f_scale = 4 * n_probe / (float(fetch[cal]["Average"]) * 1024)
    w_scale = 4 * n_probe / (float(write[cal]["Average"]) * 1024)
    text = [f"# HBM traffic per launch (rocprofv3 --pmc): every kernel of the path, {desc}", "",
            "Two counter runs, one counter each (from /tmp with TMPDIR=/tmp on the MI355X box;",
            "`python3 -m paper_1811_11141_amd.profiling run` issues them):", "",
            f"    rocprofv3 --pmc FETCH_SIZE -d <out> -o p --output-format csv -- python3 bench.py {counter_args(wl_tag, steps)}",
            f"    rocprofv3 --pmc WRITE_SIZE -d <out> -o p --output-format csv -- python3 bench.py {counter_args(wl_tag, steps)}", "",
            "`--extras 1` runs every form of the path and the library's plain copy probe, whose bytes are known.",
            "Per dispatch, KiB as the counters report them (average; minimum and maximum where one kernel runs",
            "with and without writing out[]):", "",
            "| kernel (grid size) | dispatches | FETCH_SIZE avg | min | max | WRITE_SIZE avg | min | max |",
            "|---|---|---|---|---|---|---|---|"]
    for k in sorted(fetch):
        if "mgwfbp" in k[0] and k in write and "k_spin" not in k[0] and int(fetch[k]["Dispatches"]) >= 3 and k[1] >= 128 * 2048:
            f_, w_ = fetch[k], write[k]
            text.append(f"| {short(k[0])} ({k[1]}) | {f_['Dispatches']} | {float(f_['Average']):.1f} | {float(f_['Min']):.1f} | "
                        f"{float(f_['Max']):.1f} | {float(w_['Average']):.1f} | {float(w_['Min']):.1f} | {float(w_['Max']):.1f} |")
    text += ["", f"Calibration: the copy probe reads and writes {4 * n_probe:,} B per launch; FETCH_SIZE reports "
                 f"{float(fetch[cal]['Average']) * 1024:,.0f} B (factor {f_scale:.4f}), WRITE_SIZE "
                 f"{float(write[cal]['Average']) * 1024:,.0f} B (factor {w_scale:.4f}).", "",
             "| form of the path | kernel | reads MB | writes MB | HBM bytes per launch | algorithmic / actual bytes | ratio |",
             "|---|---|---|---|---|---|---|"]
    result = {}
    spec = [("fused", KERNELS["fused"][1], "Average"), ("pack_reduce", KERNELS["fused"][1], "Average"),
            ("step", KERNELS["step"][1], "Max"), ("step_without_out", KERNELS["step"][1], "Min"),
            ("pack", KERNELS["pack"][1], "Average"), ("reduce", KERNELS["reduce"][1], "Average"),
            ("unpack", KERNELS["unpack"][1], "Average"), ("unpack_only", KERNELS["unpack"][1], "Average"),
            ("unpack_update", KERNELS["unpack_update"][1], "Max"),
            ("unpack_update_without_out", KERNELS["unpack_update"][1], "Min"),
            ("gated_all_arrived", KERNELS["gated_all_arrived"][1], "Average")]
    for variant, pattern, stat in spec:
        k = pick(pattern)
        if k is None:
            continue
        rd = float(fetch[k][stat]) * 1024 * f_scale
        wr = float(write[k][stat]) * 1024 * w_scale
        alg = 4 * UNITS[variant](n) * p
        result[variant] = int(round(rd + wr))
        text.append(f"| {variant} | {short(k[0])} | {rd / 1e6:.1f} | {wr / 1e6:.1f} | {rd + wr:,.0f} | {alg:,} | "
                    f"{(rd + wr) / alg:.4f} |")
    text.append("")
    with open(os.path.join(PROFILES, f"all_kernels_{wl_tag}_hbm_traffic.md"), "w") as f:
        f.write("\n".join(text))
    return result


def summarise() -> None:
    os.makedirs(PROFILES, exist_ok=True)
    for wl_tag, variant, steps in TRACES:
        _trace_summary(wl_tag, variant, steps)
    traffic = {}
    for wl_tag, steps in COUNTER_RUNS:
        traffic[wl_tag] = _traffic_summary(wl_tag, steps)
    with open(os.path.join(PROFILES, "traffic.json"), "w") as f:
        json.dump({"_about": "HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same "
                             "counters read for a plain copy of known size; written by "
                             "`python3 -m paper_1811_11141_amd.profiling summarise` from the runs summarised in "
                             "profiles/all_kernels_*_hbm_traffic.md", **traffic}, f, indent=1)
    print(json.dumps(traffic, indent=1))


if __name__ == "__main__":
    # run [all|traces|counters] on the GPU machine, summarise anywhere
    if len(sys.argv) > 1 and sys.argv[1] == "run":
        run(sys.argv[2] if len(sys.argv) > 2 else "all", sys.argv[3] if len(sys.argv) > 3 else "")
    else:
        summarise()
