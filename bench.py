#!/usr/bin/env python3
"""Throughput of the merged pack+reduce+unpack pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50] [--variant fused]

A step is one pass of the whole hot path over one synthetic gradient set: all N workers'
per-layer gradients are packed, summed in worker order, scaled by 1/N and written back to
per-layer tensors, for every group of the merge plan, in one fused launch
(mgwfbp_pack_reduce_unpack with group = -1).  Inputs are resident in HBM before the timed
region.  Consecutive steps rotate over several independently allocated gradient sets (and
merged buffers, where a variant reads one) so that no step finds its inputs in the 256 MB
Infinity Cache.

Prints one JSON line.  `value` = algorithmic bytes 4*(N+1)*P per step / wall time per step.
`roofline.achieved` = the same bytes / average duration per launch from HIP events recorded on
the launch stream: every timed step lies inside one bracket of 8 back-to-back steps, and a
bracket's duration / 8 is the time per launch (an event pair costs 2-5 us of stream time, which a
pair around every single launch would add to what it measures; all figures under `extra` are
taken the same way).  `roofline.traffic` = HBM bytes per launch from the rocprofv3 counter runs
summarised under profiles/ (profiles/traffic.json; null for a workload or variant that has none).

With --extras 1 (default) the same gradient sets also go through the other forms of the path
(update, materialised chain, launch per group, the two halves a transport calls, the three
materialised kernels one by one) and through plain streaming probes.  With --others 1 (default
for the default workload) the other gradient sets the paper's evaluation names -- VGG-16 at
N = 16 and N = 8 and at three start-up costs, GoogLeNet, AlexNet -- are measured too, each in a
child process of its own that is started before this process touches the GPU, and reported under
`extra.<set>` (`resnet50_n12` is the default set with 12 workers, a count the kernels have no
unrolled worker loop for).
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
EVERY = 8              # consecutive steps bracketed by one HIP-event pair

VARIANTS = ("fused", "step", "step_without_out", "materialised", "per_group", "per_group_2streams",
            "per_group_gated", "gated_all_arrived", "pack",
            "reduce", "unpack", "pack_reduce", "unpack_only", "unpack_update", "unpack_update_without_out")


def units(variant: str, N: int) -> int:
    """Algorithmic (for the materialised forms: actual) traffic in units of 4P bytes."""
    return {"fused": N + 1, "per_group": N + 1, "per_group_2streams": N + 1, "materialised": N + 1,
            "per_group_gated": N + 1, "gated_all_arrived": N + 1,
            "step": N + 5, "step_without_out": N + 4, "pack": 2 * N, "reduce": N + 1, "unpack": 2,
            "pack_reduce": N + 1, "unpack_only": 2, "unpack_update": 6, "unpack_update_without_out": 5}[variant]


KERNEL_OF = {"fused": "k_fused", "per_group": "k_fused", "per_group_2streams": "k_fused", "step": "k_fused (update)",
             "per_group_gated": "k_fused_gated", "gated_all_arrived": "k_fused_gated",
             "step_without_out": "k_fused (update)", "materialised": "k_pack+k_reduce+k_unpack", "pack": "k_pack",
             "reduce": "k_reduce", "unpack": "k_unpack", "pack_reduce": "k_fused (merged out)",
             "unpack_only": "k_unpack", "unpack_update": "k_unpack (update)",
             "unpack_update_without_out": "k_unpack (update)"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="resnet50", choices=["resnet50", "googlenet", "alexnet", "vgg16"])
    ap.add_argument("--a-ms", type=float, default=0.5)
    ap.add_argument("--n-workers", type=int, default=0, help="replicas N (0 = the workload's own: 8, VGG-16 16)")
    ap.add_argument("--mode", default="optimal", choices=["optimal", "greedy", "wfbp", "single"])
    ap.add_argument("--sets", type=int, default=0, help="gradient sets to rotate over (0 = auto)")
    ap.add_argument("--tile", type=int, default=0)
    ap.add_argument("--small", type=int, default=-1)
    ap.add_argument("--nontemporal", type=int, default=-1)
    ap.add_argument("--skip", default="", help="comma-separated variants to leave out of --extras (under a "
                    "profiler that runs one kernel at a time the signals of per_group_gated cannot run beside the launch)")
    ap.add_argument("--variant", default="fused", choices=VARIANTS, help="what one step runs (the headline is 'fused')")
    ap.add_argument("--tune", type=int, default=0,
                    help="1: let mgwfbp_tune pick the launch shape of the timed plans at set-up (untimed)")
    ap.add_argument("--extras", type=int, default=1, help="also time the other variants and the probes")
    ap.add_argument("--others", type=int, default=-1,
                    help="also measure the other gradient sets in child processes (-1: only for the default workload)")
    ap.add_argument("--also", default="", help="comma-separated variants to time besides --variant (child runs use it)")
    ap.add_argument("--cpu-baseline", type=int, default=1)
    ap.add_argument("--cpu-seconds", type=float, default=14.0)
    return ap.parse_args()


# the other gradient sets of the paper's evaluation, each measured in a child process
OTHER_SETS = (
    ("vgg16_n16", ["--workload", "vgg16", "--also", "step,pack,unpack,unpack_update,unpack_update_without_out,fused_tuned"], 40),
    ("vgg16_n8", ["--workload", "vgg16", "--n-workers", "8", "--also", "step,fused_tuned"], 60),
    ("vgg16_n16_a0.1", ["--workload", "vgg16", "--a-ms", "0.1"], 30),
    ("vgg16_n16_a2", ["--workload", "vgg16", "--a-ms", "2.0"], 30),
    ("googlenet_n8", ["--workload", "googlenet", "--also",
                      "step,per_group,per_group_2streams,per_group_gated,pack,unpack,unpack_update,unpack_update_without_out"], 200),
    ("alexnet_n8", ["--workload", "alexnet", "--also", "step,fused_tuned"], 100),
    # a worker count that is not a power of two: the worker loop of the kernels is a run-time loop
    ("resnet50_n12", ["--workload", "resnet50", "--n-workers", "12", "--also", "step"], 100),
)


def run_others():
    """Each set in a fresh process (a set allocated after another set's large blocks were freed
    measured ~3 % slower than in a run of its own).  Returns {name: result or error}."""
    res = {}
    for name, argv, steps in OTHER_SETS:
        cmd = [sys.executable, os.path.abspath(__file__), *argv, "--steps", str(steps), "--warmup", str(max(5, steps // 8)),
               "--extras", "0", "--others", "0", "--cpu-baseline", "0"]
        try:
            out = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
            line = [l for l in out.stdout.splitlines() if l.startswith("{")]
            if out.returncode != 0 or not line:
                res[name] = {"error": f"rc {out.returncode}: {(out.stderr or out.stdout)[-300:]}"}
                continue
            r = json.loads(line[-1])
            keep = {"P": r["config"]["P"], "n_workers": r["config"]["n_workers"], "a_ms": r["config"]["a_ms"],
                    "groups": r["config"]["groups"], "rotating_sets": r["config"]["rotating_sets"],
                    "fused": {"us_per_launch": r["roofline"]["kernel_avg_us"], "GBps_algorithmic": r["roofline"]["achieved"],
                              "frac_of_peak": r["roofline"]["frac"], "value_GBps": r["value"],
                              "traffic": r["roofline"]["traffic"]}}
            keep.update(r.get("extra", {}))
            res[name] = keep
        except Exception as e:  # a failing side measurement is reported, not fatal
            res[name] = {"error": f"{type(e).__name__}: {e}"}
    return res


def load_traffic():
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {}


def main():
    args = parse()
    args.steps, args.warmup = max(1, args.steps), max(0, args.warmup)
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the other workers are "
              "replicas in the same HBM); run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    do_others = args.others == 1 or (args.others < 0 and args.workload == "resnet50" and args.variant == "fused"
                                     and not args.n_workers and args.extras)
    others = run_others() if do_others else None    # before this process initialises the GPU

    import numpy as np
    import torch

    from paper_1811_11141_amd import binding as mg
    from paper_1811_11141_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda:0"
    w = wl.cnn_workload(args.workload, a_ms=args.a_ms, n_workers=args.n_workers or None)
    N, P, L = w.n_workers, w.P, w.L
    mode = {"optimal": mg.MODE_OPTIMAL, "greedy": mg.MODE_PAPER_GREEDY, "wfbp": mg.MODE_WFBP,
            "single": mg.MODE_SINGLE}[args.mode]
    traffic = load_traffic().get(f"{args.workload}_n{N}", {})

    set_bytes = 4 * (N + 1) * P
    n_sets = args.sets if args.sets > 0 else max(3, min(4, int(np.ceil(768e6 / set_bytes)) + 1))
    if args.workload == "vgg16" and args.sets <= 0:
        n_sets = 1 if N >= 16 else 2  # 9.4 GB (N = 8: 5 GB) per pass evicts itself

    def new_plan(mode=mode):
        pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, N, mode)
        if args.tile:
            pl.set_option(mg.OPT_TILE_ELEMS, args.tile)
        if args.small >= 0:
            pl.set_option(mg.OPT_SMALL_ELEMS, args.small)
        if args.nontemporal >= 0:
            pl.set_option(mg.OPT_NONTEMPORAL, args.nontemporal)
        return pl

    also = [v for v in args.also.split(",") if v]
    wanted = {args.variant, *also}
    if args.extras:
        wanted |= set(VARIANTS)
    need_ws = wanted & {"materialised", "pack", "reduce", "unpack"}
    need_mb = wanted & {"pack_reduce", "unpack_only", "unpack_update", "unpack_update_without_out"}
    need_alt = wanted & {"step_without_out", "unpack_update_without_out"}

    sets = []
    for s in range(n_sets):
        grads = wl.make_gradients(w, wl.BASE_SEED + 1000 * 2 + s, dev)
        out = [torch.empty_like(t) for t in grads[0]]
        wt, vt = wl.make_weights(w, wl.BASE_SEED + s, dev)
        pl = new_plan()
        pl.bind(grads, out, wt, vt)
        st = {"plan": pl, "grads": grads, "out": out, "w": wt, "v": vt}
        if need_mb:     # one merged buffer per set, so that a reader never finds it in the cache
            st["mb"] = torch.empty((P + 63) // 64 * 64, dtype=torch.float32, device=dev).normal_(0, 1e-3)
        if need_ws:     # reduce and unpack read what pack / reduce left there (filled at set-up)
            st["ws"] = torch.empty(pl.workspace_bytes() // 4, dtype=torch.float32, device=dev)
        if need_alt:    # the same tensors bound without out[]: the update alone
            st["plan_no_out"] = new_plan()
            st["plan_no_out"].bind(grads, None, wt, vt)
        sets.append(st)
    tuned = [s_["plan"].tune()["candidate"] for s_ in sets] if args.tune else None
    info = sets[0]["plan"].info()
    n_groups = info["n_groups"]

    # `side` signals to the gated launch on `stream`: the device must run the two side by side
    # (streams that share one of the runtime's hardware queues do not)
    for _ in range(8):
        stream = torch.cuda.Stream(device=dev)
        side = torch.cuda.Stream(device=dev)
        if sets[0]["plan"].streams_side_by_side(side, stream):
            break
    else:
        wanted -= {"per_group_gated", "gated_all_arrived"}
    wanted -= {v for v in args.skip.split(",") if v}
    for st in sets:
        st["arrival"] = 0

    def run_step(variant, i):
        st = sets[i % n_sets]
        pl = st["plan"]
        if variant == "fused":
            pl.pack_reduce_unpack(stream=stream)
        elif variant == "step":
            pl.step(0.1, 0.9, stream=stream)
        elif variant == "step_without_out":
            st["plan_no_out"].step(0.1, 0.9, stream=stream)
        elif variant == "materialised":
            pl.pack_reduce_unpack(workspace=st["ws"], stream=stream)
        elif variant == "per_group":
            for k in range(n_groups):
                pl.pack_reduce_unpack(group=k, stream=stream)
        elif variant == "per_group_2streams":
            # consecutive groups alternate between two streams of equal priority: one group's
            # ramp-up overlaps the previous group's drain (they touch disjoint tensors)
            fork = torch.cuda.Event()
            fork.record(stream)
            side.wait_event(fork)
            for k in range(n_groups):
                pl.pack_reduce_unpack(group=k, stream=stream if k % 2 == 0 else side)
            join = torch.cuda.Event()
            join.record(side)
            stream.wait_event(join)
        elif variant == "per_group_gated":
            # the whole plan is ONE launch that waits, group by group, for arrival counters which
            # a second stream bumps with one small kernel per group, back to back
            st["arrival"] += 1
            fork = torch.cuda.Event()
            fork.record(stream)
            side.wait_event(fork)
            pl.gated_launch(st["arrival"], give_up_ms=2000.0, stream=stream)
            for k in range(n_groups):
                pl.gated_signal(k, st["arrival"], stream=side)
            join = torch.cuda.Event()
            join.record(side)
            stream.wait_event(join)
        elif variant == "gated_all_arrived":
            # the same launch when every group has arrived before it starts: what the arrival-order
            # tile list and the look at the counters cost against the plain fused launch
            pl.gated_launch(st["arrival"], give_up_ms=2000.0, stream=stream)
        elif variant == "pack":
            pl.pack(st["ws"], stream=stream)
        elif variant == "reduce":
            pl.reduce(st["ws"], stream=stream)
        elif variant == "unpack":
            pl.unpack(st["ws"], stream=stream)
        elif variant == "pack_reduce":
            pl.pack_reduce(st["mb"], stream=stream)
        elif variant == "unpack_only":
            pl.unpack_update(st["mb"], stream=stream)
        elif variant == "unpack_update":
            pl.unpack_update(st["mb"], update=True, lr=0.1, momentum=0.9, stream=stream)
        elif variant == "unpack_update_without_out":
            st["plan_no_out"].unpack_update(st["mb"], update=True, lr=0.1, momentum=0.9, stream=stream)
        else:
            raise ValueError(variant)

    def timed(step_fn, steps, warmup):
        """Wall time per step and, from HIP-event brackets of up to EVERY back-to-back steps that
        together cover every timed step, the average / median / minimum time per step."""
        for i in range(warmup):
            step_fn(i)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True),
                min(EVERY, steps - i)) for i in range(0, steps, EVERY)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            if i % EVERY == 0:
                evs[i // EVERY][0].record(stream)
            step_fn(warmup + i)
            if i % EVERY == EVERY - 1 or i == steps - 1:
                evs[i // EVERY][1].record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        tot = np.array([a.elapsed_time(b) for a, b, _ in evs])
        cnt = np.array([c for _, _, c in evs], dtype=np.float64)
        per = tot / cnt
        return (t1 - t0) * 1e3 / steps, {"avg_ms": float(tot.sum() / cnt.sum()), "median_ms": float(np.median(per)),
                                         "min_ms": float(per.min()), "samples": int(cnt.sum())}

    def side_figure(variant, steps, warmup):
        for i in range(n_sets):
            run_step(variant, i)
        _, kk = timed(lambda i: run_step(variant, i), steps, warmup)
        nbytes = 4 * units(variant, N) * P
        gbps = nbytes / (kk["avg_ms"] * 1e-3) / 1e9
        fig = {"us_per_step": round(kk["avg_ms"] * 1e3, 2), "min_us": round(kk["min_ms"] * 1e3, 2),
               "bytes_per_step": nbytes, "GBps": round(gbps, 1), "frac_of_peak": round(gbps / HBM_PEAK_GBS, 4),
               "kernel": KERNEL_OF[variant], "traffic": traffic.get(variant)}
        if variant in ("per_group_gated", "gated_all_arrived"):
            fig["groups"] = n_groups
            fig["gave_up"] = any(st["plan"].gated_gave_up() for st in sets)
        if variant == "materialised":   # the chain really moves 3N + 3 units
            fig["GBps_actual_traffic"] = round(4 * (3 * N + 3) * P / (kk["avg_ms"] * 1e-3) / 1e9, 1)
        return fig

    # set-up, before the W warm-up steps: the materialised kernels need a filled workspace, and
    # one pass over every rotating set keeps code load and address translation of freshly
    # allocated tensors out of the timed steps
    for st in sets:
        if "ws" in st:
            st["plan"].pack(st["ws"], stream=stream)
            st["plan"].reduce(st["ws"], stream=stream)
    for i in range(n_sets):
        run_step(args.variant, i)
    torch.cuda.synchronize()
    ms_per_step, kern = timed(lambda i: run_step(args.variant, i), args.steps, args.warmup)
    bytes_step = 4 * units(args.variant, N) * P
    value = bytes_step / (ms_per_step * 1e-3) / 1e9
    achieved = bytes_step / (kern["avg_ms"] * 1e-3) / 1e9

    result = {
        "metric": "merged pack+reduce+unpack HBM GB/s",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}-shaped gradient set", "tensors": L, "P": P,
                   "n_workers": N, "plan": args.mode, "a_ms": w.a_ms, "b_ms_per_byte": w.b_ms_per_byte,
                   "groups": n_groups, "variant": args.variant, "rotating_sets": n_sets,
                   "tuned_launch_shape": tuned,
                   "algorithmic_bytes_per_step": bytes_step,
                   "percent_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic.get(args.variant),
                     "kernel": KERNEL_OF[args.variant],
                     "kernel_avg_us": round(kern["avg_ms"] * 1e3, 2),
                     "kernel_median_us": round(kern["median_ms"] * 1e3, 2),
                     "kernel_min_us": round(kern["min_ms"] * 1e3, 2),
                     "event_samples": kern["samples"]},
    }

    extra = {}
    k2, w2 = max(24, args.steps // 4), max(5, args.warmup // 4)

    def tuned_figure():
        """The fused pass after mgwfbp_tune (set-up, untimed) has picked the launch shape."""
        alt, picks = [], []
        for st in sets:
            pa = new_plan()
            pa.bind(st["grads"], st["out"], st["w"], st["v"])
            picks.append(pa.tune(stream)["candidate"])
            alt.append(pa)
        _, kk = timed(lambda i: alt[i % n_sets].pack_reduce_unpack(stream=stream), k2, w2)
        gb = set_bytes / (kk["avg_ms"] * 1e-3) / 1e9
        for pa in alt:
            pa.destroy()
        return {"us_per_step": round(kk["avg_ms"] * 1e3, 2), "choices": picks,
                "GBps": round(gb, 1), "frac_of_peak": round(gb / HBM_PEAK_GBS, 4)}

    try:
        for variant in also:
            if variant == "fused_tuned":
                extra[variant] = tuned_figure()
            elif variant != args.variant and variant in wanted:
                extra[variant] = side_figure(variant, k2, w2)
    except Exception as e:
        torch.cuda.synchronize()
        extra["error"] = f"{type(e).__name__}: {e}"
    if args.extras:
        # the headline line is complete without these: a failing extra is reported, not fatal
        try:
            for variant in VARIANTS:
                if variant != args.variant and variant not in extra and variant in wanted:
                    extra[variant] = side_figure(variant, k2, w2)
            # the launch-per-group sequence captured once per gradient set into a HIP graph
            graphs = []
            torch.cuda.synchronize()
            for st in sets:
                gph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gph, stream=stream):
                    cur = torch.cuda.current_stream()
                    for k in range(n_groups):
                        st["plan"].pack_reduce_unpack(group=k, stream=cur)
                graphs.append(gph)
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                _, kk = timed(lambda i: graphs[i % n_sets].replay(), k2, w2)
            extra["per_group_graph"] = {"groups": n_groups, "us_per_step": round(kk["avg_ms"] * 1e3, 2),
                                        "GBps": round(set_bytes / (kk["avg_ms"] * 1e-3) / 1e9, 1)}
            del graphs
            if not args.tune and "fused_tuned" not in extra:
                extra["fused_tuned"] = tuned_figure()
            # the two extreme plans (every tensor its own group / one group) through the same fused
            # launch: the rate should not depend on the plan
            for nm, md in (("fused_plan_wfbp", mg.MODE_WFBP), ("fused_plan_single", mg.MODE_SINGLE)):
                alt = []
                for st in sets:
                    pa = new_plan(md)
                    pa.bind(st["grads"], st["out"], st["w"], st["v"])
                    alt.append(pa)
                _, kk = timed(lambda i: alt[i % n_sets].pack_reduce_unpack(stream=stream), k2, w2)
                extra[nm] = {"groups": alt[0].info()["n_groups"], "us_per_step": round(kk["avg_ms"] * 1e3, 2),
                             "GBps": round(set_bytes / (kk["avg_ms"] * 1e-3) / 1e9, 1)}
                for pa in alt:
                    pa.destroy()
            # plain streaming kernels on buffers of the same size, rotated like the gradient sets:
            # what one read stream, one write stream, a copy and the vendor's copy reach on this machine
            n_probe = (N * P + 3) // 4 * 4
            bufs = [torch.empty(n_probe, dtype=torch.float32, device=dev).normal_() for _ in range(max(3, n_sets))]
            sink = torch.zeros(64, dtype=torch.float32, device=dev)
            nb = len(bufs)
            probes = (
                ("probe_read", lambda i: mg.mgwfbp_probe_read(bufs[i % nb], n_probe, sink, stream), 4 * n_probe),
                ("probe_fill", lambda i: mg.mgwfbp_probe_fill(bufs[i % nb], 1.0, n_probe, stream), 4 * n_probe),
                ("probe_copy", lambda i: mg.mgwfbp_probe_copy(bufs[i % nb], bufs[(i + 1) % nb], n_probe, stream), 8 * n_probe),
                ("probe_streams", lambda i: mg.mgwfbp_probe_streams(bufs[i % nb], N, n_probe // N // 4 * 4,
                                                                   n_probe // N // 4 * 4, bufs[(i + 1) % nb], stream),
                 4 * (N + 1) * (n_probe // N // 4 * 4)),
            )
            # the same copy at the size of one worker's set (what unpack moves): short launches pay
            # their ramp-up and drain
            n_small = (P + 3) // 4 * 4
            probes += (("probe_copy_one_set", lambda i: mg.mgwfbp_probe_copy(bufs[i % nb], bufs[(i + 1) % nb], n_small, stream),
                        8 * n_small),)
            for nm, fn, nbytes in probes:
                _, kk = timed(fn, k2, w2)
                gb = nbytes / (kk["avg_ms"] * 1e-3) / 1e9
                extra[nm] = {"us": round(kk["avg_ms"] * 1e3, 2), "GBps": round(gb, 1), "frac_of_peak": round(gb / HBM_PEAK_GBS, 4)}
            with torch.cuda.stream(stream):
                _, kk = timed(lambda i: bufs[(i + 1) % nb].copy_(bufs[i % nb], non_blocking=True), k2, w2)
            gb = 8 * n_probe / (kk["avg_ms"] * 1e-3) / 1e9
            extra["vendor_copy"] = {"what": "torch Tensor.copy_ device to device", "us": round(kk["avg_ms"] * 1e3, 2),
                                    "GBps": round(gb, 1), "frac_of_peak": round(gb / HBM_PEAK_GBS, 4)}
            del bufs
            # host side, once per training job: planning and binding time
            host = {}
            for nm, md in (("optimal", mg.MODE_OPTIMAL), ("theorem1", mg.MODE_PAPER_GREEDY)):
                t0 = time.perf_counter()
                for _ in range(20):
                    new_plan(md).destroy()
                host[f"plan_{nm}_us"] = round((time.perf_counter() - t0) / 20 * 1e6, 1)
            pb = new_plan()
            t0 = time.perf_counter()
            pb.bind(sets[0]["grads"], sets[0]["out"], sets[0]["w"], sets[0]["v"])
            host["bind_us"] = round((time.perf_counter() - t0) * 1e6, 1)
            pb.destroy()
            extra["host_once"] = host
            # the tiny configuration (8 layers, N = 4): launch latency only, no bandwidth claim
            lat = []
            for seed in range(8):
                tw = wl.tiny_workload(seed)
                tg = wl.make_gradients(tw, seed, dev)
                tp = mg.mgwfbp_plan(tw.p, tw.tb_ms, 0.0, tw.a_ms, tw.b_ms_per_byte, tw.n_workers, mg.MODE_OPTIMAL)
                tp.bind(tg, [torch.empty_like(t) for t in tg[0]])
                _, kk = timed(lambda i: tp.pack_reduce_unpack(stream=stream), 48, 5)
                lat.append(kk["avg_ms"] * 1e3)
                tp.destroy()
            extra["tiny_config_us_per_launch"] = {"median": round(float(np.median(lat)), 2),
                                                  "min": round(float(np.min(lat)), 2), "seeds": len(lat)}
        except Exception as e:
            torch.cuda.synchronize()
            extra["error"] = f"{type(e).__name__}: {e}"
    if others is not None:
        extra.update(others)
    if extra:
        result["extra"] = extra
    props = torch.cuda.get_device_properties(0)
    result["device"] = {"name": props.name, "compute_units": props.multi_processor_count,
                        "hbm_GiB": round(props.total_memory / 2 ** 30, 1)}

    if args.cpu_baseline:
        try:
            result["cpu_baseline"] = cpu_baseline(w, sets[0], args.cpu_seconds)
            result["cpu_baseline"]["gpu_over_cpu"] = round(value / result["cpu_baseline"]["value"], 1)
        except Exception as e:  # e.g. the oracle's C library is not built: say so in the line
            result["cpu_baseline"] = {"value": None, "unit": "GB/s", "cores": 0, "kind": "oracle",
                                      "sample": f"not measured: {type(e).__name__}: {e}"}

    print(json.dumps(result))


def cpu_baseline(w, s, budget_s):
    """The CPU oracle, as it stands, on the same gradient set: whole passes of pack -> reduce ->
    unpack per group over host copies of set 0, first on one thread, then with its element loops
    split over all host cores the process may use; the faster leg is the reported value."""
    from oracle import datapath as od

    N, P = w.n_workers, w.P
    groups = s["plan"].groups()
    g_np = [[t.cpu().numpy() for t in rep] for rep in s["grads"]]
    od.merged_gradient_path([[a[:16].copy() for a in rep] for rep in g_np], groups)  # load + warm
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    nthreads = max(1, min(od.max_threads(), usable))
    legs = {}
    for threads, share in ((1, 0.5), (nthreads, 0.5)):
        passes, t0 = 0, time.perf_counter()
        while True:
            od.merged_gradient_path(g_np, groups, threads=threads)
            passes += 1
            el = time.perf_counter() - t0
            if (el >= budget_s * share and passes >= 3) or passes >= 1000:
                break
        legs[threads] = {"threads": threads, "passes": passes, "seconds": round(el, 2),
                         "seconds_per_pass": round(el / passes, 4),
                         "value": round(4 * (N + 1) * P / (el / passes) / 1e9, 3)}
        if nthreads == 1:
            break
    best = max(legs.values(), key=lambda x: x["value"])
    total_s = sum(x["seconds"] for x in legs.values())
    return {"value": best["value"], "unit": "GB/s", "cores": best["threads"], "kind": "oracle",
            "sample": f"whole passes of the oracle (pack, reduce, unpack per group) over gradient set 0 of the same "
                      f"workload: {', '.join(str(x['passes']) + ' on ' + str(x['threads']) + ' thread(s)' for x in legs.values())}, "
                      f"{total_s:.1f} s in all",
            "seconds_per_pass": best["seconds_per_pass"], "ns_per_element": round(best["seconds_per_pass"] / P * 1e9, 3),
            "legs": list(legs.values())}


if __name__ == "__main__":
    main()
