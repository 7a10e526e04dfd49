"""Measurements around the hot path: cost-model calibration and the event-driven schedule.

    python -m paper_1811_11141_amd.experiments --workload resnet50
    python -m paper_1811_11141_amd.experiments --workload resnet50 --scaling     (host only)
    python -m paper_1811_11141_amd.experiments --workload resnet50 --producers   (kernels beside a waiting gated launch)

1. Calibration (what Section V-A does for the network): time every group of a plan alone,
   as a function of its message size M = 4 * (parameters in the group), and fit
   T(M) = a + b*M by least squares (mgwfbp_fit_cost).  Here the "all-reduce" of a group is the
   fused N-way reduction kernel on this GPU, so a is the cost of one launch and 1/b the
   effective reduction rate per message byte.
2. Schedule: plan with the fitted (a, b), run one event-driven iteration (mgwfbp_run_iteration,
   Algorithm 2 on two streams with timed stand-ins for the backward pass) for the no-merging,
   single-group, Theorem-1 and optimal plans, and compare the measured end of the last group
   with the iteration time the model predicts (Eq. 8); the same iteration is also replayed
   from a HIP graph (mgwfbp_iteration_capture) and run with the communication side as one gated
   launch (mgwfbp_run_iteration_gated).  calibrate_arrival() fits Eq. 9 to one message that
   arrives alone, for the launch per group and for the gated launch.

3. Scaling (--scaling): the trace-based simulation of Section V-C on the synthetic traces.

Only argument marshalling and timing happen here; all device work is in the library.
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def _bound_plans(mg, wl, w, mode, a, b, tb, n_sets, dev, seed=7):
    import torch

    plans = []
    for s in range(n_sets):
        grads = wl.make_gradients(w, seed + s, dev)
        out = [torch.empty_like(t) for t in grads[0]]
        pl = mg.mgwfbp_plan(w.p, tb, 0.0, a, b, w.n_workers, mode)
        pl.bind(grads, out)
        plans.append(pl)
    return plans


def measure_group_times(plans, stream, reps: int = 30, warmup: int = 3):
    """Average time of each group's fused launch, rotating over the bound plans (one per
    independently allocated gradient set) so that repeats do not hit in cache.
    Returns (message bytes per group, milliseconds per group)."""
    import torch

    info = plans[0].info()
    ng = info["n_groups"]
    nbytes = info["group_elems"].astype(np.float64) * 4.0
    ms = np.zeros(ng)
    for k in range(ng):
        for i in range(warmup):
            plans[i % len(plans)].pack_reduce_unpack(group=k, stream=stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(reps):
            plans[i % len(plans)].pack_reduce_unpack(group=k, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms[k] = e0.elapsed_time(e1) / reps
    return nbytes, ms


def calibrate(workload: str = "resnet50", n_sets: int = 3, device: str = "cuda:0"):
    """Fit (a_ms, b_ms_per_byte) from the per-layer groups of the no-merging plan."""
    import torch

    from . import binding as mg
    from . import workloads as wl

    w = wl.cnn_workload(workload)
    plans = _bound_plans(mg, wl, w, mg.MODE_WFBP, w.a_ms, w.b_ms_per_byte, w.tb_ms, n_sets, device)
    stream = torch.cuda.Stream(device=device)
    nbytes, ms = measure_group_times(plans, stream)
    a, b = mg.mgwfbp_fit_cost(nbytes, ms)
    resid = ms - (a + b * nbytes)
    big = np.argsort(nbytes)[-4:]
    return {"a_ms": a, "b_ms_per_byte": b, "samples": int(len(ms)),
            "largest_messages": [[float(nbytes[i]), float(ms[i])] for i in big],
            "bytes_min": float(nbytes.min()), "bytes_max": float(nbytes.max()),
            "rms_residual_ms": float(np.sqrt(np.mean(resid ** 2))),
            "max_residual_ms": float(np.abs(resid).max())}


def calibrate_in_schedule(workload: str = "resnet50", device: str = "cuda:0", reps: int = 5):
    """Fit (a, b) from the event-driven schedule itself: with zero backward time the groups of
    the no-merging plan run back to back on the communication stream, and the interval between
    the ends of consecutive groups is the whole per-message cost of this transport (kernel,
    launch, event record and wait), which is what Eq. 9 models."""
    import torch

    from . import binding as mg
    from . import workloads as wl

    w = wl.cnn_workload(workload)
    pl = _bound_plans(mg, wl, w, mg.MODE_WFBP, w.a_ms, w.b_ms_per_byte, w.tb_ms, 1, device)[0]
    s_comp, s_comm = torch.cuda.Stream(device=device), torch.cuda.Stream(device=device)
    zeros = np.zeros(w.L)
    pl.run_iteration(s_comp, s_comm, tb_ms=zeros)
    inter = []
    for _ in range(reps):
        t = pl.run_iteration(s_comp, s_comm, tb_ms=zeros)
        gf = t["group_finish_ms"]
        inter.append(np.diff(gf))
    inter = np.median(np.array(inter), axis=0)
    nbytes = pl.info()["group_elems"].astype(np.float64)[1:] * 4.0
    a, b = mg.mgwfbp_fit_cost(nbytes, inter)
    resid = inter - (a + b * nbytes)
    pl.destroy()
    return {"a_ms": a, "b_ms_per_byte": b, "samples": int(len(inter)),
            "rms_residual_ms": float(np.sqrt(np.mean(resid ** 2)))}


def _stream_pair(pl, device, tries: int = 8):
    """Two streams whose kernels the device runs at the same time (the gated launch needs that)."""
    import torch

    for _ in range(tries):
        a, b = torch.cuda.Stream(device=device), torch.cuda.Stream(device=device)
        if pl.streams_side_by_side(a, b):
            return a, b
    raise RuntimeError("no pair of streams ran side by side")


def calibrate_arrival(n_workers: int = 8, device: str = "cuda:0", reps: int = 7,
                      sizes=(1 << 10, 1 << 12, 1 << 14, 1 << 16, 1 << 18, 1 << 20, 1 << 21, 1 << 22, 1 << 23)):
    """Eq. 9 for one message that arrives alone: a one-layer net of p parameters, a 0.3 ms backward
    pass, and the time from the end of that pass to the end of the iteration, for the launch per
    group (mgwfbp_run_iteration) and for the gated launch (mgwfbp_run_iteration_gated).  Fits
    (a, b) to each: a is what a message costs however small it is."""
    import torch

    from . import binding as mg
    from . import workloads as wl

    tb = np.array([0.3])
    nbytes, launch, gated = [], [], []
    for p in sizes:
        w = wl.custom_workload([int(p)], n_workers, tb_ms=tb)
        grads = wl.make_gradients(w, 11, device)
        pl = mg.mgwfbp_plan(w.p, tb, 0.0, w.a_ms, w.b_ms_per_byte, n_workers, mg.MODE_SINGLE)
        pl.bind(grads, [torch.empty_like(t) for t in grads[0]])
        s_comp, s_comm = _stream_pair(pl, device)
        pl.run_iteration(s_comp, s_comm, timeline=False)
        pl.run_iteration_gated(s_comp, s_comm)
        t_l = [pl.run_iteration(s_comp, s_comm, timeline=False)["t_iter_ms"] for _ in range(reps)]
        t_g = [pl.run_iteration_gated(s_comp, s_comm) for _ in range(reps)]
        nbytes.append(4.0 * p)
        launch.append(float(np.median(t_l)) - 0.3)
        gated.append(float(np.median(t_g)) - 0.3)
        pl.destroy()
    out = {"n_workers": n_workers, "message_bytes": nbytes}
    for name, ms in (("launch_per_group", launch), ("gated_launch", gated)):
        a, b = mg.mgwfbp_fit_cost(np.array(nbytes), np.array(ms))
        out[name] = {"after_arrival_ms": ms, "a_ms": a, "b_ms_per_byte": b}
    return out


def producers_beside_gated_launch(workload: str = "resnet50", device: str = "cuda:0", give_up_ms: float = 1000.0):
    """What a waiting gated launch does to the kernels that produce the gradients.  One producer
    kernel per group on the signalling stream, each followed by the group's signal: an elementwise
    kernel (256-lane workgroups, few registers), an fp32 GEMM (160 registers, 65 KiB LDS) and an
    fp16 matrix-core GEMM (the whole register file of a SIMD), 4096^3 each.  Shapes of the launch:
    the default grid, 8 and 4 workgroups per compute unit on the whole chip, and the default grid on
    a stream confined to half the compute units.  Reports the producers' time alone and beside the
    waiting launch, and whether the launch gave up (the producers were not placed in time)."""
    import time

    import torch

    from . import binding as mg
    from . import workloads as wl

    w = wl.cnn_workload(workload)
    grads = wl.make_gradients(w, 5, device)
    out = [torch.empty_like(t) for t in grads[0]]
    wt, vt = wl.make_weights(w, 5, device)
    a32 = torch.randn(4096, 4096, device=device)
    b32 = torch.randn(4096, 4096, device=device)
    a16, b16 = a32.half(), b32.half()
    producers = {"elementwise": lambda: a32.add_(1.0), "gemm_fp32": lambda: torch.mm(a32, b32),
                 "gemm_fp16_matrix_cores": lambda: torch.mm(a16, b16)}
    n_cus = torch.cuda.get_device_properties(device).multi_processor_count
    half = n_cus // 2 // 32 * 32
    confined = mg.ConfinedStream(half)
    out_rows = {"workload": workload, "compute_units": n_cus, "shapes": {}}
    try:
        for shape, per_cu, cus in (("default", -1, 0), ("8_per_unit", 8, 0), ("4_per_unit", 4, 0),
                                   (f"default_on_{half}_units", -1, half)):
            for update in (False, True):
                pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
                pl.set_option(mg.OPT_GATED_WGS_PER_CU, per_cu)
                pl.set_option(mg.OPT_GATED_CUS, cus)
                pl.bind(grads, out, wt, vt)
                if cus:
                    s_launch = confined.stream
                    for _ in range(8):
                        s_sig = torch.cuda.Stream(device=device)
                        if pl.streams_side_by_side(s_sig, s_launch):
                            break
                    else:
                        raise RuntimeError("no stream ran beside the confined one")
                else:
                    s_sig, s_launch = _stream_pair(pl, device)
                ng = pl.info()["n_groups"]
                row = {"workgroups": pl.gated_workgroups(update)[0], "per_unit": pl.gated_workgroups(update)[1]}
                arrival = 0
                for name, fn in producers.items():
                    with torch.cuda.stream(s_sig):
                        fn(); fn()                            # first calls on a stream allocate workspaces
                        torch.cuda.synchronize()
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record(s_sig)
                        for _ in range(ng):
                            fn()
                        e1.record(s_sig)
                    torch.cuda.synchronize()
                    alone = e0.elapsed_time(e1)
                    arrival += 1
                    t0 = time.perf_counter()
                    pl.gated_launch(arrival, update=update, lr=0.1, momentum=0.9, give_up_ms=give_up_ms, stream=s_launch)
                    with torch.cuda.stream(s_sig):
                        for k in range(ng):
                            fn()
                            pl.gated_signal(k, arrival, stream=s_sig)
                    torch.cuda.synchronize()
                    row[name] = {"alone_ms": alone, "beside_the_waiting_launch_ms": (time.perf_counter() - t0) * 1e3,
                                 "gave_up": pl.gated_gave_up()}
                out_rows["shapes"][shape + ("_update" if update else "")] = row
                pl.destroy()
    finally:
        torch.cuda.synchronize()
        confined.destroy()
    return out_rows


def schedule(workload: str, a_ms: float, b_ms_per_byte: float, backward_ms: float = 5.0,
             device: str = "cuda:0", reps: int = 5):
    """Predicted (Eq. 8 with the given a, b) and measured iteration times of four plans.

    The backward times are the workload's FLOP-proportional t_b rescaled to sum to
    `backward_ms`, so that the reductions matter next to the backward pass."""
    import torch

    from . import binding as mg
    from . import workloads as wl

    w = wl.cnn_workload(workload)
    tb = w.tb_ms * (backward_ms / w.tb_ms.sum())
    s_comp = s_comm = None
    out = {"workload": workload, "a_ms": a_ms, "b_ms_per_byte": b_ms_per_byte,
           "backward_ms": backward_ms, "plans": {}}
    for name, mode in (("wfbp", mg.MODE_WFBP), ("single", mg.MODE_SINGLE),
                       ("theorem1", mg.MODE_PAPER_GREEDY), ("optimal", mg.MODE_OPTIMAL)):
        pl = _bound_plans(mg, wl, w, mode, a_ms, b_ms_per_byte, tb, 1, device)[0]
        if s_comp is None:
            s_comp, s_comm = _stream_pair(pl, device)
        elif not pl.streams_side_by_side(s_comp, s_comm):     # remembered per plan: a handshake of 20 us
            raise RuntimeError("the stream pair stopped running side by side")
        pl.run_iteration(s_comp, s_comm)                      # warm-up
        pl.run_iteration_gated(s_comp, s_comm)
        t = [pl.run_iteration(s_comp, s_comm) for _ in range(reps)]
        gated = np.array([pl.run_iteration_gated(s_comp, s_comm) for _ in range(reps)])
        light = np.array([pl.run_iteration(s_comp, s_comm, timeline=False)["t_iter_ms"] for _ in range(reps)])
        it = pl.capture_iteration(s_comp, s_comm)
        it.replay(s_comp)                                     # warm-up
        graph = np.array([it.replay(s_comp) for _ in range(reps)])
        it.destroy()
        meas = np.array([x["t_iter_ms"] for x in t])
        bwd = np.array([x["group_ready_ms"][-1] for x in t])
        inf = pl.info()
        out["plans"][name] = {"groups": inf["n_groups"], "predicted_t_iter_ms": inf["t_iter_ms"],
                              "measured_t_iter_ms": float(np.median(meas)),
                              "measured_t_iter_without_timestamps_ms": float(np.median(light)),
                              "measured_t_iter_graph_replay_ms": float(np.median(graph)),
                              "measured_t_iter_gated_launch_ms": float(np.median(gated)),
                              "measured_backward_ms": float(np.median(bwd)),
                              "not_overlapped_ms": float(np.median(meas - bwd))}
        pl.destroy()
    return out


def scaling(workload: str, workers=(4, 8, 16, 32, 64), algorithm: str = "ring", alpha_ms: float = 0.04526,
            beta_ms_per_byte: float = 8e-7, gamma_ms_per_byte: float = 0.0):
    """Trace-based weak-scaling table (Section V-C): Table II costs per worker count, planned per
    mode, Eq. 4 speedup, and the communication left outside the computation,
    t_iter - (t_f + sum t_b).  Host only.  alpha: 45.26 us is what the ring start-ups of Section
    V-A imply; beta: 10 Gb/s.  t_f is taken as half the backward pass."""
    from . import binding as mg
    from . import workloads as wl

    w = wl.cnn_workload(workload)
    tf = float(w.tb_ms.sum()) / 2.0
    comp = tf + float(w.tb_ms.sum())
    out = {"workload": workload, "algorithm": algorithm, "alpha_ms": alpha_ms, "beta_ms_per_byte": beta_ms_per_byte,
           "t_f_ms": tf, "t_b_ms": float(w.tb_ms.sum()), "workers": list(workers), "modes": {}}
    for name, mode in (("wfbp", mg.MODE_WFBP), ("single", mg.MODE_SINGLE),
                       ("theorem1", mg.MODE_PAPER_GREEDY), ("optimal", mg.MODE_OPTIMAL)):
        t_iter, speedup = mg.mgwfbp_scaling_curve(w.p, w.tb_ms, tf, algorithm, alpha_ms, beta_ms_per_byte,
                                                  gamma_ms_per_byte, list(workers), mode)
        out["modes"][name] = {"t_iter_ms": [float(x) for x in t_iter], "speedup": [float(x) for x in speedup],
                              "not_overlapped_ms": [float(x) - comp for x in t_iter]}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet50", choices=["resnet50", "googlenet", "alexnet", "vgg16"])
    ap.add_argument("--backward-ms", type=float, nargs="+", default=[5.0, 1.0])
    ap.add_argument("--scaling", action="store_true", help="only the host-side scaling table (no GPU)")
    ap.add_argument("--producers", action="store_true", help="only: producer kernels beside a waiting gated launch")
    args = ap.parse_args()
    if args.scaling:
        print(json.dumps(scaling(args.workload)))
        return
    if args.producers:
        print(json.dumps(producers_beside_gated_launch(args.workload)))
        return
    cal = calibrate(args.workload)
    cal2 = calibrate_in_schedule(args.workload)
    sched = [schedule(args.workload, cal2["a_ms"], cal2["b_ms_per_byte"], t) for t in args.backward_ms]
    print(json.dumps({"calibration_back_to_back": cal, "calibration_in_schedule": cal2,
                      "calibration_one_message_after_arrival": calibrate_arrival(), "schedule": sched}))


if __name__ == "__main__":
    main()
