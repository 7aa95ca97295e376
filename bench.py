#!/usr/bin/env python3
"""Throughput of the LASGD update path on one MI355X.

One "step" of this benchmark is one full cycle of the hot path on the
ResNet-50-shaped workload (K = 8 replicas, 161 tensors, 25,557,032 fp32
parameters each, global update every m = 4 local steps):

    m-1 x lasgd_local_step   (main stream)
    1   x lasgd_step_merge   (main stream, waits for the pending mean, re-sends)
    1   x lasgd_average      (side stream, overlapped with the next local steps)

i.e. m local updates of all K replicas plus one global update.  All inputs are
synthetic, seeded and already resident in HBM when the timed region starts.
The timed loop issues the calls exactly as a caller would (no events, no host
work in between); per-kernel launch durations for the roofline come from an
instrumented repeat of the same loop, stand-alone kernel times, the one-stream
and fused-mean cycles and the CPU oracle (all cores, one thread) from further
legs of the same run.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def algorithmic_bytes(K: int, N: int, bf16: bool) -> dict:
    """Bytes each kernel must move per launch (what the method needs, not what caches do)."""
    # local step: read g, x, v; write x, v (bf16: g and the bf16 copy are 2 bytes each)
    step = (2 + 4 + 4 + 4 + 4 + 2 if bf16 else 20) * K * N
    # fused step + global update + re-send: also read s and z (once per parameter), write s
    step_merge = step + 8 * K * N + 4 * N
    average = 4 * (K + 1) * N
    # the same with the next mean computed in the pass: z is read once and written once per parameter
    step_merge_average = step + 8 * K * N + 8 * N
    return {"local_step": step, "step_merge": step_merge, "average": average, "step_merge_average": step_merge_average}


def cpu_baseline(w, seconds: float = 10.0) -> dict:
    """The oracle as it stands, timed on this machine's host cores on whole cycles of the same
    workload (same shapes, K, cadence; one seeded gradient set reused), twice in this same
    run: the replica loop spread over all the cores it can use, and on a single thread.
    The top-level value is the all-cores leg."""
    import numpy as np
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd import workloads as W
    avail = len(os.sched_getaffinity(0))
    many = max(1, min(w.K, avail, int(os.environ.get("OMP_NUM_THREADS", "64"))))
    nt = len(w.numels)
    x0 = np.concatenate([W.initial_tensor(w, t) for t in range(nt)])
    r = np.random.Generator(np.random.Philox(key=12345))
    g = [(r.standard_normal(w.N, dtype=np.float32) * np.float32(1e-3)) for _ in range(w.K)]
    if w.storage == "bf16":
        x0 = W.to_bf16_bits(x0)
        g = [W.to_bf16_bits(a) for a in g]

    def leg(threads: int) -> dict:
        o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, [w.weight_decay] * nt, storage=w.storage, threads=threads)
        o.set_model(x0)
        o.prologue(g, w.lr)

        def cycle():
            for _ in range(w.m):
                o.iteration(g, w.lr, w.m)

        t0 = time.perf_counter()
        cycle()
        first = time.perf_counter() - t0
        warm = "after one untimed cycle"
        if first >= 0.6 * seconds:          # a cycle this long is its own sample
            n, dt, warm = 1, first, "no warm-up"
        else:
            n = int(max(1, min(20, seconds / max(first, 1e-3))))
            t0 = time.perf_counter()
            for _ in range(n):
                cycle()
            dt = time.perf_counter() - t0
        return {"value": w.K * w.N * w.m * n / dt, "unit": "params/s", "cores": threads, "kind": "oracle",
                "sample": f"{n} full cycle(s) (m={w.m} local steps + global update + mean) of {w.name}, "
                          f"all K={w.K} replicas and all {w.N} parameters, {warm}",
                "ms_per_cycle": 1e3 * dt / n}

    out = leg(many)
    out["host_cores_available"] = avail
    out["single_thread"] = leg(1) if many > 1 else dict(out)
    return out


def run_variant(args, w, make, alg) -> dict:
    """Timed loops over the extended entry points; one JSON line in the same format.
    Bytes are algorithmic: 20 B per replica-parameter that steps, +8 B (+4/K for z) per
    replica-parameter that merges and re-sends, 4(P+1) B per parameter for a mean over P."""
    import numpy as np
    import torch
    K, N = w.K, w.N
    full = (1 << K) - 1
    dev = make(side=True)
    c = dev.ctx
    per_rp_step = alg["local_step"] / (K * N)
    steps_done = 0          # replica-steps, for params/s
    nbytes = 0.0

    if args.mode == "sgd_ar":
        def one():
            nonlocal steps_done, nbytes
            c.sgd_ar_step(w.lr)
            steps_done += K
            nbytes += alg["local_step"]
        what = "one lasgd_sgd_ar_step: mean of the K gradients + the same local update on all K replicas"
    else:
        if args.mode == "elastic":
            c.set_elastic(0.5, 0.5)
        dev.prologue(w.lr)
        rng = np.random.default_rng(0)
        p = np.array([11.2, 72.8, 11.1, 0.2, 0.6, 3.9])
        rot = [0]

        def one():
            nonlocal steps_done, nbytes
            if args.mode == "dynamic":
                # steps per All-Reduce from the paper's histogram (tau_max = 5), slower nodes take fewer
                base = min(int(rng.choice(6, p=p / p.sum())) + 1, 5)
                counts = [max(1, base - (k % 3 == 0)) for k in range(K)]
                for j in range(max(counts)):
                    mask = sum(1 << k for k in range(K) if counts[k] > j)
                    lrs = [w.lr] * K
                    act = bin(mask).count("1")
                    if j == max(counts) - 1:
                        c.step_merge_ex(lrs, mask, full, True)
                        c.average()
                        nbytes += act * N * per_rp_step + 8 * K * N + 4 * N + alg["average"]
                    else:
                        c.local_step_ex(lrs, mask)
                        nbytes += act * N * per_rp_step
                    steps_done += act
            elif args.mode == "partial":
                # three quarters of the replicas take part in each All-Reduce, rotating
                P = max(1, (3 * K) // 4)
                part = sum(1 << ((rot[0] + i) % K) for i in range(P))
                rot[0] += 1
                late = part & ~one.prev
                for _ in range(w.m - 1):
                    c.local_step(w.lr)
                c.step_merge_ex([w.lr] * K, full, one.prev, True)
                if late:
                    c.snapshot_ex(late)
                c.average_ex(part)
                one.prev = part
                steps_done += K * w.m
                nbytes += w.m * alg["local_step"] + bin(one.prev).count("1") * N * 8 + 4 * N + 4 * (P + 1) * N \
                    + bin(late).count("1") * N * 8
            else:   # elastic: the headline cycle with alpha = beta = 0.5
                for _ in range(w.m - 1):
                    c.local_step(w.lr)
                c.step_merge(w.lr, True)
                c.average()
                steps_done += K * w.m
                nbytes += (w.m - 1) * alg["local_step"] + alg["step_merge"] + alg["average"] + 4 * N
        one.prev = full
        what = {"dynamic": "one All-Reduce round: 1..5 masked local steps per replica (paper's histogram), fused step+merge, mean",
                "partial": "one cycle with 3/4 of the replicas in each All-Reduce (rotating); latecomers re-send",
                "elastic": "the headline cycle with alpha = beta = 0.5"}[args.mode]

    for _ in range(args.warmup):
        one()
    c.sync(); torch.cuda.synchronize()
    steps_done, nbytes = 0, 0.0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one()
    c.sync(); torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tuning = c.get_tuning()
    dev.close()
    gbps = nbytes / dt / 1e9
    return {"metric": "params/sec and HBM GB/s (% of peak) for fused LASGD step+merge, K replicas",
            "value": steps_done * N / dt, "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16 storage, f32 arithmetic" if w.storage == "bf16" else "f32", "data": "synthetic",
            "config": {"workload": f"configs[{args.config}]: {w.name}, K={K}, {N} params/replica, mode={args.mode}",
                       "step": what, "mode": args.mode, "tuning": tuning},
            "roofline": {"bound": "hbm", "kernel": "whole step (all launches)", "achieved": gbps, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": gbps / HBM_PEAK_GBS, "traffic": None}}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="index into the baseline's config list")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-detail", action="store_true", help="skip the isolated per-kernel and serial legs")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run three plain 1 GiB device copies first (a kernel of known traffic, "
                         "to calibrate profiler byte counters)")
    ap.add_argument("--mode", default="lasgd", choices=["lasgd", "sgd_ar", "dynamic", "elastic", "partial"],
                    help="lasgd: the headline cycle; the others time the extended entry points "
                         "(SGD All-Reduce step, scripted adaptive cadence, alpha=beta=0.5, 75%% partial All-Reduce)")
    ap.add_argument("--tune", type=str, default="", help="k=v,k=v launch-shape knobs (lasgd_tuning fields)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (K replicas are resident on it and the All-Reduce is a "
              "reduction in HBM); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2203_13085_amd import binding as B
    from paper_2203_13085_amd import workloads as W
    from paper_2203_13085_amd.driver import DeviceReplicas

    B.load()
    w = W.config(args.config)
    bf16 = w.storage == "bf16"
    tune = {k: int(v) for k, v in (kv.split("=") for kv in args.tune.split(",") if kv)}

    def make(side: bool) -> DeviceReplicas:
        dev = DeviceReplicas(w, side_stream=side)
        if tune:
            dev.ctx.set_tuning(**tune)
        nt = len(w.numels)
        x0 = np.concatenate([W.initial_tensor(w, t) for t in range(nt)])
        if bf16:
            x0 = W.to_bf16_bits(x0)
        dev.load_model(x0)
        # gradients: N(0, 1e-3^2), drawn on the device with a seeded generator (values do not
        # affect timing; the parity tests use the host-keyed generator instead)
        gen = torch.Generator(device=dev.dev)
        gen.manual_seed(w.seed + 1)
        for k in range(w.K):
            dev.g[k].copy_((torch.randn(dev.g[k].numel(), generator=gen, device=dev.dev) * 1e-3).to(dev.g[k].dtype))
        torch.cuda.synchronize()
        return dev

    def cycle(dev, tau=0):
        for _ in range(w.m):
            tau = dev.iteration(w.lr, tau, w.m)

    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    alg = algorithmic_bytes(w.K, w.N, bf16)
    cycle_bytes = (w.m - 1) * alg["local_step"] + alg["step_merge"] + alg["average"]
    if args.mode != "lasgd":
        print(json.dumps(run_variant(args, w, make, alg)), flush=True)
        return 0

    # ---------------- the timed region: whole cycles, issued exactly as a caller would issue them
    # (no events, no host work between launches); the mean runs on a second stream where the
    # workload says so (the ResNet-50 configurations), else on the main stream ----------------
    dev = make(side=w.side_stream)
    dev.prologue(w.lr)
    for _ in range(args.warmup):
        cycle(dev)
    dev.ctx.sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        cycle(dev)
    dev.ctx.sync()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    value = w.K * w.N * w.m * args.steps / dt

    # ---------------- the same loop again with a HIP event pair around every launch, each on the
    # stream its kernel runs on: per-kernel launch durations inside the pipelined run, and how long
    # the main stream stood ready for a global update before the mean it needs had ended ----------
    ev = {"local_step": [], "step_merge": [], "average": []}
    ready, mean_end = [], []

    def instrumented_cycle():
        for _ in range(w.m - 1):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(dev.main)
            dev.ctx.local_step(w.lr)
            b.record(dev.main)
            ev["local_step"].append((a, b))
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(dev.main)
        dev.ctx.step_merge(w.lr, True)
        b.record(dev.main)
        ev["step_merge"].append((a, b))
        ready.append(a)
        c, d = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if dev.side is not dev.main:
            dev.side.wait_stream(dev.main)       # so that c marks the start of the mean, not of its wait
        c.record(dev.side)
        dev.ctx.average()
        d.record(dev.side)
        ev["average"].append((c, d))
        mean_end.append(d)

    n_inst = max(4, min(args.steps, 100))
    t0 = time.perf_counter()
    for _ in range(n_inst):
        instrumented_cycle()
    dev.ctx.sync()
    torch.cuda.synchronize()
    ms_instrumented = 1e3 * (time.perf_counter() - t0) / n_inst
    kern_ms = {k: float(np.mean([p[0].elapsed_time(p[1]) for p in v])) for k, v in ev.items() if v}
    # > 0: the mean of cycle i-1 ended that long AFTER the main stream was ready for cycle i's global update
    gaps = [ready[i].elapsed_time(mean_end[i - 1]) for i in range(1, len(ready))]
    wait = float(np.mean([max(0.0, g) for g in gaps])) if gaps else 0.0
    slack = float(np.mean(gaps)) if gaps else 0.0
    tuning = dev.ctx.get_tuning()

    detail = {}
    if not args.no_detail:
        # ---- each kernel alone (nothing else on the GPU) ----
        def alone(fn, n=30):
            dev.ctx.sync(); torch.cuda.synchronize()
            ts = []
            for _ in range(n):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                fn(a, b)
                dev.ctx.sync(); torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            return float(np.median(ts))

        def f_step(a, b):
            a.record(dev.main); dev.ctx.local_step(w.lr); b.record(dev.main)

        t_step = alone(f_step)

        def f_sm(a, b):
            # the pending mean is complete before the clock starts
            dev.ctx.sync()
            a.record(dev.main); dev.ctx.step_merge(w.lr, True); b.record(dev.main)
            dev.ctx.sync()
            dev.ctx.average()

        t_sm = alone(f_sm)

        def f_av(a, b):
            dev.ctx.merge(True)
            dev.ctx.sync()
            a.record(dev.side); dev.ctx.average(); b.record(dev.side)

        t_av = alone(f_av)

        def f_sma(a, b):
            dev.ctx.sync()
            a.record(dev.main); dev.ctx.step_merge_average(w.lr); b.record(dev.main)

        t_sma = alone(f_sma)
        dev.close()
        del dev
        torch.cuda.empty_cache()

        # ---- whole cycles, wall clock: two streams, one stream, one stream with the global update and
        # the next mean fused into one pass (lasgd_step_merge_average), and a HIP-graph replay ----
        def wall(two: bool, fused_mean: bool = False) -> float:
            d = make(side=two)
            d.prologue(w.lr)

            def cyc():
                tau = 0
                for _ in range(w.m):
                    tau = d.iteration(w.lr, tau, w.m, fused_mean=fused_mean)

            for _ in range(args.warmup):
                cyc()
            d.ctx.sync(); torch.cuda.synchronize()
            n = max(10, args.steps // 4)
            t0 = time.perf_counter()
            for _ in range(n):
                cyc()
            d.ctx.sync(); torch.cuda.synchronize()
            out = 1e3 * (time.perf_counter() - t0) / n
            d.close()
            del d
            torch.cuda.empty_cache()
            return out

        ms_two = wall(True)
        ms_serial = wall(False)
        ms_fused_mean = wall(False, fused_mean=True)
        ns = max(10, args.steps // 4)
        gr = make(side=w.side_stream)          # the graph forks to a second stream only where the workload does
        gr.prologue(w.lr)
        gr.ctx.step_merge(w.lr, True)            # close the open cycle: models sent, no mean pending
        graph = gr.capture_cycle(w.lr, w.m)
        with torch.cuda.stream(gr.main):
            for _ in range(args.warmup):
                graph.replay()
        gr.ctx.sync(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(gr.main):
            for _ in range(ns):
                graph.replay()
        gr.ctx.sync(); torch.cuda.synchronize()
        ms_graph = 1e3 * (time.perf_counter() - t0) / ns
        del graph
        gr.close()
        del gr
        torch.cuda.empty_cache()
        # ---- and the fused-mean cycle as a graph on one stream ----
        gf = make(side=False)
        gf.prologue(w.lr)
        for _ in range(w.m - 1):
            gf.ctx.local_step(w.lr)
        gf.ctx.step_merge_average(w.lr)          # from here on z is made on the main stream
        graph = gf.capture_fused_cycle(w.lr, w.m)
        with torch.cuda.stream(gf.main):
            for _ in range(args.warmup):
                graph.replay()
        gf.ctx.sync(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(gf.main):
            for _ in range(ns):
                graph.replay()
        gf.ctx.sync(); torch.cuda.synchronize()
        ms_fused_graph = 1e3 * (time.perf_counter() - t0) / ns
        del graph
        gf.close()
        fused_bytes = (w.m - 1) * alg["local_step"] + alg["step_merge_average"]
        detail = {
            "alone_ms": {"local_step": t_step, "step_merge": t_sm, "average": t_av, "step_merge_average": t_sma},
            "alone_GBps": {"local_step": alg["local_step"] / t_step / 1e6, "step_merge": alg["step_merge"] / t_sm / 1e6,
                           "average": alg["average"] / t_av / 1e6,
                           "step_merge_average": alg["step_merge_average"] / t_sma / 1e6},
            "ms_per_cycle_one_stream": ms_serial,
            "ms_per_cycle_two_streams": ms_two,
            "ms_per_cycle_hip_graph": ms_graph,
            "fused_mean_cycle": {"what": "m-1 local_step + 1 lasgd_step_merge_average on one stream: the sent models are "
                                         "not read back for the mean",
                                 "ms_per_cycle": ms_fused_mean, "ms_per_cycle_hip_graph": ms_fused_graph,
                                 "algorithmic_bytes": fused_bytes,
                                 "GBps_algorithmic": fused_bytes / ms_fused_mean / 1e6,
                                 "params_per_s": w.K * w.N * w.m / ms_fused_mean * 1e3,
                                 "speedup_vs_one_stream": ms_serial / ms_fused_mean},
            "overlap": None if not w.side_stream else {
                "T_avg_alone_ms": t_av, "T_avg_overlapped_ms": kern_ms["average"], "T_wait_ms": wait,
                "mean_ended_before_merge_by_ms": -slack,
                # share of the mean's stand-alone time during which the main stream did not wait for it
                "hidden_frac": 1.0 - min(1.0, wait / t_av),
                # what the overlap buys in cycle time, in units of the mean's stand-alone time (both kernels
                # are HBM-bound on one GPU, so this stays near 0: the bytes are moved either way)
                "time_saved_frac": (ms_serial - ms_two) / t_av,
                "contention_cost": (ms_two - (ms_serial - t_av)) / t_av},
        }
    else:
        dev.close()

    dom = "local_step" if (w.m - 1) * kern_ms.get("local_step", 0.0) >= kern_ms["step_merge"] else "step_merge"
    achieved = alg[dom] / kern_ms[dom] / 1e6          # bytes / ms -> GB/s
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            rec = json.load(open(tpath))
            traffic = rec.get(w.name, {}).get(dom)
            if traffic is not None:
                traffic_source = rec.get("_source")
        except Exception:
            traffic = None
    out = {
        "metric": "params/sec and HBM GB/s (% of peak) for fused LASGD step+merge, K replicas",
        "value": value, "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 storage, f32 arithmetic" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}]: {w.name}, K={w.K} replicas, {len(w.numels)} tensors, "
                               f"{w.N} params/replica, merge every m={w.m} local steps, mean on "
                               f"{'a side stream' if w.side_stream else 'the main stream'}",
                   "step": "one cycle = m-1 local_step + 1 step_merge(resnapshot) + 1 average",
                   "K": w.K, "N": w.N, "m": w.m, "lr": w.lr, "momentum": w.momentum, "weight_decay": w.weight_decay,
                   "nesterov": w.nesterov, "tuning": tuning},
        "cycle_GBps_algorithmic": cycle_bytes / ms_per_step / 1e6,
        "cycle_frac_of_peak": cycle_bytes / ms_per_step / 1e6 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": alg[dom], "avg_launch_ms": kern_ms[dom],
                     "timing": f"HIP events on the kernel's own stream around every launch of {n_inst} cycles issued "
                               f"right after the timed region, same pipelined pattern ({ms_instrumented:.4f} ms per "
                               f"cycle with the events, {ms_per_step:.4f} without)"},
        "kernels_in_instrumented_repeat": {k: {"avg_ms": v, "GBps": alg[k] / v / 1e6, "frac": alg[k] / v / 1e6 / HBM_PEAK_GBS,
                                               "launches": len(ev[k])} for k, v in kern_ms.items()},
        "ms_per_cycle_instrumented": ms_instrumented,
    }
    out.update(detail)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
