#!/usr/bin/env python3
"""Benchmark of the DARIS hot path on one MI355X.

Workload of the headline line: the largest single-GPU configuration, the MIXED set -- 8 periodic tasks (ResNet-18 x2
high-priority; ResNet-50 x2, VGG-16 x2, MobileNetV2 x2 low-priority), batch 1, fp32, 3x224x224 ~ N(0,1), random He-init
weights with folded BN, 3 stages per DNN, 4 partitions of 96/96/128/192 CUs (512/256 = 2x oversubscribed), periods
uniform in [20, 80] ms from the seed.  `--config 2` (4x ResNet-18 fp32 on 3 x 128 CUs) and `--config 3` (6x ResNet-50
bf16 on 4 x 128 CUs) run the same measurement on the other configurations; their saturated figures are also attached to
the default line as `other_configs`.

A "step" is one pass of the whole hot path over one batch of synthetic input: JOBS_PER_TASK_PER_STEP jobs of every task,
each going through admission, stage dispatch on the CU-masked queues, the conv / depthwise / pool / FC kernels and the
stage-boundary synchronisations.  The timed region runs the saturated (closed-loop) variant: every task releases its next
job the instant the previous one finishes, until K steps' worth of jobs have been released over all tasks together (tasks
in faster partitions therefore contribute more jobs); value = completed inferences / wall time, median of `--repeats`
timed regions of K steps each (all reported).  The periodic run at the nominal periods follows and supplies the
deadline-miss rates and response times.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = {"f32": 157.3, "bf16": 2500.0}     # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0
JOBS_PER_TASK_PER_STEP = 32
WORKLOADS = {
    2: "4x ResNet-18 (2 HP + 2 LP), batch 1, fp32, 3x224x224, 3 stages/DNN, 3 partitions x 128 CUs (1.5x oversubscribed), closed-loop releases",
    3: "6x ResNet-50 (2 HP + 4 LP), batch 1, bf16 storage / fp32 accumulate, 3x224x224, 4 stages/DNN, 4 partitions x 128 CUs (2x oversubscribed), closed-loop releases",
    4: "mixed 8 tasks: ResNet-18 x2 (HP), ResNet-50 x2, VGG-16 x2, MobileNetV2 x2 (LP), batch 1, fp32, 3x224x224, 3 stages/DNN, partitions 96/96/128/192 CUs (2x oversubscribed), closed-loop releases",
}
TRAFFIC_PROFILE = {2: "bench_config2_hbm_traffic.md", 3: "bench_config3_hbm_traffic.md", 4: "bench_config4_hbm_traffic.md"}


def read_traffic(config, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this configuration (FETCH_SIZE +
    WRITE_SIZE, scaled by the copy-kernel calibration); None if no summary covers this kernel."""
    path = os.path.join(ROOT, "profiles", TRAFFIC_PROFILE[config])
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch[") and line.split("[")[1].split("]")[0] == kernel:
                return int(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_oracle_report(threads_note):
    """The CPU side of the measurement on its own: the oracle's forward pass per network (median of 3, on the threads
    OMP_NUM_THREADS allows) and the oracle's discrete-event scheduler model in events/s.  No GPU is touched."""
    import numpy as np
    import workloads as wl
    from oracle import des
    from oracle import forward as F
    nets = {}
    for net, dtype in (("tiny", "fp32"), ("resnet18", "fp32"), ("resnet50", "bf16"), ("mobilenet_v2", "fp32"), ("vgg16", "fp32")):
        layers, shp = wl.build_net(net)
        weights = wl.make_weights(layers, 1)
        x = wl.make_inputs(shp, 1, 1, "normal")[0]
        F.forward(layers, weights, x, dtype)             # builds / loads the checker, warms the caches
        ts = []
        for _ in range(3):
            t0 = time.perf_counter()
            F.forward(layers, weights, x, dtype)
            ts.append(time.perf_counter() - t0)
            print(f"oracle {net} {dtype}: {ts[-1]:.3f} s", file=sys.stderr, flush=True)
        nets[f"{net}_{dtype}"] = round(1.0 / float(np.median(ts)), 4)
    # scheduler model: config 2 in virtual time, 400 jobs per task
    tset = wl.make_taskset(2, n_jobs=400)
    et = wl.virtual_et_table(tset, load_scale=25.0)
    afet = [[int(np.mean(et[i][j][0][:8])) for j in range(t.n_stages)] for i, t in enumerate(tset.tasks)]
    model = des.SchedulerModel([1] * len(tset.partitions), [des.TaskParam(t.period_ns, t.deadline_ns, t.priority, afet[i]) for i, t in enumerate(tset.tasks)])
    cmds = [("release", t, i) for t, i, _ in tset.releases()]
    t0 = time.perf_counter()
    trace = des.run_virtual(model, cmds, et)
    dt = time.perf_counter() - t0
    print(json.dumps({"cpu_oracle": {"threads": threads_note, "forward_inferences_per_s": nets,
                                     "scheduler_model_trace_records_per_s": round(len(trace) / dt, 1), "scheduler_model_trace_records": len(trace)}}))


def kernel_roofline(name, launches, ms, flops):
    """Roofline entry of one kernel from its sampled launches: MFMA-bound convolutions against the dense peak of their
    arithmetic type; memory-bound kernels against HBM (the caller fills in the FC kernel's rate: its bytes are the
    weights it streams, one element per MAC)."""
    t_s = max(ms, 1e-9) * 1e-3
    if name.startswith("conv_wave"):
        dt = "bf16" if "_bf16_" in name else "f32"
        achieved, peak, unit, bound = flops / t_s / 1e12, PEAK_MFMA_TFLOPS[dt], "TFLOP/s", "mfma"
    else:
        achieved, peak, unit, bound = None, PEAK_HBM_GBS, "GB/s", "hbm"
    return dict(bound=bound, kernel=name, sampled_launches=launches, avg_launch_us=round(ms * 1e3 / max(launches, 1), 3),
                achieved=None if achieved is None else round(achieved, 3), peak=peak, unit=unit,
                frac=None if achieved is None else round(achieved / peak, 5))


def measure(config, args, full):
    """One configuration: saturated throughput (median of args.repeats timed regions of args.steps steps), and, when
    `full`, the periodic run (deadline metrics), the sampled per-kernel timings and the solo layer profile."""
    import numpy as np
    import torch
    import paper_2504_08795_amd as D
    from paper_2504_08795_amd import harness
    import workloads as wl

    ts = wl.make_taskset(config, n_jobs=64)
    g = harness.GpuTaskSet(ts, flags=args.flags, seed=wl.tasksets.SEED, plan_cus=args.plan_cus)
    nt = g.n_tasks
    try:
        g.calibrate(3)
        D.daris_commit()
        per_step = nt * JOBS_PER_TASK_PER_STEP
        if args.warmup > 0:
            D.daris_run_closed_loop([args.warmup * per_step] * nt, args.warmup * per_step)
        torch.cuda.synchronize()
        if full and not args.no_profile:
            D.daris_kernel_timing_start(args.sample_every, 200000)   # dispatch time stamps of every launch of the sampled jobs
        roof_us = harness.taskset_roofline_us(ts)
        runs = []
        for _ in range(max(args.repeats, 1)):
            before = g.stats()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            D.daris_run_closed_loop([args.steps * per_step] * nt, args.steps * per_step)
            torch.cuda.synchronize()
            elapsed = time.perf_counter() - t0
            after = g.stats()
            done = [a["completed"] - b["completed"] for a, b in zip(after, before)]
            rej = sum((a["rejected_admission"] + a["rejected_overrun"]) - (b["rejected_admission"] + b["rejected_overrun"]) for a, b in zip(after, before))
            resp = [(a["resp_sum_ns"] - b["resp_sum_ns"]) / max(d, 1) / 1e6 for a, b, d in zip(after, before, done)]
            runs.append(dict(elapsed=elapsed, completed=sum(done), per_task=done, rejected=rej, value=sum(done) / elapsed,
                             mean_response_ms=[round(v, 4) for v in resp],
                             roofline_time_over_wall=sum(d * r for d, r in zip(done, roof_us)) * 1e-6 / elapsed))
        timing, pair_ms = (None, 0.0) if (not full or args.no_profile) else D.daris_kernel_timing_read()
        med = sorted(runs, key=lambda r: r["value"])[len(runs) // 2]
        out = dict(config=config, workload=WORKLOADS[config], tasks=nt, partitions=ts.partitions, plan_cus=g.plan_cus, stages=[t.n_stages for t in ts.tasks],
                   nets=[t.net for t in ts.tasks], dtype=ts.tasks[0].dtype,
                   periods_ms=[round(t.period_ns / 1e6, 3) for t in ts.tasks], value=med["value"], elapsed=med["elapsed"],
                   values=[round(r["value"], 2) for r in runs],
                   spread_pct=round(100.0 * (max(r["value"] for r in runs) - min(r["value"] for r in runs)) / med["value"], 2),
                   saturated=dict(completed=med["completed"], completed_per_task=med["per_task"], rejected=med["rejected"],
                                  mean_response_ms=med["mean_response_ms"], roofline_time_over_wall=round(med["roofline_time_over_wall"], 4)),
                   t_roof_us_per_inference=[round(v, 2) for v in roof_us])
        if not full:
            return out, None

        # ---- periodic run: the deadline metrics ---------------------------------------------------------------------
        periodic = None
        if args.periodic_jobs > 0:
            D.trace_read_all()                               # drop the records of the runs above
            res = harness.run_periodic(g, args.periodic_jobs)
            res["response_ms"] = harness.response_percentiles(D.trace_read_all(), [t.priority for t in ts.tasks])
            res["jobs_per_task"] = args.periodic_jobs
            periodic = res
        out["periodic"] = periodic

        # ---- roofline of the dominant kernel ---------------------------------------------------------------------------
        # Durations are the start and end time stamps that the command processor of the queue a kernel runs on writes into
        # that dispatch's completion signal (the figures a kernel trace reports), for every launch of each
        # `sample_every`-th job INSIDE the timed regions above (all tasks running concurrently on overlapping partitions).
        # On a queue that never runs dry a dispatch's start stamp follows its predecessor's end stamp directly, so the
        # ~1.6 us the command processor needs per packet is inside these durations.  FLOPs are the algorithmic 2*MACs of
        # the layers those launches computed.
        roofline = None
        if timing:
            dom = max(timing, key=lambda k: timing[k][1])
            n_launch, t_ms, flops = timing[dom]
            roofline = kernel_roofline(dom, n_launch, t_ms, flops)
            if roofline["achieved"] is None and dom == "fc":
                es = 2 if ts.tasks[0].dtype == "bf16" else 4
                gbs = flops / 2 * es / (t_ms * 1e-3) / 1e9
                roofline.update(achieved=round(gbs, 1), frac=round(gbs / PEAK_HBM_GBS, 5))
            roofline["timing"] = "dispatch time stamps in completion signals, sampled inside the timed regions"
            roofline["traffic"] = read_traffic(config, dom)
            per_kernel = {}
            for k, (n, ms, fl) in timing.items():
                e = kernel_roofline(k, n, ms, fl)
                per_kernel[k] = dict(launches=n, avg_us=e["avg_launch_us"], share_of_sampled_time=round(ms / sum(v[1] for v in timing.values()), 4))
                if e["achieved"] is not None:
                    per_kernel[k].update(achieved=e["achieved"], unit=e["unit"], frac=e["frac"])
            roofline["all_sampled_kernels"] = per_kernel
            conv = [(k, v) for k, v in timing.items() if k.startswith("conv_wave")]
            if conv:
                dt = "bf16" if "_bf16_" in conv[0][0] else "f32"
                cf, cms = sum(v[2] for _, v in conv), sum(v[1] for _, v in conv)
                roofline["all_conv_kernels"] = dict(achieved=round(cf / (cms * 1e-3) / 1e12, 3), unit="TFLOP/s", peak=PEAK_MFMA_TFLOPS[dt],
                                                    frac=round(cf / (cms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS[dt], 5))
            roofline["run"] = dict(roofline_time_over_wall=round(med["roofline_time_over_wall"], 4))
        return out, roofline
    finally:
        g.close()


def cpu_baseline(config, seconds):
    """The oracle's forward pass, as it stands, on the host cores: rounds of one inference of every distinct network of
    the configuration (the per-task mix of one step), for about `seconds` seconds."""
    import workloads as wl
    from oracle import forward as F
    ts = wl.make_taskset(config, n_jobs=1)
    seen, work = set(), []
    for t in ts.tasks:
        if (t.net, t.dtype) in seen:
            continue
        seen.add((t.net, t.dtype))
        layers, shp = wl.build_net(t.net)
        work.append((t.net, t.dtype, layers, wl.make_weights(layers, t.seed), wl.make_inputs(shp, t.seed, 1, t.input_dist)[0]))
    F.forward(work[0][2], work[0][3], work[0][4], work[0][1])          # builds / loads the checker, warms the caches
    rounds, tc = 0, time.perf_counter()
    while rounds == 0 or time.perf_counter() - tc < seconds:
        for w in work:
            F.forward(w[2], w[3], w[4], w[1])
        rounds += 1
    dt = time.perf_counter() - tc
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    nets = ", ".join(f"{w[0]} {w[1]}" for w in work)
    return dict(value=round(rounds * len(work) / dt, 4), unit="inferences/s", cores=cores, kind="oracle",
                sample=f"{rounds} rounds of one forward pass of each distinct network of the configuration ({nets}) = {rounds * len(work)} inferences in {dt:.1f} s")


def pmc_pass(config):
    """Counter-collection helper for `rocprofv3 --pmc`: three 64 MiB device copies (the known-size reference kernel), then
    10 forward passes of each distinct network of the configuration, alone on the partition it is assigned to."""
    import torch
    import paper_2504_08795_amd as D
    from paper_2504_08795_amd import harness
    import workloads as wl
    ts = wl.make_taskset(config, n_jobs=4)
    g = harness.GpuTaskSet(ts, seed=wl.tasksets.SEED)
    try:
        a = torch.zeros(16 << 20, dtype=torch.float32, device="cuda")      # 64 MiB read + 64 MiB written per copy
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        seen = set()
        for i, t in enumerate(ts.tasks):
            if (t.net, t.dtype) in seen:
                continue
            seen.add((t.net, t.dtype))
            for _ in range(10):
                D.daris_forward(i, g.inputs[i][0], g.logits[i][0], i % len(ts.partitions))
    finally:
        g.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, choices=(2, 3, 4), help="configuration of the headline line (default: the mixed set)")
    ap.add_argument("--other-configs", default="2,3", help="configurations whose saturated figure is attached as other_configs ('' = none)")
    ap.add_argument("--plan-cus", type=int, default=0, help="partition size the launch plans are balanced for (0: the partitions' size when all "
                    "are equal, else 128)")
    ap.add_argument("--repeats", type=int, default=3, help="timed regions of --steps steps each; the median is the value")
    ap.add_argument("--periodic-jobs", type=int, default=40, help="jobs per task of the periodic (deadline) run; 0 skips it")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the CPU-oracle baseline; 0 skips it")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--sample-every", type=int, default=8, help="kernel timing: time stamps for the launches of every n-th job")
    ap.add_argument("--flags", type=int, default=0, help="extra daris_init flags (A/B switches of daris.h)")
    ap.add_argument("--pmc-pass", action="store_true",
                    help="counter-collection helper for `rocprofv3 --pmc` (see pmc_pass); prints nothing, times nothing")
    ap.add_argument("--cpu-oracle-report", action="store_true",
                    help="instead of the benchmark: time the CPU oracle alone (forward pass of every network, scheduler model); no GPU")
    args = ap.parse_args()
    if args.cpu_oracle_report:
        return cpu_oracle_report(os.environ.get("OMP_NUM_THREADS", str(os.cpu_count() or 1)))
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
    if args.pmc_pass:
        return pmc_pass(args.config)

    main_res, roofline = measure(args.config, args, full=True)
    others = {}
    for c in [int(v) for v in args.other_configs.split(",") if v.strip()]:
        if c == args.config:
            continue
        r, _ = measure(c, args, full=False)
        others[str(c)] = dict(workload=r["workload"], value=round(r["value"], 2), unit="inferences/s", values=r["values"], dtype=r["dtype"],
                              roofline_time_over_wall=r["saturated"]["roofline_time_over_wall"])
    cpu = cpu_baseline(args.config, args.cpu_seconds) if args.cpu_seconds > 0 else None

    periodic = main_res.get("periodic")
    line = {
        "metric": "aggregate batch-1 inferences/s on 1 MI355X; HP/LP deadline-miss %",
        "value": round(main_res["value"], 2), "unit": "inferences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * main_res["elapsed"] / args.steps, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if main_res["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": main_res["workload"], "baseline_config": args.config, "tasks": main_res["tasks"], "nets": main_res["nets"],
                   "partitions": main_res["partitions"], "plan_cus": main_res["plan_cus"], "stages": main_res["stages"], "periods_ms": main_res["periods_ms"],
                   "jobs_per_step": main_res["tasks"] * JOBS_PER_TASK_PER_STEP},
        "repeats": {"values": main_res["values"], "spread_pct": main_res["spread_pct"], "value_is": "median"},
        "saturated": main_res["saturated"],
        "hp_miss_pct": None if periodic is None else periodic["hp"]["miss_pct"],
        "lp_miss_pct": None if periodic is None else periodic["lp"]["miss_pct"],
        "periodic": periodic, "roofline": roofline, "cpu_baseline": cpu, "other_configs": others,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
