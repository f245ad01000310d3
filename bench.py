#!/usr/bin/env python3
"""Benchmark of the DARIS hot path on one MI355X.

Workload (the configuration the headline metric is quoted on): 4 periodic tasks (2 HP, 2 LP), each a ResNet-18
(batch 1, fp32, 3x224x224 ~ N(0,1), random He-init weights, BN folded), 3 stages per DNN, 3 partitions of 128 CUs
(384/256 = 1.5x oversubscribed).

A "step" is one pass of the whole hot path for every task: each task releases one job, which goes through
admission, stage dispatch on the CU-masked streams, the conv/pool/FC kernels and the stage-boundary
synchronisations.  The timed region runs the saturated (closed-loop) variant: every task releases its next job
the instant the previous one finishes, until K steps = K x 4 jobs have been released over all tasks (tasks that
own a partition alone therefore contribute more jobs than the two that share one); value = completed
inferences / wall time.  The periodic
run at the nominal periods (HP 20 ms, LP 40 ms) follows and supplies the deadline-miss rates and response times.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3


def read_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, scaled by
    the copy-kernel calibration); None if the summary does not cover this kernel."""
    path = os.path.join(ROOT, "profiles", "conv_kernels_resnet18_hbm_traffic.md")
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--periodic-jobs", type=int, default=100, help="jobs per task of the periodic (deadline) run; 0 skips it")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the CPU-oracle baseline; 0 skips it")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--sample-every", type=int, default=8, help="kernel timing: bracket the conv launches of every n-th job")
    ap.add_argument("--pmc-pass", action="store_true",
                    help="counter-collection helper for `rocprofv3 --pmc`: three 64 MiB device copies (the known-size reference "
                         "kernel), then 20 forward passes of task 0 alone; prints nothing, times nothing")
    ap.add_argument("--cpu-oracle-report", action="store_true",
                    help="instead of the benchmark: time the CPU oracle alone (forward pass of every network, scheduler model); no GPU")
    args = ap.parse_args()
    if args.cpu_oracle_report:
        return cpu_oracle_report(os.environ.get("OMP_NUM_THREADS", str(os.cpu_count() or 1)))
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    import paper_2504_08795_amd as D
    from paper_2504_08795_amd import harness
    import workloads as wl

    ts = wl.make_taskset(2, n_jobs=max(min(args.steps, 2000), args.periodic_jobs, 1))
    D.daris_init(0, wl.tasksets.SEED, 0)
    for n in ts.partitions:
        D.daris_create_partition(n)
    keep, ins, outs, nets = [], [], [], []
    for i, t in enumerate(ts.tasks):
        layers, shp = wl.build_net(t.net)
        weights = wl.make_weights(layers, t.seed)
        dnn, k = D.make_dnn(layers, weights, shp, t.dtype)
        keep.append(k)
        h = D.daris_register_task(dnn, t.period_ns, t.deadline_ns, t.priority)
        D.daris_split_stages(h, t.n_stages)
        xs = wl.make_inputs(shp, t.seed, ts.n_inputs, t.input_dist)
        nets.append((layers, weights, xs))
        ins.append(torch.from_numpy(xs).cuda())
        outs.append(torch.zeros((ts.n_jobs, layers[-1].c_out), dtype=torch.float32, device="cuda"))
        D.daris_task_set_io(h, ins[i], ts.n_inputs, outs[i], ts.n_jobs)
    nt = len(ts.tasks)
    if args.pmc_pass:
        a = torch.zeros(16 << 20, dtype=torch.float32, device="cuda")      # 64 MiB read + 64 MiB written per copy
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        for _ in range(20):
            D.daris_forward(0, ins[0][0], outs[0][0], 0)
        D.daris_shutdown()
        return
    for i in range(nt):
        D.daris_calibrate_afet(i, i % len(ts.partitions), 3)
    D.daris_commit()

    # ---- saturated run: warm-up, then exactly K steps between synchronisations --------------------------------
    D.daris_run_closed_loop([args.warmup * nt] * nt, args.warmup * nt)
    torch.cuda.synchronize()
    if not args.no_profile:
        D.daris_kernel_timing_start(args.sample_every, 20000)   # dispatch time stamps of every launch of the sampled jobs
    before = [D.daris_get_stats(i) for i in range(nt)]
    t0 = time.perf_counter()
    D.daris_run_closed_loop([args.steps * nt] * nt, args.steps * nt)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    after = [D.daris_get_stats(i) for i in range(nt)]
    timing, pair_ms = (None, 0.0) if args.no_profile else D.daris_kernel_timing_read()
    completed = sum(a["completed"] - b["completed"] for a, b in zip(after, before))
    rejected = sum((a["rejected_admission"] + a["rejected_overrun"]) - (b["rejected_admission"] + b["rejected_overrun"])
                   for a, b in zip(after, before))
    value = completed / elapsed
    # run-level roofline: time the whole chip would need for the completed inferences at each layer's roofline / wall time
    roof_us = harness.taskset_roofline_us(ts)
    run_frac = sum((a["completed"] - b["completed"]) * r for a, b, r in zip(after, before, roof_us)) * 1e-6 / elapsed
    sat_resp_ms = [(a["resp_sum_ns"] - b["resp_sum_ns"]) / max(a["completed"] - b["completed"], 1) / 1e6 for a, b in zip(after, before)]

    # ---- periodic run: the deadline metrics -----------------------------------------------------------------------
    periodic = None
    if args.periodic_jobs > 0:
        b2 = [D.daris_get_stats(i) for i in range(nt)]
        D.trace_read_all()                               # drop the records of the runs above
        tp = time.perf_counter()
        D.daris_run_periodic(None, [args.periodic_jobs] * nt)
        wall = time.perf_counter() - tp
        pct = harness.response_percentiles(D.trace_read_all(), [t.priority for t in ts.tasks])
        a2 = [D.daris_get_stats(i) for i in range(nt)]

        def agg(prio):
            idx = [i for i, t in enumerate(ts.tasks) if t.priority == prio]
            acc = sum(a2[i]["accepted"] - b2[i]["accepted"] for i in idx)
            mis = sum(a2[i]["missed"] - b2[i]["missed"] for i in idx)
            rej = sum((a2[i]["rejected_admission"] + a2[i]["rejected_overrun"]) - (b2[i]["rejected_admission"] + b2[i]["rejected_overrun"]) for i in idx)
            done = sum(a2[i]["completed"] - b2[i]["completed"] for i in idx)
            resp = sum(a2[i]["resp_sum_ns"] - b2[i]["resp_sum_ns"] for i in idx) / max(done, 1) / 1e6
            return dict(accepted=acc, missed=mis, rejected=rej, miss_pct=100.0 * mis / max(acc, 1), mean_response_ms=round(resp, 4),
                        max_response_ms=round(max(a2[i]["resp_max_ns"] for i in idx) / 1e6, 4))
        done_all = sum(a2[i]["completed"] - b2[i]["completed"] for i in range(nt))
        periodic = dict(jobs_per_task=args.periodic_jobs, inferences_per_s=round(done_all / wall, 2), hp=agg(wl.HP), lp=agg(wl.LP),
                        response_ms=pct)

    # ---- roofline of the dominant kernel --------------------------------------------------------------------------------
    # Durations are the start and end time stamps that the command processor of the queue a kernel runs on writes into
    # that dispatch's completion signal (the figures a kernel trace reports), for every launch of each
    # `sample_every`-th job INSIDE the timed region above (three DNNs running concurrently on overlapping
    # partitions).  On a queue that never runs dry a dispatch's start stamp follows its predecessor's end stamp
    # directly, so the ~1.6 us the command processor needs per packet is inside these durations.  FLOPs are the
    # algorithmic 2*MACs of the layers those launches computed.
    roofline = None
    if timing:
        dom = max(timing, key=lambda k: timing[k][1])
        n_launch, t_raw_ms, flops = timing[dom]
        t_ms = max(t_raw_ms - n_launch * pair_ms, 1e-9)   # pair_ms: fixed cost of the timing method, 0 for time stamps
        achieved = flops / (t_ms * 1e-3) / 1e12
        layers = nets[0][0]
        ms, kid, fl = D.daris_profile_layers(0, 0, 20, len(layers))          # the same task alone, for reference
        solo = {}
        for m, k, f in zip(ms, kid, fl):
            e = solo.setdefault(D.daris_kernel_name(int(k)), [0.0, 0])
            e[0] += float(m)
            e[1] += 1
        roofline = dict(bound="mfma", kernel=dom, sampled_launches=n_launch, avg_launch_us=round(t_ms * 1e3 / n_launch, 3),
                        timing="dispatch time stamps in completion signals",
                        achieved=round(achieved, 3), peak=PEAK_FP32_MFMA_TFLOPS, unit="TFLOP/s",
                        frac=round(achieved / PEAK_FP32_MFMA_TFLOPS, 5), traffic=read_traffic(dom),
                        all_sampled_kernels={k: dict(launches=v[0], avg_us=round((v[1] / v[0] - pair_ms) * 1e3, 3)) for k, v in timing.items()},
                        solo_layer_ms_per_inference={k: round(v[0], 4) for k, v in solo.items()},
                        solo_network_kernel_time_ms=round(float(ms.sum()), 4),
                        run=dict(t_roof_us_per_inference=round(roof_us[0], 2), roofline_time_over_wall=round(run_frac, 4)))
    D.daris_shutdown()

    # ---- CPU oracle on the host cores, bounded sample of the same workload ----------------------------------------------------
    cpu = None
    if args.cpu_seconds > 0:
        from oracle import forward as F
        layers, weights, xs = nets[0]
        F.forward(layers, weights, xs[0], "fp32")          # builds / loads the checker, warms the caches
        n, tc = 0, time.perf_counter()
        while time.perf_counter() - tc < args.cpu_seconds:
            F.forward(layers, weights, xs[n % len(xs)], "fp32")
            n += 1
        dt = time.perf_counter() - tc
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = dict(value=round(n / dt, 4), unit="inferences/s", cores=cores, kind="oracle",
                   sample=f"{n} ResNet-18 fp32 forward passes of task 0's seeded inputs ({dt:.1f} s)")

    line = {
        "metric": "aggregate batch-1 inferences/s on 1 MI355X; HP/LP deadline-miss %",
        "value": round(value, 2), "unit": "inferences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * elapsed / args.steps, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "4x ResNet-18 (2 HP + 2 LP), batch 1, fp32, 3x224x224, 3 stages/DNN, 3 partitions x 128 CUs (1.5x oversubscribed), closed-loop releases",
                   "tasks": nt, "partitions": ts.partitions, "stages": 3, "hp_period_ms": 20, "lp_period_ms": 40},
        "saturated": {"completed": completed, "rejected": rejected, "mean_response_ms": [round(v, 4) for v in sat_resp_ms]},
        "hp_miss_pct": None if periodic is None else periodic["hp"]["miss_pct"],
        "lp_miss_pct": None if periodic is None else periodic["lp"]["miss_pct"],
        "periodic": periodic, "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
