"""Experiment driver (the paper's Sec. V protocol on this library): builds a task set on the GPU, runs it
periodically or saturated, and reports jobs/s, deadline-miss rates (missed / accepted) and response times.

    python -m paper_2504_08795_amd.harness --config 2 --jobs 200
    python -m paper_2504_08795_amd.harness --config 5 --rate 1.5 --oversub 2.0 --jobs 100 --migrate-every 100

Only argument marshalling and bookkeeping live here; every step of the path runs inside libdaris.so.
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np

from . import binding as D


class GpuTaskSet:
    """Registers every task of a `workloads.TaskSet` (weights, stages, I/O pools) on device 0."""

    def __init__(self, ts, flags=0, afet=None, streams_per_partition=None, seed=0, plan_cus=0):
        """plan_cus: partition size the launch plans are balanced for; 0 = the partitions' size when they are all equal,
        else the library's default of 128 (measured on the mixed 96/96/128/192 set: plans for 96 CUs gain 6 % on the 96-CU
        partitions and lose 10 % on the 128-CU one, 0.5 % less in total)."""
        import torch
        import workloads as wl
        self.ts = ts
        D.daris_init(0, seed, flags)
        self.plan_cus = plan_cus or (ts.partitions[0] if len(set(ts.partitions)) == 1 else 128)
        D.daris_set_plan_cus(self.plan_cus)
        ns = streams_per_partition or ts.streams_per_partition
        for n in ts.partitions:
            p = D.daris_create_partition(n)
            if ns != 1:
                D.daris_partition_set_streams(p, ns)
        self.keep, self.inputs, self.logits, self.nets = [], [], [], []
        cache = {}
        for i, t in enumerate(ts.tasks):
            layers, shp = wl.build_net(t.net)
            if (t.net, t.seed) not in cache:
                cache[(t.net, t.seed)] = wl.make_weights(layers, t.seed)
            weights = cache[(t.net, t.seed)]
            dnn, keep = D.make_dnn(layers, weights, shp, t.dtype)
            h = D.daris_register_task(dnn, t.period_ns, t.deadline_ns, t.priority)
            assert h == i
            D.daris_split_stages(h, t.n_stages)
            xs = wl.make_inputs(shp, t.seed, ts.n_inputs, t.input_dist)
            self.nets.append((layers, weights, xs, t.dtype))
            self.inputs.append(torch.from_numpy(xs).cuda())
            self.logits.append(torch.full((ts.n_jobs, layers[-1].c_out), float("nan"), dtype=torch.float32, device="cuda"))
            D.daris_task_set_io(h, self.inputs[i], ts.n_inputs, self.logits[i], ts.n_jobs)
            if afet is not None:
                for j, a in enumerate(afet[i]):
                    D.daris_set_afet(h, j, a)
            del keep
        self.n_tasks = len(ts.tasks)

    def calibrate(self, reps=3, loaded=False):
        """AFET of every stage, each task on partition (index mod N_c), alone or (Sec. IV-A1) while the other
        streams run other tasks; returns the values."""
        for i in range(self.n_tasks):
            (D.daris_calibrate_afet_loaded if loaded else D.daris_calibrate_afet)(i, i % len(self.ts.partitions), reps)
        return [[D.daris_get_mret(i, j) for j in range(t.n_stages)] for i, t in enumerate(self.ts.tasks)]

    def stats(self):
        return [D.daris_get_stats(i) for i in range(self.n_tasks)]

    def close(self):
        D.daris_shutdown()


def summarise(ts, before, after, wall_s):
    """Per-priority metrics between two `stats()` snapshots."""
    out = {}
    for name, prio in (("hp", 1), ("lp", 0)):
        idx = [i for i, t in enumerate(ts.tasks) if t.priority == prio]
        d = lambda k: sum(after[i][k] - before[i][k] for i in idx)  # noqa: E731
        acc, done = d("accepted"), d("completed")
        out[name] = dict(released=d("released"), accepted=acc, completed=done, missed=d("missed"),
                         rejected_admission=d("rejected_admission"), rejected_overrun=d("rejected_overrun"),
                         miss_pct=100.0 * d("missed") / max(acc, 1),
                         mean_response_ms=round(d("resp_sum_ns") / max(done, 1) / 1e6, 4),
                         max_response_ms=round(max([after[i]["resp_max_ns"] for i in idx] or [0]) / 1e6, 4))
    total = sum(after[i]["completed"] - before[i]["completed"] for i in range(len(ts.tasks)))
    out["completed"] = total
    out["inferences_per_s"] = round(total / wall_s, 2)
    out["wall_s"] = round(wall_s, 4)
    # what the whole chip would need for the completed inferences at its rooflines, over the wall time
    roof = taskset_roofline_us(ts)
    out["roofline_time_over_wall"] = round(sum((after[i]["completed"] - before[i]["completed"]) * roof[i] for i in range(len(ts.tasks))) * 1e-6 / wall_s, 4)
    return out


def response_percentiles(trace, priorities):
    """Per-priority response times (ms) of the jobs that completed inside `trace` (list of record tuples): a job's
    response = its JOB_DONE time - its nominal release (RELEASE time - the lateness stored in aux)."""
    RELEASE, JOB_DONE = 1, 7
    rel, resp = {}, {0: [], 1: []}
    for seq, t, typ, level, stage, part, task, stream, job, aux in trace:
        if typ == RELEASE:
            rel[(task, job)] = t - aux
        elif typ == JOB_DONE and (task, job) in rel:
            resp[priorities[task]].append((t - rel.pop((task, job))) / 1e6)
    out = {}
    for name, prio in (("hp", 1), ("lp", 0)):
        v = np.sort(np.asarray(resp[prio]))
        out[name] = None if len(v) == 0 else dict(jobs=int(len(v)), min_ms=round(float(v[0]), 4), p50_ms=round(float(np.percentile(v, 50)), 4),
                                                  p99_ms=round(float(np.percentile(v, 99)), 4), max_ms=round(float(v[-1]), 4))
    return out


def run_periodic(g: GpuTaskSet, n_jobs, migrate_every=0, seed=1):
    """Periodic releases at the nominal periods.  With migrate_every > 0 the run is cut into chunks and a seeded LP
    task is forced to a seeded other partition between chunks (one migration per `migrate_every` completed jobs)."""
    ts = g.ts
    before = g.stats()
    t0 = time.perf_counter()
    if migrate_every <= 0:
        D.daris_run_periodic(None, [n_jobs] * g.n_tasks)
    else:
        rng = np.random.Generator(np.random.PCG64(seed))
        lp = [i for i, t in enumerate(ts.tasks) if t.priority == 0]
        chunk = max(1, migrate_every // g.n_tasks)
        done = 0
        while done < n_jobs:
            step = min(chunk, n_jobs - done)
            D.daris_run_periodic(None, [step] * g.n_tasks)
            done += step
            if lp and done < n_jobs:
                t = int(rng.choice(lp))
                cur = D.daris_get_partition(t)
                others = [p for p in range(len(ts.partitions)) if p != cur]
                if others:
                    D.daris_migrate(t, int(rng.choice(others)))
    wall = time.perf_counter() - t0
    return summarise(ts, before, g.stats(), wall)


def run_saturated(g: GpuTaskSet, total_jobs, driver_profile=False):
    before = g.stats()
    if driver_profile:
        D.daris_driver_profile(True)
    t0 = time.perf_counter()
    D.daris_run_closed_loop([total_jobs] * g.n_tasks, total_jobs)
    wall = time.perf_counter() - t0
    res = summarise(g.ts, before, g.stats(), wall)
    if driver_profile:
        pr = D.daris_driver_profile(False)
        n = max(pr["stages"], 1)
        res["driver_profile_us_per_stage"] = {k[:-3]: round(v / n / 1e3, 2) for k, v in pr.items() if k != "stages"}
        res["driver_profile_us_per_stage"]["stages"] = pr["stages"]
        res["driver_profile_us_per_stage"]["wall_us"] = round(wall * 1e6, 1)
    return res


PEAK_TFLOPS = {"fp32": 157.3, "bf16": 2500.0}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0


def layer_rooflines(layers, shp, dtype):
    """Per layer: (algorithmic FLOPs, algorithmic bytes, t_roof in us on the whole chip).  Bytes = weights once + one fp32
    bias per output channel + the input tensor(s) read once + the output written once, at the element size of the task;
    FLOPs = 2 x MACs; t_roof = max(FLOPs / dense MFMA peak of the dtype, bytes / HBM peak).  Host arithmetic on the layer
    table only."""
    import workloads as wl
    es = 4 if dtype == "fp32" else 2
    shapes = wl.layer_shapes(layers, shp)
    macs = wl.net_macs(layers, shp)
    out = []
    for l, L in enumerate(layers):
        c, h, w = shapes[l]
        ci, hi, wi = shp if L.in_from < 0 else shapes[L.in_from]
        if L.op == wl.nets.OP_CONV:
            w_elems, b_elems = L.c_out * (L.c_in // L.groups) * L.k * L.k, L.c_out
        elif L.op == wl.nets.OP_FC:
            w_elems, b_elems = L.c_out * L.c_in, L.c_out
        else:
            w_elems = b_elems = 0
        by = w_elems * es + b_elems * 4 + ci * hi * wi * es + c * h * w * es
        if L.res_from >= 0:
            by += c * h * w * es
        fl = 2.0 * macs[l]
        out.append((fl, by, max(fl / (PEAK_TFLOPS[dtype] * 1e12), by / (PEAK_HBM_GBS * 1e9)) * 1e6))
    return out


def taskset_roofline_us(ts):
    """Sum of layer rooflines (whole chip) of one inference of each task of a task set, us."""
    import workloads as wl
    cache, out = {}, []
    for t in ts.tasks:
        if (t.net, t.dtype) not in cache:
            layers, shp = wl.build_net(t.net)
            cache[(t.net, t.dtype)] = sum(r[2] for r in layer_rooflines(layers, shp, t.dtype))
        out.append(cache[(t.net, t.dtype)])
    return out


def layer_profile(net, dtype, n_cu, reps=50, plan_cus=0):
    """Every layer of one DNN alone on an n_cu partition: kernel, time, and its roofline.  Algorithmic bytes of a layer =
    its weights and biases once + its input tensor(s) read once + its output written once (element size of the
    task); algorithmic FLOPs = 2 x MACs.  t_roof = max(FLOPs / MFMA peak of the dtype, bytes / HBM peak), whole chip."""
    import torch
    import workloads as wl
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, 1)
    es = 4 if dtype == "fp32" else 2
    D.daris_init(0, 0, 0)
    try:
        if plan_cus:
            D.daris_set_plan_cus(plan_cus)
        p = D.daris_create_partition(n_cu)
        dnn, keep = D.make_dnn(layers, weights, shp, dtype)
        t = D.daris_register_task(dnn, 10**7, 10**7, 0)
        x = torch.from_numpy(wl.make_inputs(shp, 1, 1, "normal")[0]).cuda()
        y = torch.zeros(layers[-1].c_out, device="cuda")
        D.daris_forward(t, x, y, p)
        ms, kid, fl = D.daris_profile_layers(t, p, reps, len(layers))
        plans = [D.daris_get_launch_plan(t, l) for l in range(len(layers))]
        # one job after the other through the scheduler (one stage per job, buffers of an I/O pool): the production path
        xs = x.unsqueeze(0).contiguous()
        ys = torch.zeros(4, layers[-1].c_out, device="cuda")
        torch.cuda.synchronize()
        D.daris_task_set_io(t, xs, 1, ys, 4)
        D.daris_calibrate_afet(t, p, 2)
        D.daris_run_closed_loop([20], 0)
        t0 = time.perf_counter()
        D.daris_run_closed_loop([200], 0)
        latency_us = (time.perf_counter() - t0) / 200 * 1e6
    finally:
        D.daris_shutdown()
    shapes = wl.layer_shapes(layers, shp)
    roofs = layer_rooflines(layers, shp, dtype)
    rows = []
    for l, L in enumerate(layers):
        c, h, w = shapes[l]
        by, t_roof = roofs[l][1], roofs[l][2]
        assert roofs[l][0] == fl[l], (l, roofs[l][0], fl[l])      # the library counts the same MACs as the layer table
        us = float(ms[l]) * 1e3
        rows.append(dict(layer=l, name=L.name, kernel=D.daris_kernel_name(kid[l]), M=h * w, N=c, us=round(us, 2),
                         gflop=round(fl[l] / 1e9, 4), mbytes=round(by / 1e6, 3),
                         tflops=round(fl[l] / us / 1e6, 2) if us > 0.2 else None, gbs=round(by / us / 1e3, 1) if us > 0.2 else None,
                         bound="mfma" if fl[l] / (PEAK_TFLOPS[dtype] * 1e12) > by / (PEAK_HBM_GBS * 1e9) else "hbm",
                         t_roof_us=round(t_roof, 3), frac=round(t_roof / us, 4) if us > 0.2 else None,
                         joint_launch_with=plans[l]["pair_with"] if plans[l]["pair_with"] >= 0 else None))
    return dict(net=net, dtype=dtype, n_cu=n_cu, kernel_time_us=round(float(sum(r["us"] for r in rows)), 1), job_latency_us=round(latency_us, 1),
                t_roof_us=round(sum(r["t_roof_us"] for r in rows), 2), layers=rows)


def queue_scaling(net, dtype, n_max=8, jobs_per_task=150, n_stages=3):
    """Separates the number of concurrently fed hardware queues from the size of their partitions: the same DNN as N
    tasks on N partitions with one stream each, N = 1..n_max, once with equal DISJOINT masks of 256 / n_max CUs and once
    with every partition on the full 256-CU mask; saturated closed loop.  Per row: aggregate inferences/s, and per stage
    the GPU span (first kernel's start stamp to last kernel's end stamp) and the host's share of the wall time."""
    import workloads as wl
    rows = []
    for shape in ("disjoint", "full"):
        for n in range(1, n_max + 1):
            n_cu = 256 // n_max if shape == "disjoint" else 256
            period = 10_000_000
            tasks = [wl.TaskSpec(net, dtype, wl.LP, period, period, n_stages, wl.tasksets.SEED + 90_000) for _ in range(n)]
            ts = wl.TaskSet(f"queues_{shape}_{n}", tasks, [n_cu] * n, 8, n_inputs=1)
            g = GpuTaskSet(ts)
            try:
                g.calibrate(2)
                D.daris_commit()
                assert sorted(D.daris_get_partition(i) for i in range(n)) == list(range(n))      # one task per partition
                D.daris_run_closed_loop([20] * n, 0)
                res = run_saturated(g, jobs_per_task * n, driver_profile=True)
                pr = res["driver_profile_us_per_stage"]
                rows.append(dict(masks=shape, queues=n, cus_per_queue=n_cu, inferences_per_s=res["inferences_per_s"],
                                 per_queue=round(res["inferences_per_s"] / n, 1), gpu_span_us=pr["gpu"],
                                 stage_wall_us=round(pr["wall_us"] * n / max(pr["stages"], 1), 2)))
            finally:
                g.close()
    return rows


def stress_sweep(jobs, rates=(0.5, 0.75, 1.0, 1.5, 2.0, 2.5, 3.0), oversubs=(1.0, 1.5, 2.0, 2.5), migrate_every=100):
    """Configuration 5: 4 HP ResNet-50 (bf16) + 12 LP MobileNetV2 / ResNet-18 (fp32) tasks on four equal partitions, the
    release rate scaled from 0.5x to 3x of the nominal 40 / 80 ms periods and the oversubscription level from 1.0 to
    2.5 (64 / 96 / 128 / 160 CUs per partition), one forced migration per `migrate_every` completed jobs.  One row per
    point; the sweep of a level stops after the first rate whose LP miss rate exceeds 2 %."""
    import workloads as wl
    rows = []
    for osub in oversubs:
        for rate in rates:
            ts = wl.make_taskset(5, n_jobs=jobs, rate_scale=rate, oversub=osub)
            ts.n_inputs = 1
            g = GpuTaskSet(ts)
            try:
                g.calibrate(2)
                D.daris_commit()
                res = run_periodic(g, jobs, migrate_every)
                pct = response_percentiles(D.trace_read_all(), [t.priority for t in ts.tasks])
            finally:
                g.close()
            rows.append(dict(oversub=osub, cus=ts.partitions[0], rate=rate, offered=round(sum(1e9 / t.period_ns for t in ts.tasks), 1),
                             served=res["inferences_per_s"], hp_miss=round(res["hp"]["miss_pct"], 2), lp_miss=round(res["lp"]["miss_pct"], 2),
                             lp_rejected=res["lp"]["rejected_admission"] + res["lp"]["rejected_overrun"],
                             hp_p99=pct["hp"]["p99_ms"] if pct["hp"] else None, lp_p99=pct["lp"]["p99_ms"] if pct["lp"] else None))
            print(json.dumps(rows[-1]), flush=True)
            if rows[-1]["lp_miss"] > 2.0:
                break
    return rows


def main():
    import workloads as wl
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--jobs", type=int, default=100, help="jobs per task (periodic) / total jobs x tasks (saturated)")
    ap.add_argument("--rate", type=float, default=1.0, help="config 5: release-rate scale")
    ap.add_argument("--oversub", type=float, default=2.0, help="config 5: oversubscription level")
    ap.add_argument("--streams", type=int, default=1, help="streams per partition (N_s)")
    ap.add_argument("--stages", type=int, default=0, help="override the stage count of every task (1 = no staging)")
    ap.add_argument("--flags", default="", help="comma list of no_last,no_prior,no_fixed,hp_admission,wave_prio,shared_queue")
    ap.add_argument("--migrate-every", type=int, default=0)
    ap.add_argument("--saturated", action="store_true")
    ap.add_argument("--driver-profile", action="store_true", help="--saturated: where a stage's wall time goes")
    ap.add_argument("--loaded-afet", action="store_true", help="AFET measured while the other streams run other tasks (Sec. IV-A1)")
    ap.add_argument("--paper-set", default="", help="Table-II-shaped set of this DNN type instead of --config (e.g. resnet18)")
    ap.add_argument("--n-high", type=int, default=17)
    ap.add_argument("--n-low", type=int, default=34)
    ap.add_argument("--task-jps", type=float, default=30.0, help="jobs per second released by every task of a --paper-set")
    ap.add_argument("--nc", type=int, default=6, help="--paper-set: number of partitions N_c")
    ap.add_argument("--os", default="2", help="--paper-set: oversubscription OS as a fraction, e.g. 3/2 (1 <= OS <= N_c)")
    ap.add_argument("--layer-profile", default="", help="instead of a run: per-layer kernel times and rooflines of this DNN alone (e.g. resnet18)")
    ap.add_argument("--dtype", default="fp32", help="--layer-profile and --paper-set: fp32 | bf16")
    ap.add_argument("--ncu", type=int, default=128, help="--layer-profile: partition size")
    ap.add_argument("--table", action="store_true", help="--layer-profile: markdown table instead of JSON")
    ap.add_argument("--plan-cus", type=int, default=0, help="partition size the launch plans are balanced for (0: --layer-profile keeps the library's 128; "
                    "task sets use their partitions' size when all are equal)")
    ap.add_argument("--queue-scaling", default="", help="instead of a run: this DNN on 1..8 queues with disjoint 32-CU masks and with full masks (markdown table)")
    ap.add_argument("--stress-sweep", action="store_true", help="instead of a run: configuration 5 over release rate x oversubscription (--jobs per task and point)")
    ap.add_argument("--rates", default="0.5,0.75,1,1.5,2,2.5,3", help="--stress-sweep: release-rate scales (the configuration's range is 0.5 to 3; larger values look for the knee)")
    ap.add_argument("--oversubs", default="1,1.5,2,2.5", help="--stress-sweep: oversubscription levels")
    a = ap.parse_args()
    if a.stress_sweep:
        rows = stress_sweep(a.jobs, tuple(float(v) for v in a.rates.split(",")), tuple(float(v) for v in a.oversubs.split(",")))
        print("\n| OS | CUs per partition | rate | offered inf/s | served inf/s | HP miss % | LP miss % | LP rejected | HP p99 ms | LP p99 ms |\n|---|---|---|---|---|---|---|---|---|---|")
        for r in rows:
            print(f"| {r['oversub']} | {r['cus']} | {r['rate']} | {r['offered']} | {r['served']} | {r['hp_miss']} | {r['lp_miss']} | {r['lp_rejected']} | {r['hp_p99']} | {r['lp_p99']} |")
        return
    if a.queue_scaling:
        rows = queue_scaling(a.queue_scaling, a.dtype)
        print("| masks | queues | CUs per queue | inferences/s | per queue | GPU span per stage us | wall per stage us |\n|---|---|---|---|---|---|---|")
        for r in rows:
            print(f"| {r['masks']} | {r['queues']} | {r['cus_per_queue']} | {r['inferences_per_s']} | {r['per_queue']} | {r['gpu_span_us']} | {r['stage_wall_us']} |")
        return
    if a.layer_profile:
        r = layer_profile(a.layer_profile, a.dtype, a.ncu, plan_cus=a.plan_cus)
        if not a.table:
            print(json.dumps(r))
            return
        print(f"{r['net']} {r['dtype']} alone on {r['n_cu']} CUs: kernels {r['kernel_time_us']} us, job latency through the scheduler {r['job_latency_us']} us, "
              f"sum of layer rooflines {r['t_roof_us']} us\n")
        print("| # | layer | kernel | M | N | us | GFLOP | MB | TFLOP/s | GB/s | bound | t_roof us | frac |\n|---|---|---|---|---|---|---|---|---|---|---|---|---|")
        for x in r["layers"]:
            note = f" (launched with layer {x['joint_launch_with']})" if x["joint_launch_with"] is not None else ""
            print(f"| {x['layer']} | {x['name']}{note} | {x['kernel']} | {x['M']} | {x['N']} | {x['us']} | {x['gflop']} | {x['mbytes']} | {x['tflops']} | {x['gbs']} | "
                  f"{x['bound']} | {x['t_roof_us']} | {x['frac']} |")
        return
    if a.paper_set:
        # Table II shape: N_c equal partitions of ceil_even(OS * 256 / N_c) CUs (Sec. III-C2), OS given as a fraction
        num, den = (int(v) for v in (a.os.split("/") + ["1"])[:2])
        n_cu = min(256, D.daris_cu_per_partition(num, den, 256, a.nc))
        ts = wl.make_paper_taskset(a.paper_set, a.n_high, a.n_low, a.task_jps, [n_cu] * a.nc, n_jobs=a.jobs, n_stages=a.stages or 4,
                                   dtype=a.dtype)
    else:
        ts = wl.make_taskset(a.config, n_jobs=a.jobs, rate_scale=a.rate, oversub=a.oversub)
    if a.stages:
        for t in ts.tasks:
            t.n_stages = a.stages
    fl = 0
    for name in filter(None, a.flags.split(",")):
        fl |= {"no_last": D.NO_LAST, "no_prior": D.NO_PRIOR, "no_fixed": D.NO_FIXED, "hp_admission": D.HP_ADMISSION, "wave_prio": D.WAVE_PRIORITY, "shared_queue": D.SHARED_QUEUE}[name]
    g = GpuTaskSet(ts, flags=fl, streams_per_partition=a.streams)
    try:
        g.calibrate(loaded=a.loaded_afet)
        D.daris_commit()
        res = run_saturated(g, a.jobs * g.n_tasks, a.driver_profile) if a.saturated else run_periodic(g, a.jobs, a.migrate_every)
        res["response_ms"] = response_percentiles(D.trace_read_all(), [t.priority for t in ts.tasks])
        res["config"] = dict(name=ts.name, partitions=ts.partitions, streams=a.streams, tasks=g.n_tasks, rate=a.rate, oversub=a.oversub,
                             stages=[t.n_stages for t in ts.tasks], flags=a.flags)
        print(json.dumps(res))
    finally:
        g.close()


if __name__ == "__main__":
    main()
