"""The benchmark task sets (which networks, priorities, periods, partitions) and
seeded execution-time tables for virtual-time runs.

Everything here is workload description: lists of integers.  No scheduling rule
is evaluated in this module.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

from .nets import build_net, net_macs

LP, HP = 0, 1
SEED = 20250408
MS = 1_000_000


@dataclass
class TaskSpec:
    net: str
    dtype: str          # "fp32" | "bf16"
    priority: int       # HP | LP
    period_ns: int
    deadline_ns: int
    n_stages: int
    seed: int           # weight / input seed
    input_dist: str = "normal"


@dataclass
class TaskSet:
    name: str
    tasks: List[TaskSpec]
    partitions: List[int]           # CUs per partition
    n_jobs: int                     # jobs per task
    n_inputs: int = 4               # seeded inputs per task, cycled by job index
    streams_per_partition: int = 1
    notes: str = ""
    phases_ns: List[int] = field(default_factory=list)

    def releases(self):
        """All (release_ns, task, job) triples, ordered by (time, task, job)."""
        ph = self.phases_ns or [0] * len(self.tasks)
        r = [(ph[i] + m * t.period_ns, i, m) for i, t in enumerate(self.tasks) for m in range(self.n_jobs)]
        r.sort()
        return r


def make_taskset(config: int, *, seed: int = SEED, n_jobs: int | None = None, rate_scale: float = 1.0,
                 oversub: float = 2.0) -> TaskSet:
    """Task set of benchmark configuration `config` (1..5)."""
    def spec(net, dtype, prio, period_ms, k, idx, dist="normal"):
        p = int(round(period_ms * MS))
        return TaskSpec(net, dtype, prio, p, p, k, seed + 1000 * config + idx, dist)

    if config == 1:
        tasks = [spec("tiny", "fp32", HP, 10, 2, 0, "uniform"), spec("tiny", "fp32", LP, 10, 2, 1, "uniform")]
        return TaskSet("tiny", tasks, [128, 128], n_jobs or 20)
    if config == 2:
        tasks = [spec("resnet18", "fp32", HP, 20, 3, i) for i in range(2)] + \
                [spec("resnet18", "fp32", LP, 40, 3, 2 + i) for i in range(2)]
        return TaskSet("resnet18x4", tasks, [128, 128, 128], n_jobs or 500)
    if config == 3:
        tasks = [spec("resnet50", "bf16", HP, 25, 4, i) for i in range(2)] + \
                [spec("resnet50", "bf16", LP, 50, 4, 2 + i) for i in range(4)]
        return TaskSet("resnet50x6_bf16", tasks, [128, 128, 128, 128], n_jobs or 1000)
    if config == 4:
        g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 4, 77])))
        periods_us = [int(v) for v in g.integers(20000, 80001, 8)]
        nets = ["resnet18", "resnet18", "resnet50", "resnet50", "vgg16", "vgg16", "mobilenet_v2", "mobilenet_v2"]
        tasks = [spec(n, "fp32", HP if i < 2 else LP, periods_us[i] / 1000.0, 3, i) for i, n in enumerate(nets)]
        return TaskSet("mixed8", tasks, [96, 96, 128, 192], n_jobs or 500)
    if config == 5:
        tasks = [spec("resnet50", "bf16", HP, 40.0 / rate_scale, 4, i) for i in range(4)]
        for i in range(12):
            tasks.append(spec("mobilenet_v2" if i % 2 == 0 else "resnet18", "fp32", LP, 80.0 / rate_scale, 3, 4 + i))
        cu = {1.0: 64, 1.5: 96, 2.0: 128, 2.5: 160}[oversub]
        return TaskSet(f"stress16_r{rate_scale}_os{oversub}", tasks, [cu] * 4, n_jobs or 200,
                       notes="one forced migration per 100 completed jobs")
    raise ValueError(config)


def virtual_et_table(ts: TaskSet, seed: int = SEED, *, load_scale: float = 1.0, spike_prob: float = 0.03):
    """Synthetic stage execution times, integer ns: table[task][stage] -> int64 [n_partitions][n_jobs].

    base(task, n_cu) = 15 us per layer + MACs / (n_cu * 40 GMAC/s), split over the
    stages by seeded shares in [0.7, 1.3] (normalised); each job gets a seeded
    multiplicative jitter in [0.9, 1.25] and, with probability `spike_prob`, a
    further x1.8 spike.  `load_scale` multiplies everything.
    """
    table = []
    for i, t in enumerate(ts.tasks):
        layers, shp = build_net(t.net)
        macs = sum(net_macs(layers, shp))
        g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 9000 + i])))
        share = g.uniform(0.7, 1.3, t.n_stages)
        share = share / share.sum()
        per_stage = []
        for j in range(t.n_stages):
            arr = np.empty((len(ts.partitions), ts.n_jobs), dtype=np.int64)
            for k, ncu in enumerate(ts.partitions):
                base = (15_000.0 * len(layers) + macs / (ncu * 40.0)) * share[j] * load_scale
                jit = g.uniform(0.9, 1.25, ts.n_jobs)
                spike = np.where(g.uniform(0, 1, ts.n_jobs) < spike_prob, 1.8, 1.0)
                arr[k] = np.maximum(1, np.floor(base * jit * spike)).astype(np.int64)
            per_stage.append(arr)
        table.append(per_stage)
    return table


def make_paper_taskset(net: str, n_high: int, n_low: int, task_jps: float, partitions, *, n_jobs: int = 100, seed: int = SEED,
                       dtype: str = "fp32", n_stages: int = 4, weight_sets: int = 8) -> TaskSet:
    """Task set shaped like the paper's Table II: n_high HP + n_low LP tasks of one DNN type, each releasing `task_jps`
    jobs per second (implicit deadlines), on the given partition sizes.  Tasks cycle through `weight_sets` distinct seeds
    so that set-up time stays bounded for dozens of tasks."""
    period = int(round(1e9 / task_jps))
    tasks = []
    for i in range(n_high + n_low):
        tasks.append(TaskSpec(net, dtype, HP if i < n_high else LP, period, period, n_stages, seed + 50_000 + (i % weight_sets)))
    return TaskSet(f"paper_{net}_{n_high}h{n_low}l_{task_jps:g}jps", tasks, list(partitions), n_jobs, n_inputs=2)
