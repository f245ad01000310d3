"""The whole hot path on the GPU: periodic task sets released through the scheduler on CU-masked streams.
Virtual-time mode: trace bit-exact against the oracle's event model AND every job's logits against the oracle.
Real-time mode: the recorded trace is replayed through the oracle, which must reproduce every decision."""
import numpy as np
import pytest
import torch

import paper_2504_08795_amd as D
import workloads as wl
from gpu_helpers import TOL, rel_err
from paper_2504_08795_amd import harness
from lib_helpers import load_et
from oracle import des
from oracle import forward as F
from sched_helpers import check_trace_invariants

pytestmark = pytest.mark.gpu


class GpuTaskSet(harness.GpuTaskSet):
    """The harness's task-set registration plus the oracle-side checks."""

    def __init__(self, ts, flags=0, afet=None, streams=None):
        super().__init__(ts, flags=flags, afet=afet, seed=wl.tasksets.SEED, streams_per_partition=streams)
        self.want = []

    def oracle_logits(self):
        if not self.want:
            for layers, weights, xs, dtype in self.nets:
                self.want.append([F.forward(layers, weights, x, dtype) for x in xs])
        return self.want

    def check_logits(self, trace):
        """Every completed job's logits row against the oracle entry of the input it used."""
        want = self.oracle_logits()
        done = [(r[6], r[8]) for r in trace if r[2] == des.JOB_DONE]
        assert done
        worst = 0.0
        outs = [l.cpu().numpy() for l in self.logits]
        for task, job in done:
            dtype = self.ts.tasks[task].dtype
            e_max, e_l2 = rel_err(outs[task][job], want[task][job % self.ts.n_inputs])
            worst = max(worst, e_max)
            assert e_max <= TOL[dtype] and e_l2 <= TOL[dtype], (task, job, e_max, e_l2)
        # rows of rejected jobs were never written
        rejected = [(r[6], r[8]) for r in trace if r[2] == des.REJECT]
        for task, job in rejected:
            assert np.isnan(outs[task][job]).all()
        return worst, len(done)

def oracle_model(ts, afet, n_streams=None, flags=0):
    tasks = [des.TaskParam(t.period_ns, t.deadline_ns, t.priority, list(afet[i])) for i, t in enumerate(ts.tasks)]
    return des.SchedulerModel(n_streams or [1] * len(ts.partitions), tasks, flags=flags)


@pytest.mark.parametrize("config,n_jobs,load", [(1, 20, 300.0), (2, 12, 25.0)])
def test_virtual_time_trace_and_logits(config, n_jobs, load):
    ts = wl.make_taskset(config, n_jobs=n_jobs)
    et = wl.virtual_et_table(ts, load_scale=load)
    afet = [[int(np.mean(et[i][j][0][:8])) for j in range(t.n_stages)] for i, t in enumerate(ts.tasks)]
    g = GpuTaskSet(ts, flags=D.VIRTUAL_TIME, afet=afet)
    try:
        load_et(et, len(ts.partitions))
        D.daris_run_periodic(None, [n_jobs] * len(ts.tasks))
        got = D.trace_read_all()
        m = oracle_model(ts, afet)
        want = des.run_virtual(m, [("release", t, i) for t, i, _ in ts.releases()], et)
        for a, b in zip(got, want):
            assert a == b, f"first difference at seq {a[0]}: library {a}, oracle {b}"
        assert len(got) == len(want)
        worst, n = g.check_logits(got)
        print(f"config {config}: {n} jobs checked, worst logits error {worst:.3e}")
    finally:
        g.close()


def _replay_and_check(ts, afet, got, n_streams=None, flags=0):
    m = oracle_model(ts, afet, n_streams, flags)
    again = des.run_replay(m, got)
    for a, b in zip(got, again):
        assert a == b, f"first difference at seq {a[0]}: library {a}, oracle replay {b}"
    assert len(got) == len(again)
    check_trace_invariants(got, m.n_streams, [t.priority for t in ts.tasks], [t.n_stages for t in ts.tasks], flags=flags)
    return m


@pytest.mark.parametrize("config,n_jobs", [(1, 20), (2, 25), (3, 8), (4, 5)])
def test_real_time_periodic_run_replays_through_oracle(config, n_jobs):
    """Configs 3 (6x ResNet-50 bf16, 4 partitions) and 4 (mixed 8 tasks incl. VGG-16 and MobileNetV2) run with few
    jobs and two inputs per task so that the oracle's share stays within seconds."""
    ts = wl.make_taskset(config, n_jobs=n_jobs)
    if config >= 3:
        ts.n_inputs = 2
    g = GpuTaskSet(ts)
    try:
        for i in range(len(ts.tasks)):
            D.daris_calibrate_afet(i, i % len(ts.partitions), 3)
        afet = [[D.daris_get_mret(i, j) for j in range(t.n_stages)] for i, t in enumerate(ts.tasks)]
        D.daris_run_periodic(None, [n_jobs] * len(ts.tasks))
        got = D.trace_read_all()
        stats = [D.daris_get_stats(i) for i in range(len(ts.tasks))]
        m = _replay_and_check(ts, afet, got)
        worst, n = g.check_logits(got)
        for s, o in zip(stats, m.stats()):
            assert (s["accepted"], s["completed"], s["missed"]) == (o["accepted"], o["completed"], o["missed"])
        hp = [s for s, t in zip(stats, ts.tasks) if t.priority == wl.HP]
        assert all(s["missed"] == 0 and s["completed"] == n_jobs for s in hp), hp
        print(f"config {config}: {n} jobs, worst logits error {worst:.3e}, responses (ms) "
              + ", ".join(f"{s['resp_sum_ns'] / max(s['completed'], 1) / 1e6:.3f}" for s in stats))
    finally:
        g.close()


def test_closed_loop_with_forced_migrations():
    ts = wl.make_taskset(2, n_jobs=40)
    g = GpuTaskSet(ts)
    try:
        for i in range(len(ts.tasks)):
            D.daris_calibrate_afet(i, 0, 2)
        afet = [[D.daris_get_mret(i, j) for j in range(t.n_stages)] for i, t in enumerate(ts.tasks)]
        D.daris_commit()
        D.daris_migrate(3, (D.daris_get_partition(3) + 1) % 3)      # while idle: applies at once
        D.daris_run_closed_loop([40] * 4)
        D.daris_migrate(2, (D.daris_get_partition(2) + 1) % 3)
        D.daris_run_closed_loop([10] * 4)
        got = D.trace_read_all()
        m = _replay_and_check(ts, afet, got)
        assert sum(1 for r in got if r[2] == des.MIGRATE and (r[9] >> 8)) == 2
        # logits rows are reused modulo n_jobs in the second run: check the rows that hold a final value
        st = [D.daris_get_stats(i) for i in range(4)]
        assert all(s["completed"] + s["rejected_admission"] + s["rejected_overrun"] == 50 for s in st)
        outs = [l.cpu().numpy() for l in g.logits]
        want = g.oracle_logits()
        for task in range(4):
            for job in range(10, 40):
                if not np.isnan(outs[task][job]).any():
                    e_max, _ = rel_err(outs[task][job], want[task][job % ts.n_inputs])
                    assert e_max <= TOL["fp32"]
    finally:
        g.close()


def test_driver_profile_accounts_for_the_stages_it_saw():
    """The stage-boundary accounting covers every stage of the run and its parts are consistent with each other."""
    ts = wl.make_taskset(2, n_jobs=12)
    g = GpuTaskSet(ts)
    try:
        for i in range(len(ts.tasks)):
            D.daris_calibrate_afet(i, 0, 2)
        D.daris_commit()
        D.daris_driver_profile(True)
        D.daris_run_closed_loop([12] * 4)
        pr = D.daris_driver_profile(False)
        assert pr["stages"] == 4 * 12 * 3
        # the kernels of a stage run inside the interval in which the host enqueues and waits for them
        assert 0 < pr["gpu_ns"] <= pr["enqueue_ns"] + pr["wait_ns"]
        assert all(pr[k] >= 0 for k in pr)
        D.daris_run_closed_loop([2] * 4)
        assert D.daris_driver_profile(False)["stages"] == 0       # switched off: nothing gathered
        outs = [l.cpu().numpy() for l in g.logits]
        want = g.oracle_logits()
        for task in range(4):
            for job in range(2, 12):
                assert rel_err(outs[task][job], want[task][job % ts.n_inputs])[0] <= TOL["fp32"]
    finally:
        g.close()


def test_kernel_timing_covers_every_launch_of_the_sampled_jobs():
    """Sampling every job: each kernel id is counted once per launch of the network, the durations are the dispatch
    time stamps (positive, microseconds), and together they fit into the stages' GPU spans; logits stay right."""
    ts = wl.make_taskset(2, n_jobs=6)
    g = GpuTaskSet(ts)
    try:
        for i in range(len(ts.tasks)):
            D.daris_calibrate_afet(i, 0, 2)
        D.daris_commit()
        layers = g.nets[0][0]
        plans = [D.daris_get_launch_plan(0, l) for l in range(len(layers))]
        per_job = {}
        for pl in plans:
            if pl["pair_with"] >= 0 and not pl["pair_lead"]:
                continue                                      # launched together with the next layer
            name = D.daris_kernel_name(pl["kernel_id"])
            per_job[name] = per_job.get(name, 0) + 1
            splitk = max(pl["splitk"], plans[pl["pair_with"]]["splitk"]) if pl["pair_with"] >= 0 else pl["splitk"]
            if pl["dense_conv"] and splitk > 1:
                per_job["splitk_reduce"] = per_job.get("splitk_reduce", 0) + 1
        D.daris_driver_profile(True)
        D.daris_kernel_timing_start(1, 100000)
        D.daris_run_closed_loop([6] * 4)
        timing, fixed_ms = D.daris_kernel_timing_read()
        pr = D.daris_driver_profile(False)
        assert fixed_ms == 0.0
        assert {k: v[0] for k, v in timing.items()} == {k: n * 4 * 6 for k, n in per_job.items()}
        for name, (n, ms, fl) in timing.items():
            assert 0.5e-3 < ms / n < 1.0, (name, ms / n)       # between half a microsecond and a millisecond per launch
        assert sum(v[1] for v in timing.values()) * 1e6 <= pr["gpu_ns"] * 1.001
        D.daris_run_closed_loop([2] * 4)
        assert D.daris_kernel_timing_read()[0] == {}           # sampling was switched off by the read
        outs = [l.cpu().numpy() for l in g.logits]
        want = g.oracle_logits()
        for task in range(4):
            for job in range(2, 6):
                assert rel_err(outs[task][job], want[task][job % ts.n_inputs])[0] <= TOL["fp32"]
    finally:
        g.close()


def test_explicit_buffers_and_pool_buffers_give_the_same_logits():
    """A job released with explicit device pointers (argument blocks patched at launch time) and a job of the I/O pool
    (argument blocks prepared in device memory) run the same kernels on the same data: bit-identical logits."""
    ts = wl.make_taskset(1, n_jobs=4)
    g = GpuTaskSet(ts)
    try:
        for i in range(len(ts.tasks)):
            D.daris_calibrate_afet(i, i % 2, 2)
        D.daris_commit()
        D.daris_run_periodic(None, [4] * len(ts.tasks))
        pooled = [l.cpu().numpy().copy() for l in g.logits]
        for task in range(len(ts.tasks)):
            for job in range(4):
                y = torch.full((g.logits[task].shape[1],), float("nan"), dtype=torch.float32, device="cuda")
                torch.cuda.synchronize()
                D.daris_release_job(task, g.inputs[task][job % ts.n_inputs], y, -1)
                D.daris_run_until_idle()
                assert np.array_equal(y.cpu().numpy(), pooled[task][job]), (task, job)
    finally:
        g.close()


@pytest.mark.parametrize("shape", ["conversions", "single_fc", "two_convs"])
def test_pool_jobs_of_networks_with_unusual_first_and_last_launches(shape):
    """The launches that read a job's input and write its logits differ by network: a layout conversion before an
    8-channel first convolution and another one after a last layer that is not an FC; an FC that does both at once
    behind the input conversion; a fused 3-channel first convolution.  Jobs of an I/O pool (argument blocks prepared per
    buffer) must give what a direct forward pass with explicit pointers gives, bit for bit, and agree with the oracle."""
    N = wl.nets
    rng = np.random.default_rng(5)
    if shape == "conversions":
        layers, shp = [N.Layer(op=N.OP_CONV, c_in=8, c_out=24, k=3, stride=1, pad=1, act=1, in_from=-1),
                       N.Layer(op=N.OP_CONV, c_in=24, c_out=12, k=1, stride=1, pad=0, act=0, in_from=0)], (8, 9, 11)
    elif shape == "single_fc":
        layers, shp = [N.Layer(op=N.OP_FC, c_in=5 * 4 * 3, c_out=7, in_from=-1)], (5, 4, 3)
    else:
        layers, shp = [N.Layer(op=N.OP_CONV, c_in=3, c_out=16, k=3, stride=2, pad=1, act=1, in_from=-1),
                       N.Layer(op=N.OP_CONV, c_in=16, c_out=8, k=3, stride=1, pad=1, act=2, in_from=0)], (3, 17, 15)
    weights = []
    for L in layers:
        cg = L.c_in // L.groups
        w = rng.normal(0, 0.2, (L.c_out, cg, L.k, L.k) if L.op == N.OP_CONV else (L.c_out, L.c_in)).astype(np.float32)
        weights.append((w, rng.normal(0, 0.3, L.c_out).astype(np.float32)))
    n_in, n_slots, n_jobs = 3, 5, 7
    xs = rng.normal(0, 1, (n_in,) + shp).astype(np.float32)
    want = [F.forward(layers, weights, x, "fp32").ravel() for x in xs]
    n_out = want[0].size
    D.daris_init(0, 0, 0)
    try:
        p = D.daris_create_partition(64)
        dnn, keep = D.make_dnn(layers, weights, shp, "fp32")
        t = D.daris_register_task(dnn, 2_000_000, 2_000_000, D.HP)
        xd = torch.from_numpy(xs).cuda()
        yd = torch.full((n_slots, n_out), float("nan"), dtype=torch.float32, device="cuda")
        D.daris_task_set_io(t, xd, n_in, yd, n_slots)
        D.daris_calibrate_afet(t, p, 2)
        D.daris_run_periodic(None, [n_jobs])
        assert D.daris_get_stats(t)["completed"] == n_jobs
        got = yd.cpu().numpy()
        for slot in range(n_slots):
            job = max(j for j in range(n_jobs) if j % n_slots == slot)      # the last job that wrote this row
            direct = torch.full((n_out,), float("nan"), dtype=torch.float32, device="cuda")
            D.daris_forward(t, xd[job % n_in], direct, p)
            assert np.array_equal(got[slot], direct.cpu().numpy()), (shape, slot)
            e_max, e_l2 = rel_err(got[slot], want[job % n_in])
            assert e_max <= 2e-5 and e_l2 <= 2e-5, (shape, slot, e_max, e_l2)
    finally:
        D.daris_shutdown()


def _probe(p, n_groups=8192, spin=3000):
    """Distinct compute units (XCC id, and bits 8..15 of the hardware id register: CU, shader array, shader engine) that
    the workgroups of one probe launch on partition p ran on."""
    ids = D.daris_probe_cus(p, n_groups, spin)
    return {(int(x) & 0xF, (int(h) >> 8) & 0xFF) for x, h in ids}


def test_cu_masks_are_honoured():
    """A partition's workgroups run on exactly as many distinct CUs as the partition owns, an eighth of them on each of
    the eight XCDs (mask bit i lands on XCD i mod 8, so a cyclic run of n bits is spread evenly); partitions whose CU ranges
    do not overlap use disjoint CUs, and together the whole chip."""
    D.daris_init(0, 0, 0)
    try:
        sizes = (32, 128, 256)
        parts = [D.daris_create_partition(n) for n in sizes]
        for p, n in zip(parts, sizes):
            cus = _probe(p)
            per_xcc = [sum(1 for x, _ in cus if x == k) for k in range(8)]
            print(f"partition of {n} CUs: {len(cus)} distinct CUs, per XCC {per_xcc}")
            assert len(cus) == n, (n, len(cus), per_xcc)
            assert per_xcc == [n // 8] * 8, per_xcc
    finally:
        D.daris_shutdown()
    D.daris_init(0, 0, 0)
    try:
        sizes = (64, 64, 96, 32)                      # 256 in all: cyclic ranges [0,64) [64,128) [128,224) [224,256)
        parts = [D.daris_create_partition(n) for n in sizes + (64,)]   # the fifth wraps around onto the first one's CUs
        sets = [_probe(p) for p in parts[:4]]
        for n, c in zip(sizes, sets):
            assert len(c) == n, (n, len(c))
        for i in range(len(sets)):
            for j in range(i + 1, len(sets)):
                assert not (sets[i] & sets[j]), (i, j, len(sets[i] & sets[j]))
        assert len(set().union(*sets)) == 256
        assert _probe(parts[4]) == sets[0]              # oversubscription (Sec. III-C2): the same CUs, shared
    finally:
        D.daris_shutdown()


def test_wait_limit_turns_a_late_gpu_into_an_error_and_the_library_recovers_after_shutdown():
    """Host-side failure handling, forced from the host: with a wait limit of 1 ns the host gives up on a ResNet-18
    forward pass (about 0.2 ms of kernels, which all complete normally on the GPU) at its first look at the clock.  The
    call returns DARIS_EHIP instead of hanging, later calls are refused, the accessors still answer, daris_shutdown lets
    the queue run dry before freeing the buffers, and a fresh session computes the right logits."""
    layers, shp = wl.build_net("resnet18")
    weights = wl.make_weights(layers, 77)
    x = wl.make_inputs(shp, 77, 1, "normal")[0]
    xd = torch.from_numpy(x).cuda()
    try:
        D.daris_init(0, 0, 0)
        p = D.daris_create_partition(128)
        dnn, keep = D.make_dnn(layers, weights, shp, "fp32")
        t = D.daris_register_task(dnn, 10_000_000, 10_000_000, D.LP)
        y = torch.zeros(1000, device="cuda")
        torch.cuda.synchronize()
        D.daris_forward(t, xd, y, p)                  # creates the streams, warms up
        good = y.cpu().numpy().copy()
        D.daris_set_timeout(1)
        with pytest.raises(D.DarisError) as e:
            D.daris_forward(t, xd, y, p)
        assert e.value.code == D.EHIP and "wait limit" in str(e.value)
        with pytest.raises(D.DarisError) as e:
            D.daris_forward(t, xd, y, p)              # refused: the state of the GPU work is unknown
        assert e.value.code == D.EHIP
        with pytest.raises(D.DarisError):
            D.daris_run_closed_loop([1], 0)
        assert D.daris_get_stats(t)["released"] == 0  # read-only accessors still answer
    finally:
        D.daris_set_timeout(20_000_000_000)
        D.daris_shutdown()
    D.daris_init(0, 0, 0)
    try:
        p = D.daris_create_partition(128)
        dnn, keep = D.make_dnn(layers, weights, shp, "fp32")
        t = D.daris_register_task(dnn, 10_000_000, 10_000_000, D.LP)
        y = torch.full((1000,), float("nan"), device="cuda")
        torch.cuda.synchronize()
        D.daris_forward(t, xd, y, p)
        np.testing.assert_array_equal(y.cpu().numpy(), good)
        assert rel_err(good, F.forward(layers, weights, x, "fp32"))[0] <= TOL["fp32"]
    finally:
        D.daris_shutdown()


def test_stress_set_with_forced_migrations_between_chunks():
    """Config 5 shape at one sweep point (rate 1.0, oversubscription 2.0): 4 HP ResNet-50 bf16 + 12 LP fp32 tasks on 4
    partitions, periodic releases in two chunks with forced migrations between them; trace replays through the oracle and
    every completed job's logits match."""
    ts = wl.make_taskset(5, n_jobs=4, rate_scale=1.0, oversub=2.0)
    ts.n_inputs = 1
    g = GpuTaskSet(ts)
    try:
        for i in range(len(ts.tasks)):
            D.daris_calibrate_afet(i, i % 4, 2)
        afet = [[D.daris_get_mret(i, j) for j in range(t.n_stages)] for i, t in enumerate(ts.tasks)]
        res = harness.run_periodic(g, 4, migrate_every=32, seed=3)
        got = D.trace_read_all()
        m = _replay_and_check(ts, afet, got)
        assert sum(1 for r in got if r[2] == des.CMD_MIGRATE) >= 1
        worst, n = g.check_logits(got)
        assert res["hp"]["missed"] == 0 and res["hp"]["completed"] == 16
        print(f"stress point: {n} jobs, worst logits error {worst:.3e}, {res['inferences_per_s']} inf/s, LP miss {res['lp']['miss_pct']:.1f} %")
    finally:
        g.close()


@pytest.mark.parametrize("streams,lib_flags,des_flags", [(2, 0, 0), (1, D.NO_FIXED, des.F_NO_FIXED), (2, D.NO_LAST | D.NO_PRIOR, des.F_NO_LAST | des.F_NO_PRIOR),
                                                         (1, D.WAVE_PRIORITY, 0), (2, D.SHARED_QUEUE, 0), (3, D.SHARED_QUEUE, 0)])
def test_saturated_run_with_streams_and_ablation_flags(streams, lib_flags, des_flags):
    """Two streams per partition (the paper's MPS+STR shape), the ablation switches, the wave-priority option and the
    streams of a partition sharing one hardware queue (both change kernel timing only), saturated so that stages really
    compete: the recorded trace replays through the oracle with the same switches, logits match."""
    ts = wl.make_taskset(2, n_jobs=30)
    g = GpuTaskSet(ts, flags=lib_flags, streams=streams)
    try:
        afet = g.calibrate(2)
        D.daris_commit()
        D.daris_run_closed_loop([30] * 4, 0)
        got = D.trace_read_all()
        _replay_and_check(ts, afet, got, [streams] * 3, des_flags)
        worst, n = g.check_logits(got)
        assert n == 120
        if streams >= 2:
            assert any(r[2] == des.DISPATCH and r[7] == 1 for r in got), "second stream never used"
    finally:
        g.close()


@pytest.mark.parametrize("config", [4, 3])
def test_saturated_closed_loop_in_the_benchmark_configuration(config):
    """One step of `bench.py`'s timed region in its own launch configuration -- every task of the configuration releasing
    back to back on its partition, 32 jobs per task released over all tasks from a common budget -- with the logits of
    EVERY completed job checked against the oracle and the recorded trace replayed through it."""
    per_step = 32
    ts = wl.make_taskset(config, n_jobs=per_step * 8)          # a task may take far more than its share of the budget
    ts.n_inputs = 2
    nt = len(ts.tasks)
    g = GpuTaskSet(ts)
    try:
        afet = g.calibrate(3)
        D.daris_commit()
        D.daris_run_closed_loop([per_step * nt] * nt, per_step * nt)
        got = D.trace_read_all()
        _replay_and_check(ts, afet, got)
        worst, n = g.check_logits(got)
        stats = g.stats()
        assert n == sum(s["completed"] for s in stats) and n + sum(s["rejected_admission"] + s["rejected_overrun"] for s in stats) == per_step * nt
        assert all(s["completed"] > 0 for s in stats)
        print(f"config {config} saturated: {n} jobs, per task {[s['completed'] for s in stats]}, worst logits error {worst:.3e}")
    finally:
        g.close()


def _full_size_run(config, hp_jobs):
    """A configuration at the job count it is specified with, at its nominal periods: the trace replays through the
    oracle, no HP job misses its deadline, fewer than 2 % of the LP jobs do, none is rejected, and the logits of every
    20th job of every task match the oracle."""
    ts = wl.make_taskset(config)
    ts.n_inputs = 2                                   # the oracle computes one forward pass per (task, input)
    g = GpuTaskSet(ts)
    try:
        afet = g.calibrate(3)
        res = harness.run_periodic(g, ts.n_jobs)
        got = D.trace_read_all()
        _replay_and_check(ts, afet, got)
        assert res["hp"]["completed"] == hp_jobs and res["hp"]["missed"] == 0, res["hp"]
        assert res["lp"]["miss_pct"] < 2.0 and res["lp"]["rejected_admission"] == 0 and res["lp"]["rejected_overrun"] == 0, res["lp"]
        assert res["hp"]["completed"] + res["lp"]["completed"] == ts.n_jobs * len(ts.tasks)
        want = g.oracle_logits()
        outs = [l.cpu().numpy() for l in g.logits]
        worst = 0.0
        for task, t in enumerate(ts.tasks):
            for job in range(0, ts.n_jobs, 20):
                e_max, e_l2 = rel_err(outs[task][job], want[task][job % ts.n_inputs])
                worst = max(worst, e_max)
                assert e_max <= TOL[t.dtype] and e_l2 <= TOL[t.dtype], (task, job, e_max, e_l2)
        print(f"config {config} full size: {res['inferences_per_s']} inf/s over {res['wall_s']} s, HP resp {res['hp']['mean_response_ms']} ms (max {res['hp']['max_response_ms']}), "
              f"LP resp {res['lp']['mean_response_ms']} ms (max {res['lp']['max_response_ms']}), LP miss {res['lp']['miss_pct']:.2f} %, worst logits error {worst:.2e}")
    finally:
        g.close()


def test_config3_full_size_periodic_run():
    """6x ResNet-50 bf16 on 4 x 128 CUs, 1000 jobs per task at 25 / 50 ms (50 s of wall time)."""
    _full_size_run(3, hp_jobs=2000)


def test_config4_full_size_periodic_run():
    """The mixed 8-task set on 96/96/128/192 CUs, 500 jobs per task at 20-80 ms periods (about 40 s of wall time)."""
    _full_size_run(4, hp_jobs=1000)


def _solo_job_ns(net, dtype, n_cu):
    """Execution time of one DNN alone on a partition, for sizing periods relative to it."""
    layers, shp = wl.build_net(net)
    D.daris_init(0, 0, 0)
    try:
        p = D.daris_create_partition(n_cu)
        dnn, keep = D.make_dnn(layers, wl.make_weights(layers, 1), shp, dtype)
        t = D.daris_register_task(dnn, 10_000_000, 10_000_000, D.LP)
        D.daris_calibrate_afet(t, p, 3)
        return D.daris_get_mret(t, 0)
    finally:
        D.daris_shutdown()


def test_paper_shaped_set_with_loaded_afet_replays_through_oracle():
    """The shape of the paper's main experiment (Table II: HP : LP = 1 : 2, every task at the same rate, about 150 % of
    what the GPU sustains, equal partitions of ceil_even(OS * 256 / N_c) CUs) with the AFET of every stage measured the
    way Sec. IV-A1 describes it: while the other streams run other tasks.  The trace replays through the oracle from those
    AFETs, HP jobs are never rejected or migrated, LP jobs are shed by the admission test, logits match."""
    solo = _solo_job_ns("resnet18", "fp32", 128)
    n_high, n_low, n_c = 6, 12, 3                                  # per task u is about 0.25: two HP tasks reserve half a context
    jps = 1.5 * n_c * (1e9 / solo) / (n_high + n_low)            # 150 % of three partitions serving jobs back to back
    n_cu = D.daris_cu_per_partition(3, 2, 256, n_c)
    assert n_cu == 128
    ts = wl.make_paper_taskset("resnet18", n_high, n_low, jps, [n_cu] * n_c, n_jobs=30, n_stages=3)
    g = GpuTaskSet(ts)
    try:
        plain = g.calibrate(2)
        loaded = g.calibrate(3, loaded=True)
        assert all(b >= 1 for a in loaded for b in a)
        assert sum(sum(a) for a in loaded) > 0.9 * sum(sum(a) for a in plain)      # co-runners do not make a stage faster
        res = harness.run_periodic(g, ts.n_jobs)
        got = D.trace_read_all()
        _replay_and_check(ts, loaded, got)
        assert res["hp"]["rejected_admission"] == 0 and res["hp"]["completed"] == n_high * ts.n_jobs
        assert not any(r[2] == des.MIGRATE and ts.tasks[r[6]].priority == wl.HP for r in got)
        assert res["lp"]["rejected_admission"] + res["lp"]["rejected_overrun"] > 0, "the set was meant to overload the GPU"
        assert res["lp"]["completed"] > 0, "the admission test was meant to let part of the LP load through"
        worst, n = g.check_logits(got)
        print(f"paper-shaped set at {jps:.0f} jobs/s per task: {res['inferences_per_s']} inf/s, HP miss {res['hp']['miss_pct']:.1f} %, LP miss {res['lp']['miss_pct']:.1f} %, "
              f"LP rejected {res['lp']['rejected_admission']}+{res['lp']['rejected_overrun']}, {n} jobs checked, worst logits error {worst:.2e}; "
              f"AFET solo {[sum(a) for a in plain][:3]} loaded {[sum(a) for a in loaded][:3]} ns")
    finally:
        g.close()


def test_hp_admission_under_hp_heavy_overload():
    """Overload + HP admission (Sec. VI-I) on the GPU: two partitions, each home to one HP task whose utilisation is about
    0.6 and to LP tasks of about 0.3 each.  With the admission test applied to HP jobs too, an HP release that finds its
    context's booked LP work above what is left is rejected (never migrated, never queued); others are admitted.  The
    recorded trace replays through the oracle with the same switch, and every completed job's logits match."""
    solo = _solo_job_ns("resnet18", "fp32", 128)
    specs = [(wl.HP, 0.6), (wl.HP, 0.6), (wl.LP, 0.3), (wl.LP, 0.3), (wl.LP, 0.3), (wl.LP, 0.3)]
    tasks = [wl.TaskSpec("resnet18", "fp32", prio, int(solo / u), int(solo / u), 3, wl.tasksets.SEED + 70_000 + (i % 2)) for i, (prio, u) in enumerate(specs)]
    ts = wl.TaskSet("hp_heavy_overload", tasks, [128, 128], 60, n_inputs=2)
    g = GpuTaskSet(ts, flags=D.HP_ADMISSION)
    try:
        afet = g.calibrate(3)
        res = harness.run_periodic(g, ts.n_jobs)
        got = D.trace_read_all()
        _replay_and_check(ts, afet, got, flags=des.F_HP_ADMISSION)
        hp_rej = [r for r in got if r[2] == des.REJECT and ts.tasks[r[6]].priority == wl.HP]
        assert hp_rej, "no HP job was rejected: the load was meant to exceed the HP tasks' contexts"
        assert res["hp"]["completed"] > 0 and res["hp"]["completed"] + len(hp_rej) == 2 * ts.n_jobs
        assert not any(r[2] in (des.QUEUED, des.MIGRATE) and ts.tasks[r[6]].priority == wl.HP for r in got)
        worst, n = g.check_logits(got)
        print(f"HP admission under overload: HP completed {res['hp']['completed']}, HP rejected {len(hp_rej)} "
              f"({sum(1 for r in hp_rej if r[9] == des.REJECT_ADMISSION)} by the test), HP miss {res['hp']['miss_pct']:.1f} %, "
              f"LP completed {res['lp']['completed']}, {n} jobs checked, worst logits error {worst:.2e}")
    finally:
        g.close()


def test_config2_full_size_periodic_run():
    """The benchmark configuration at its full size (500 jobs per task at 20 / 40 ms periods, about 20 s of wall time):
    trace replays through the oracle, no HP miss, LP misses under 2 %, and every 20th job's logits are checked."""
    ts = wl.make_taskset(2)
    assert ts.n_jobs == 500
    g = GpuTaskSet(ts)
    try:
        afet = g.calibrate(3)
        res = harness.run_periodic(g, ts.n_jobs)
        got = D.trace_read_all()
        _replay_and_check(ts, afet, got)
        assert res["hp"]["completed"] == 1000 and res["hp"]["missed"] == 0
        assert res["lp"]["miss_pct"] < 2.0 and res["lp"]["rejected_admission"] == 0
        want = g.oracle_logits()
        outs = [l.cpu().numpy() for l in g.logits]
        for task in range(4):
            for job in range(0, 500, 20):
                e_max, e_l2 = rel_err(outs[task][job], want[task][job % ts.n_inputs])
                assert e_max <= TOL["fp32"] and e_l2 <= TOL["fp32"], (task, job, e_max)
        print(f"config 2 full size: {res['inferences_per_s']} inf/s, HP resp {res['hp']['mean_response_ms']} ms, LP resp {res['lp']['mean_response_ms']} ms")
    finally:
        g.close()
