"""Pins of the scheduler oracle: closed forms of eq. 1-8 and the partition formula, hand-worked golden
traces, reductions to textbook schedulers, and invariants on large seeded runs."""
import random

import numpy as np
import pytest

import workloads as wl
from oracle import des
from sched_helpers import (check_trace_invariants, load_golden, model_from_golden, np_edf_single,
                           np_fixed_priority_single)


# ---- closed forms ------------------------------------------------------------------------------------
def test_mret_window_micro_case():
    ws, afet = 5, 77
    s = []
    assert des.mret_of(s, ws, afet) == 77              # t = 0: AFET
    for v, want in [(3, 3), (9, 9), (4, 9), (4, 9), (4, 9), (4, 9), (4, 4)]:
        s.append(v)
        assert des.mret_of(s, ws, afet) == want         # 9 leaves the window after five newer samples


def test_virtual_deadlines_sum_to_deadline():
    rnd = random.Random(7)
    for _ in range(10000):
        n = rnd.randint(1, 6)
        m = [rnd.randint(1, 10**7) for _ in range(n)]
        d = rnd.randint(1, 10**9)
        r = rnd.randint(0, 10**12)
        vd = des.virtual_deadlines(r, d, m)
        assert vd[-1] == r + d and all(a <= b for a, b in zip(vd, vd[1:])) and vd[0] >= r
        # each share is within one unit of the real-valued eq. (8)
        prev = r
        for j in range(n):
            share = vd[j] - prev
            assert abs(share - d * m[j] / sum(m)) < 1.0 + 1e-6
            prev = vd[j]
    assert des.virtual_deadlines(0, 100, [10, 30]) == [25, 100]


def test_ceil_even_and_partition_size():
    assert des.partition_cus(3, 2, 256, 3) == 128       # OS 1.5, N_c 3
    assert des.partition_cus(2, 1, 256, 4) == 128
    assert des.ceil_even(68, 3) == 24                   # 22.67 -> 24
    assert des.ceil_even(128, 1) == 128 and des.ceil_even(127, 1) == 128 and des.ceil_even(1, 1) == 2
    assert [des.partition_cus(n, 2, 256, 4) for n in (2, 3, 4, 5)] == [64, 96, 128, 160]
    assert des.partition_cus(6, 1, 68, 6) == 68         # OS = N_c: every context sees all SMs (2080 Ti has 68)


def test_utilisation_fixed_point_and_strict_admission():
    assert des.utilisation(50, 100) == 1 << 31
    assert des.utilisation(1, 3) == (1 << 32) // 3
    # equality must reject: HP u = 0.5, LP u = 0.5 in a one-stream context
    tasks = [des.TaskParam(100, 100, des.HP, [50]), des.TaskParam(100, 100, des.LP, [50])]
    m = des.SchedulerModel([1], tasks)
    m.commit()
    assert not m.admission_ok(0, m.u_task(1))
    tasks[1].afet[0] = 49
    m2 = des.SchedulerModel([1], tasks)
    m2.commit()
    assert m2.admission_ok(0, m2.u_task(1))
    # two streams double the capacity (U^r = N_s - U^h)
    m3 = des.SchedulerModel([2], [des.TaskParam(100, 100, des.HP, [50]), des.TaskParam(100, 100, des.LP, [140])])
    m3.commit()
    assert m3.admission_ok(0, m3.u_task(1))


def test_algorithm1_balances_hp_then_lp():
    # utilisations .5 .3 (HP) then .4 .4 .1 (LP) on two contexts:
    # HP: .5->c0, .3->c1 ; LP: .4->c1 (.3<.5) => [.5,.7]; .4->c0 => [.9,.7]; .1->c1
    tasks = [des.TaskParam(100, 100, des.LP, [40]), des.TaskParam(100, 100, des.HP, [50]), des.TaskParam(100, 100, des.LP, [40]),
             des.TaskParam(100, 100, des.HP, [30]), des.TaskParam(100, 100, des.LP, [10])]
    m = des.SchedulerModel([1, 1], tasks)
    m.commit()
    assert [t.ctx for t in m.tasks] == [1, 0, 0, 1, 1]


def test_level_order():
    lv = des.stage_level
    assert lv(des.HP, False, False) > lv(des.LP, True, True)          # HP always first
    assert lv(des.HP, True, False) > lv(des.HP, False, True)          # last stage above missed-predecessor
    assert sorted({lv(p, a, b) for p in (0, 1) for a in (0, 1) for b in (0, 1)}) == list(range(8))
    assert lv(des.HP, True, True, des.F_NO_FIXED) == 0
    assert lv(des.LP, True, True, des.F_NO_LAST) == 1 and lv(des.LP, True, True, des.F_NO_PRIOR) == 2


# ---- hand-worked traces --------------------------------------------------------------------------------
VIRTUAL_GOLDENS = ["sched_single_task.json", "sched_hp_preempts_lp.json", "sched_admission_migration.json",
                   "sched_migration_target_choice.json", "sched_forced_migration_at_boundary.json", "sched_hp_admission.json"]


@pytest.mark.parametrize("name", VIRTUAL_GOLDENS)
def test_golden_traces(name):
    g, cmds, et, want = load_golden(name)
    m = model_from_golden(g)
    got = des.run_virtual(m, cmds, et)
    for a, b in zip(got, want):
        assert a == b, f"first difference at seq {a[0]}: got {a}, want {b}"
    assert len(got) == len(want)
    check_trace_invariants(got, g["partitions"], [t["prio"] for t in g["tasks"]], [len(t["afet"]) for t in g["tasks"]], flags=m.flags)


def test_golden_traces_make_the_choices_they_were_written_for():
    """What each of the later hand-worked traces is there to pin, read off the trace itself."""
    _g, _c, _e, tr = load_golden("sched_migration_target_choice.json")
    mig = [(r[1], r[5], r[9]) for r in tr if r[2] == des.MIGRATE and r[6] == 5]
    assert mig == [(35, 2, 0), (100, 0, 258), (125, 1, 0)]      # higher index by predicted finish; forced; tie -> lowest index
    _g, _c, _e, tr = load_golden("sched_forced_migration_at_boundary.json")
    assert [(r[1], r[2]) for r in tr if r[6] == 0 and r[2] in (des.CMD_MIGRATE, des.MIGRATE)] == [(10, des.CMD_MIGRATE), (30, des.MIGRATE)]
    _g, _c, _e, tr = load_golden("sched_hp_admission.json")
    assert [(r[1], r[9]) for r in tr if r[2] == des.REJECT and r[6] == 0] == [(100, des.REJECT_ADMISSION), (240, des.REJECT_OVERRUN)]
    assert not any(r[2] in (des.MIGRATE, des.QUEUED) for r in tr)


def test_replay_uses_the_recorded_dispatch_clock():
    """A hand-written recording whose DISPATCH clock lags the events: execution times, the next job's virtual deadlines
    and a stage's miss flag all depend on it (see the file's `why`)."""
    g, _cmds, _et, rec = load_golden("sched_replay_dispatch_clock.json")
    assert any(r[2] == des.DISPATCH and r[1] != rec[i - 1][1] for i, r in enumerate(rec))
    m = model_from_golden(g)
    got = des.run_replay(m, rec)
    for a, b in zip(got, rec):
        assert a == b, f"first difference at seq {a[0]}: got {a}, want {b}"
    assert len(got) == len(rec)
    assert m.tasks[0].rings == [[30, 73], [10, 15]]             # et = completion - dispatch clock


# ---- reductions to textbook schedulers -------------------------------------------------------------------
def _single_stage_run(jobs_by_task, prios, flags=0):
    """jobs_by_task[i] = list of (release, exec); one partition, one stream, one stage, huge periods (no admission
    effect), deadline = per-task relative deadline given as third tuple element."""
    tasks, cmds, et = [], [], []
    for i, (jobs, d) in enumerate(jobs_by_task):
        tasks.append(des.TaskParam(10**9, d, prios[i], [1]))
        et.append([[[c for _r, c in jobs]]])
        cmds += [("release", r, i) for r, _c in jobs]
    cmds.sort(key=lambda c: (c[1], c[2]))
    m = des.SchedulerModel([1], tasks, flags=flags)
    tr = des.run_virtual(m, cmds, et)
    starts = {(r[6], r[8]): r[1] for r in tr if r[2] == des.DISPATCH}
    ends = {(r[6], r[8]): r[1] for r in tr if r[2] == des.JOB_DONE}
    return tr, starts, ends


def test_reduces_to_nonpreemptive_edf():
    rnd = random.Random(3)
    for trial in range(50):
        spec, ref_jobs = [], []
        for i in range(4):
            d = rnd.randint(20, 200)
            rel, jobs = 0, []
            for m in range(5):
                c = rnd.randint(1, 15)
                jobs.append((rel, c))
                ref_jobs.append((rel, c, rel + d, (i, m)))
                rel += rnd.randint(60, 120)       # spaced so a task never overruns its own previous job
            spec.append((jobs, d))
        tr, starts, ends = _single_stage_run(spec, [des.LP] * 4)
        ref = np_edf_single(ref_jobs)
        assert {i: (s, f) for s, f, i in ref} == {k: (starts[k], ends[k]) for k in starts}


def test_reduces_to_nonpreemptive_fixed_priority():
    rnd = random.Random(4)
    for trial in range(50):
        spec, ref_jobs = [], []
        # one HP and one LP task with the SAME relative deadline and release pattern offsets: EDF inside a level
        # never decides between them, the level does
        for i, prio in enumerate((des.LP, des.HP)):
            rel, jobs = rnd.randint(0, 5), []
            for m in range(6):
                c = rnd.randint(5, 30)
                jobs.append((rel, c))
                ref_jobs.append((rel, c, prio, (i, m)))
                rel += rnd.randint(70, 90)
            spec.append((jobs, 10**6))
        tr, starts, ends = _single_stage_run(spec, [des.LP, des.HP])
        ref = np_fixed_priority_single(ref_jobs)
        assert {i: (s, f) for s, f, i in ref} == {k: (starts[k], ends[k]) for k in starts}


def test_one_task_alone_response_is_sum_of_stage_times():
    et = [[[[7, 9]], [[11, 200]], [[13, 5]]]]
    m = des.SchedulerModel([1], [des.TaskParam(100, 100, des.LP, [10, 10, 10])])
    des.run_virtual(m, [("release", 0, 0), ("release", 1000, 0)], et)
    st = m.stats()[0]
    assert st["responses"] == [31, 214] and st["missed"] == 1 and st["accepted"] == 2


# ---- brute force on a tiny set: every dispatch decision re-derived by exhaustive comparison ----------------
def test_dispatch_choice_bruteforce_small():
    rnd = random.Random(11)
    for trial in range(30):
        ntask = 3
        tasks = [des.TaskParam(rnd.choice([50, 80, 120]), 0, rnd.choice([0, 1]), [rnd.randint(3, 9) for _ in range(rnd.randint(1, 3))])
                 for _ in range(ntask)]
        for t in tasks:
            t.deadline = t.period
        et = [[[[rnd.randint(2, 14) for _ in range(3)]] for _ in t.afet] for t in tasks]
        cmds = sorted([("release", m * t.period, i) for i, t in enumerate(tasks) for m in range(3)], key=lambda c: (c[1], c[2]))
        m = des.SchedulerModel([1], tasks)
        tr = des.run_virtual(m, cmds, et)
        check_trace_invariants(tr, [1], [t.prio for t in tasks], [len(t.afet) for t in tasks])
        # re-derive: at each DISPATCH the chosen (level, vd, task, job) must be the lexicographic best of the stages
        # ready at that instant, reconstructed from the trace alone
        ready, rel = {}, {}
        for (_s, t, typ, lvl, stage, part, task, stream, job, aux) in tr:
            if typ == des.RELEASE:
                rel[(task, job)] = t
            elif typ == des.ACCEPT:
                ready[(task, job)] = (0, False)
            elif typ == des.STAGE_DONE and stage + 1 < len(tasks[task].afet):
                ready[(task, job)] = (stage + 1, bool(aux))
            elif typ == des.DISPATCH:
                mine_lvl = lvl
                for (tk, jb), (stg, pm) in ready.items():
                    if (tk, jb) == (task, job):
                        continue
                    other = des.stage_level(tasks[tk].prio, stg == len(tasks[tk].afet) - 1, pm)
                    assert other <= mine_lvl
                del ready[(task, job)]


# ---- large seeded runs: invariants + qualitative direction ---------------------------------------------------
@pytest.mark.parametrize("config,load", [(2, 25.0), (3, 18.0), (4, 22.0)])
def test_invariants_on_benchmark_shaped_sets(config, load):
    ts = wl.make_taskset(config, n_jobs=60)
    et = wl.virtual_et_table(ts, load_scale=load)
    tasks = [des.TaskParam(t.period_ns, t.deadline_ns, t.priority, [int(np.mean(et[i][j][0][:8])) for j in range(t.n_stages)])
             for i, t in enumerate(ts.tasks)]
    m = des.SchedulerModel([1] * len(ts.partitions), tasks)
    cmds = [("release", t, i) for t, i, _ in ts.releases()]
    # a forced migration now and then
    extra = [("migrate", cmds[n][1], (n // 37) % len(tasks), (n // 13) % len(ts.partitions)) for n in range(40, len(cmds), 97)]
    allc = sorted(cmds + extra, key=lambda c: c[1])
    tr = des.run_virtual(m, allc, et)
    check_trace_invariants(tr, m.n_streams, [t.prio for t in tasks], [len(t.afet) for t in tasks])
    st = m.stats()
    hp = [s for s, t in zip(st, tasks) if t.prio == des.HP]
    lp = [s for s, t in zip(st, tasks) if t.prio == des.LP]
    assert all(s["accepted"] == s["released"] for s in hp)          # HP jobs are never rejected
    assert sum(s["completed"] for s in st) == sum(s["accepted"] for s in st)
    # determinism: same inputs, same trace
    m2 = des.SchedulerModel([1] * len(ts.partitions), tasks)
    assert des.run_virtual(m2, allc, et) == tr


def test_staging_reduces_hp_blocking():
    """Qualitative direction of the 'No Staging' ablation (Sec. VI): with k=1 an HP job can wait for a whole LP
    job, with k stages only for one stage, so the worst HP response does not get better without staging."""
    def run(k):
        lp_total, hp_total = 9000, 3000
        tasks = [des.TaskParam(10_000, 10_000, des.HP, [hp_total // k] * k), des.TaskParam(20_000, 20_000, des.LP, [lp_total // k] * k)]
        et = [[[[hp_total // k] * 40] for _ in range(k)], [[[lp_total // k] * 40] for _ in range(k)]]
        cmds = sorted([("release", 500 + m * 10_000, 0) for m in range(40)] + [("release", m * 20_000, 1) for m in range(20)],
                      key=lambda c: (c[1], c[2]))
        m = des.SchedulerModel([1], tasks)
        des.run_virtual(m, cmds, et)
        return max(m.stats()[0]["responses"])
    assert run(3) < run(1)


def test_replay_reproduces_a_virtual_trace():
    """Feeding a trace's own input events (release / command / completion times) back must regenerate it."""
    g, cmds, et, want = load_golden("sched_admission_migration.json")
    m = model_from_golden(g)
    rec = des.run_virtual(m, cmds, et)
    # in a real-time run the dispatch pass follows every input; at distinct event times both drivers coincide
    g2, cmds2, et2, want2 = load_golden("sched_hp_preempts_lp.json")
    m2 = model_from_golden(g2)
    rec2 = des.run_virtual(m2, cmds2, et2)
    again = des.run_replay(model_from_golden(g2), rec2)
    assert again == rec2
