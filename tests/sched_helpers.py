"""Helpers shared by the scheduler tests: golden loader, an independent trace invariant checker and
two textbook single-processor simulators."""
import json
import os

from oracle import des

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
NAME2TYPE = {v: k for k, v in des.TYPE_NAMES.items()}


def load_golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        g = json.load(f)
    npart = len(g["partitions"])
    ntask = len(g["tasks"])
    et = []
    for i in range(ntask):
        per_stage = g.get("et", {}).get(str(i), [])
        et.append([[list(jobs) for _ in range(npart)] for jobs in per_stage])
    cmds = [tuple(c) for c in g.get("commands", [])]
    trace = [(s, r[0], NAME2TYPE[r[1]], *r[2:]) for s, r in enumerate(g["trace"])]
    return g, cmds, et, trace


GOLDEN_FLAGS = {"no_last": des.F_NO_LAST, "no_prior": des.F_NO_PRIOR, "no_fixed": des.F_NO_FIXED, "hp_admission": des.F_HP_ADMISSION}


def golden_flags(g):
    """Scheduler switches a golden file asks for (its "flags" list), as the oracle's flag bits."""
    f = 0
    for name in g.get("flags", []):
        f |= GOLDEN_FLAGS[name]
    return f


def model_from_golden(g, flags=None):
    flags = golden_flags(g) if flags is None else flags
    tasks = [des.TaskParam(t["period"], t["deadline"], t["prio"], list(t["afet"])) for t in g["tasks"]]
    return des.SchedulerModel(g["partitions"], tasks, ws=g.get("ws", 5), flags=flags)


def check_trace_invariants(trace, n_streams, prios, n_stages, flags=0):
    """Properties every valid trace has, checked without re-running the scheduling rule:
    at most N_s running stages per partition, stages of a job in order and not overlapping, a dispatched
    stage is maximal in (level, -virtual deadline) among the stages ready in its partition, work
    conservation (no idle stream while a stage is ready after a dispatch pass) and the HP-wait invariant
    (while an HP stage is ready in partition k no LP stage is dispatched on k)."""
    nc = len(n_streams)
    running = [dict() for _ in range(nc)]            # stream -> (task, job, stage)
    ready = [dict() for _ in range(nc)]              # (task, job) -> dict(stage, prev_missed, vd_rel unknown)
    active = {}                                      # task -> dict(job, part, next_stage, release)
    release_time = {}
    last_t = None
    for idx, (seq, t, typ, level, stage, part, task, stream, job, aux) in enumerate(trace):
        assert seq == idx
        if last_t is not None:
            assert t >= last_t, "time must not go backwards"
        last_t = t
        if typ == des.RELEASE:
            release_time[(task, job)] = t
        elif typ == des.ACCEPT:
            assert task not in active, "one active job per task"
            active[task] = dict(job=job, part=part, next=0)
            ready[part][(task, job)] = dict(stage=0, prev_missed=False)
        elif typ == des.MIGRATE:
            if task in active:
                a = active[task]
                if (task, a["job"]) in ready[a["part"]]:
                    ready[part][(task, a["job"])] = ready[a["part"]].pop((task, a["job"]))
                a["part"] = part
            forced = aux >> 8
            if prios[task] == des.HP:
                assert forced, "HP tasks migrate only when forced"
        elif typ == des.DISPATCH:
            assert stream not in running[part] and len(running[part]) < n_streams[part]
            ent = ready[part].pop((task, job))
            assert ent["stage"] == stage == active[task]["next"]
            want = des.stage_level(prios[task], stage == n_stages[task] - 1, ent["prev_missed"], flags)
            assert level == want, (idx, level, want)
            hp_ready = any(prios[tk] == des.HP for (tk, _j) in ready[part])
            if prios[task] == des.LP and not (flags & des.F_NO_FIXED):
                assert not hp_ready, "LP stage dispatched while an HP stage was ready in the partition"
            running[part][stream] = (task, job, stage)
            ent["vd_abs"] = release_time[(task, job)] + aux
            # maximality in level among what stays ready is checked at the end of the pass (below)
            ready_levels = [des.stage_level(prios[tk], e["stage"] == n_stages[tk] - 1, e["prev_missed"], flags)
                            for (tk, _j), e in ready[part].items()]
            assert all(level >= rl for rl in ready_levels), "dispatched stage is not of maximal level"
        elif typ == des.STAGE_DONE:
            assert running[part].pop(stream) == (task, job, stage)
            a = active[task]
            a["next"] = stage + 1
            if stage + 1 < n_stages[task]:
                ready[part][(task, job)] = dict(stage=stage + 1, prev_missed=bool(aux & 1))
        elif typ == des.JOB_DONE:
            assert active[task]["next"] == n_stages[task]
            ready[part].pop((task, job), None)
            del active[task]
        # work conservation: when the next record belongs to a later time (or the trace ends), no partition
        # may hold both an idle stream and a ready stage
        nxt = trace[idx + 1] if idx + 1 < len(trace) else None
        if nxt is None or nxt[1] > t:
            for k in range(nc):
                # a MIGRATE at a boundary moves the entry after STAGE_DONE re-added it: fix up lazily
                for key in list(ready[k]):
                    if key[0] in active and active[key[0]]["part"] != k:
                        ready[active[key[0]]["part"]][key] = ready[k].pop(key)
            for k in range(nc):
                assert not (ready[k] and len(running[k]) < n_streams[k]), (idx, k, ready[k], running[k])
    return True


def np_edf_single(jobs):
    """Textbook non-preemptive EDF on one processor. jobs: list of (release, exec, abs_deadline, id).
    Returns list of (start, finish, id) in execution order; ties by id."""
    pending = sorted(jobs)
    t, out, readyq = 0, [], []
    pending = list(pending)
    while pending or readyq:
        while pending and pending[0][0] <= t:
            r, c, d, i = pending.pop(0)
            readyq.append((d, i, c))
        if not readyq:
            t = pending[0][0]
            continue
        readyq.sort()
        d, i, c = readyq.pop(0)
        out.append((t, t + c, i))
        t += c
    return out


def np_fixed_priority_single(jobs):
    """Textbook non-preemptive fixed-priority on one processor. jobs: (release, exec, prio(high wins), id)."""
    pending = sorted(jobs)
    t, out, readyq = 0, [], []
    while pending or readyq:
        while pending and pending[0][0] <= t:
            r, c, p, i = pending.pop(0)
            readyq.append((-p, r, i, c))
        if not readyq:
            t = pending[0][0]
            continue
        readyq.sort()
        _p, _r, i, c = readyq.pop(0)
        out.append((t, t + c, i))
        t += c
    return out
