"""Discrete-event model of the DARIS scheduler -- TEST INFRASTRUCTURE ONLY.

Pure-Python integers (nanoseconds, Q32 utilisations).  The steps follow the
paper's Sec. III (task model, MRET eq. 1-2, utilisation eq. 3-7, virtual
deadline eq. 8, partition size formula of Sec. III-C2) and Sec. IV (Algorithm 1,
admission test eq. 11-12, stage scheduler), in the paper's notation.  Where the
paper is silent the reading taken is written next to the step.

Nothing here is shared with the HIP library; the library's host scheduler is a
separate C++ implementation that must reproduce this model's trace bit for bit.

Trace record (one tuple per event, mirrors the library's 32-byte record):
    (seq, t_ns, type, level, stage, partition, task, stream, job, aux)
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

LP, HP = 0, 1

# record types
RELEASE, ACCEPT, REJECT, MIGRATE, DISPATCH, STAGE_DONE, JOB_DONE, QUEUED, CMD_MIGRATE = range(1, 10)
TYPE_NAMES = {RELEASE: "RELEASE", ACCEPT: "ACCEPT", REJECT: "REJECT", MIGRATE: "MIGRATE", DISPATCH: "DISPATCH",
              STAGE_DONE: "STAGE_DONE", JOB_DONE: "JOB_DONE", QUEUED: "QUEUED", CMD_MIGRATE: "CMD_MIGRATE"}
REJECT_ADMISSION, REJECT_OVERRUN = 1, 2
NO_JOB = 0xFFFFFFFF

# scheduler switches (ablations of Sec. VI "modules contribution", and the HP admission variant)
F_NO_LAST, F_NO_PRIOR, F_NO_FIXED, F_HP_ADMISSION = 1, 2, 4, 8

Q = 1 << 32  # utilisations are integers in units of 2^-32


def ceil_even(num: int, den: int) -> int:
    """Smallest even integer >= num/den (Sec. III-C2: "rounds up to the nearest even number")."""
    return 2 * (-((-num) // (2 * den)))


def partition_cus(os_num: int, os_den: int, n_max: int, n_c: int) -> int:
    """N_SM = ceil_even(OS * N_SM,max / N_c) with OS = os_num/os_den (Sec. III-C2)."""
    return ceil_even(os_num * n_max, os_den * n_c)


def mret_of(samples: Sequence[int], ws: int, afet: int) -> int:
    """Eq. (1): max over the last `ws` executions; fewer than ws samples -> max of those;
    no sample yet -> the stage's AFET (Sec. IV-A1, t = 0 case)."""
    if not samples:
        return afet
    return max(samples[-ws:])


def utilisation(mret_i: int, period: int) -> int:
    """Eq. (3) in Q32: floor(mret_i * 2^32 / T_i)."""
    return (mret_i * Q) // period


def virtual_deadlines(release: int, deadline: int, mret_stages: Sequence[int]) -> List[int]:
    """Eq. (8), cumulative from the release: vd_j = r + floor(D_i * S_j / S_n), S_j = sum_{l<=j} mret_{i,l}.

    The per-stage shares of eq. (8) sum to D_i, so the last value is r + D_i exactly."""
    total = sum(mret_stages)
    out, s = [], 0
    for m in mret_stages:
        s += m
        out.append(release + (deadline * s) // total)
    return out


def stage_level(prio: int, is_last: bool, prev_missed: bool, flags: int = 0) -> int:
    """Sec. IV-B2: eight fixed levels. HP over LP first, then last stage, then predecessor-missed."""
    if flags & F_NO_FIXED:
        return 0
    lvl = 4 * (1 if prio == HP else 0)
    if is_last and not (flags & F_NO_LAST):
        lvl += 2
    if prev_missed and not (flags & F_NO_PRIOR):
        lvl += 1
    return lvl


@dataclass
class TaskParam:
    period: int
    deadline: int
    prio: int
    afet: List[int]  # per-stage AFET, ns (len = number of stages)


@dataclass
class _Job:
    task: int
    index: int
    release: int
    vd: List[int]
    part: int
    u: int = 0
    stage: int = 0            # next / current stage
    prev_missed: bool = False
    running: bool = False
    stream: int = -1
    t_dispatch: int = 0


@dataclass
class _TaskState:
    p: TaskParam
    ctx: int = 0
    rings: List[List[int]] = field(default_factory=list)
    active: Optional[_Job] = None
    fifo: List[Tuple[int, int]] = field(default_factory=list)  # queued HP releases (job, release)
    pending_migrate: int = -1
    n_released: int = 0
    accepted: int = 0
    completed: int = 0
    missed: int = 0
    rej_adm: int = 0
    rej_over: int = 0
    responses: List[int] = field(default_factory=list)


class SchedulerModel:
    """State + the four transitions (release, migrate command, stage done, dispatch)."""

    def __init__(self, n_streams: Sequence[int], tasks: Sequence[TaskParam], ws: int = 5, flags: int = 0):
        self.n_streams = list(n_streams)
        self.nc = len(self.n_streams)
        self.ws = ws
        self.flags = flags
        self.tasks = [_TaskState(p=t, rings=[[] for _ in t.afet]) for t in tasks]
        self.streams: List[List[Optional[_Job]]] = [[None] * ns for ns in self.n_streams]
        self.ready: List[List[_Job]] = [[] for _ in range(self.nc)]
        self.ula = [0] * self.nc            # U^{l,a}_k: stored u of active LP jobs
        self.trace: List[tuple] = []
        self.committed = False

    # ---- bookkeeping -----------------------------------------------------------------------------
    def _rec(self, t, typ, level=0, stage=0, part=0, task=0, stream=0, job=0, aux=0):
        self.trace.append((len(self.trace), t, typ, level, stage, part, task, stream, job, aux & 0xFFFFFFFF))

    def mret_stage(self, i: int, j: int) -> int:
        ts = self.tasks[i]
        return mret_of(ts.rings[j], self.ws, ts.p.afet[j])

    def mret_task(self, i: int) -> int:  # eq. (2)
        return sum(self.mret_stage(i, j) for j in range(len(self.tasks[i].p.afet)))

    def u_task(self, i: int) -> int:  # eq. (3)
        return utilisation(self.mret_task(i), self.tasks[i].p.period)

    def u_high_total(self, k: int) -> int:  # eq. (4): all HP tasks whose context is k
        return sum(self.u_task(i) for i, ts in enumerate(self.tasks) if ts.p.prio == HP and ts.ctx == k)

    def backlog(self, k: int) -> int:
        """Sum of current MRETs of every unfinished stage of the active jobs placed in partition k."""
        s = 0
        for i, ts in enumerate(self.tasks):
            jb = ts.active
            if jb is not None and jb.part == k:
                s += sum(self.mret_stage(i, j) for j in range(jb.stage, len(ts.p.afet)))
        return s

    # ---- offline phase: Algorithm 1 --------------------------------------------------------------
    def commit(self):
        """HP tasks, then LP tasks, each in registration order, go to the context of minimum total
        utilisation (ties: lowest index); u_i(0) = afet_i / T_i."""
        if self.committed:
            return
        total = [0] * self.nc
        for prio in (HP, LP):
            for i, ts in enumerate(self.tasks):
                if ts.p.prio != prio:
                    continue
                k = min(range(self.nc), key=lambda c: (total[c], c))
                ts.ctx = k
                total[k] += utilisation(sum(ts.p.afet), ts.p.period)
        self.committed = True

    # ---- online phase ----------------------------------------------------------------------------
    def admission_ok(self, k: int, u: int) -> bool:
        """Eq. (11)-(12): U^{l,a}_k + u < N_s - U^{h,t}_k, strict, in Q32 integers."""
        return self.ula[k] + u + self.u_high_total(k) < self.n_streams[k] * Q

    def release(self, t: int, i: int, r: Optional[int] = None) -> int:
        """Release processed at time t; deadlines and response time count from the nominal release r <= t
        (r = t in virtual time; a real-time run may process a release slightly late)."""
        self.commit()
        r = t if r is None else min(r, t)
        ts = self.tasks[i]
        m = ts.n_released
        ts.n_released += 1
        self._rec(t, RELEASE, part=ts.ctx, task=i, job=m, aux=t - r)
        if ts.active is not None:
            if ts.p.prio == HP and not (self.flags & F_HP_ADMISSION):
                ts.fifo.append((m, r))               # HP jobs are always scheduled: wait behind the running job
                self._rec(t, QUEUED, part=ts.ctx, task=i, job=m)
                return QUEUED
            ts.rej_over += 1                         # previous job of the task still active
            self._rec(t, REJECT, part=ts.ctx, task=i, job=m, aux=REJECT_OVERRUN)
            return REJECT
        return self._start_job(t, i, m, r, queued=False)

    def _start_job(self, t: int, i: int, m: int, r: int, queued: bool) -> int:
        ts = self.tasks[i]
        n = len(ts.p.afet)
        u = 0
        result = ACCEPT
        k = ts.ctx
        if ts.p.prio == HP:
            # HP jobs are not tested (Sec. IV-B1).  Overload+HPA variant (Sec. VI-I): the job must fit its own
            # context, whose U^{h,t} already contains this task; it is dropped otherwise, never migrated.
            if (self.flags & F_HP_ADMISSION) and not self.admission_ok(k, 0):
                ts.rej_adm += 1
                self._rec(t, REJECT, part=k, task=i, job=m, aux=REJECT_ADMISSION)
                return REJECT
        else:
            u = self.u_task(i)
            if not self.admission_ok(k, u):
                cands = [c for c in range(self.nc) if c != ts.ctx and self.admission_ok(c, u)]
                if not cands:
                    ts.rej_adm += 1
                    self._rec(t, REJECT, part=ts.ctx, task=i, job=m, aux=REJECT_ADMISSION)
                    return REJECT
                mi = self.mret_task(i)
                # earliest predicted finish: t + (backlog_k + mret_i) / N_s,k ; ties -> lowest index
                k = min(cands, key=lambda c: ((self.backlog(c) + mi) // self.n_streams[c], c))
                self._rec(t, MIGRATE, part=k, task=i, job=m, aux=ts.ctx)
                ts.ctx = k
                result = MIGRATE
            self.ula[k] += u
        vd = virtual_deadlines(r, ts.p.deadline, [self.mret_stage(i, j) for j in range(n)])
        jb = _Job(task=i, index=m, release=r, vd=vd, part=k, u=u)
        ts.active = jb
        ts.accepted += 1
        self._rec(t, ACCEPT, part=k, task=i, job=m, aux=1 if queued else 0)
        self.ready[k].append(jb)
        return result

    def _apply_migration(self, t: int, i: int, target: int):
        ts = self.tasks[i]
        ts.pending_migrate = -1
        if target == ts.ctx:
            return
        jb = ts.active
        self._rec(t, MIGRATE, part=target, task=i, job=jb.index if jb else NO_JOB, aux=ts.ctx | (1 << 8))
        if jb is not None:
            if jb in self.ready[jb.part]:
                self.ready[jb.part].remove(jb)
                self.ready[target].append(jb)
            if ts.p.prio == LP:
                self.ula[jb.part] -= jb.u
                self.ula[target] += jb.u
            jb.part = target
        ts.ctx = target

    def migrate_command(self, t: int, i: int, target: int):
        """Forced migration: applied now unless a stage of the task is running, else at its boundary."""
        self.commit()
        ts = self.tasks[i]
        self._rec(t, CMD_MIGRATE, part=target, task=i, job=ts.active.index if ts.active else NO_JOB)
        if ts.active is not None and ts.active.running:
            ts.pending_migrate = target
        else:
            self._apply_migration(t, i, target)

    def stage_done(self, t: int, i: int):
        ts = self.tasks[i]
        jb = ts.active
        assert jb is not None and jb.running
        j = jb.stage
        n = len(ts.p.afet)
        et = t - jb.t_dispatch
        ring = ts.rings[j]
        ring.append(et)
        del ring[:-self.ws]
        missed = t > jb.vd[j]
        self._rec(t, STAGE_DONE, stage=j, part=jb.part, task=i, stream=jb.stream, job=jb.index, aux=int(missed))
        self.streams[jb.part][jb.stream] = None
        jb.running = False
        if j + 1 < n:
            jb.stage = j + 1
            jb.prev_missed = missed
            if ts.pending_migrate >= 0:
                self._apply_migration(t, i, ts.pending_migrate)
            self.ready[jb.part].append(jb)
            return
        # job finished
        late = t > jb.release + ts.p.deadline
        ts.completed += 1
        ts.missed += int(late)
        ts.responses.append(t - jb.release)
        self._rec(t, JOB_DONE, stage=j, part=jb.part, task=i, stream=jb.stream, job=jb.index, aux=int(late))
        if ts.p.prio == LP:
            self.ula[jb.part] -= jb.u
        ts.active = None
        if ts.pending_migrate >= 0:
            self._apply_migration(t, i, ts.pending_migrate)
        if ts.fifo:
            m, r = ts.fifo.pop(0)
            self._start_job(t, i, m, r, queued=True)

    def _pick(self, k: int) -> _Job:
        def key(jb: _Job):
            ts = self.tasks[jb.task]
            lvl = stage_level(ts.p.prio, jb.stage == len(ts.p.afet) - 1, jb.prev_missed, self.flags)
            return (-lvl, jb.vd[jb.stage], jb.task, jb.index)
        return min(self.ready[k], key=key)

    def dispatch(self, t: int, time_of=None) -> List[_Job]:
        """Every idle stream takes the ready stage of highest level, then earliest absolute virtual
        deadline, then lowest task id, then lowest job index (Sec. IV-B2)."""
        started = []
        for k in range(self.nc):
            for s in range(self.n_streams[k]):
                if self.streams[k][s] is not None or not self.ready[k]:
                    continue
                jb = self._pick(k)
                self.ready[k].remove(jb)
                ts = self.tasks[jb.task]
                lvl = stage_level(ts.p.prio, jb.stage == len(ts.p.afet) - 1, jb.prev_missed, self.flags)
                td = t if time_of is None else time_of(t)
                jb.running, jb.stream, jb.t_dispatch = True, s, td
                self.streams[k][s] = jb
                self._rec(td, DISPATCH, level=lvl, stage=jb.stage, part=k, task=jb.task, stream=s, job=jb.index,
                          aux=jb.vd[jb.stage] - jb.release)
                started.append(jb)
        return started

    # ---- metrics (Sec. V: DMR = missed / accepted) -------------------------------------------------
    def stats(self):
        out = []
        for ts in self.tasks:
            out.append(dict(released=ts.n_released, accepted=ts.accepted, completed=ts.completed, missed=ts.missed,
                            rejected_admission=ts.rej_adm, rejected_overrun=ts.rej_over,
                            responses=list(ts.responses), ctx=ts.ctx))
        return out


def run_virtual(model: SchedulerModel, commands, et_table):
    """Virtual-time run.

    commands: list of ("release", t, task) / ("migrate", t, task, partition), sorted by time (stable).
    et_table[task][stage][partition][job] -> execution time in ns (>= 1).
    Order at equal time: stage completions (by task, job), then commands in list order, then dispatch.
    """
    model.commit()
    heap: list = []
    ci = 0
    while ci < len(commands) or heap:
        t_cmd = commands[ci][1] if ci < len(commands) else None
        t_done = heap[0][0] if heap else None
        t = t_cmd if t_done is None else (t_done if t_cmd is None else min(t_cmd, t_done))
        while heap and heap[0][0] == t:
            _, i, _m = heapq.heappop(heap)
            model.stage_done(t, i)
        while ci < len(commands) and commands[ci][1] == t:
            c = commands[ci]
            ci += 1
            if c[0] == "release":
                model.release(t, c[2])
            else:
                model.migrate_command(t, c[2], c[3])
        for jb in model.dispatch(t):
            et = int(et_table[jb.task][jb.stage][jb.part][jb.index])
            assert et >= 1
            heapq.heappush(heap, (t + et, jb.task, jb.index))
    return model.trace


def run_replay(model: SchedulerModel, recorded):
    """Replay a trace recorded by a real-time run.

    Inputs taken from the recording: RELEASE, CMD_MIGRATE and STAGE_DONE events (type, time, task) and the
    clock value of each DISPATCH.  Everything else (accept / reject / migrate decisions, which stage is
    dispatched where and at what level, miss flags) is recomputed.  A dispatch pass follows every input."""
    model.commit()
    n = len(recorded)

    def next_dispatch_time(default):
        idx = len(model.trace)  # the recorded record aligned with the one about to be produced
        if idx < n and recorded[idx][2] == DISPATCH:
            return recorded[idx][1]
        return default

    for rec in recorded:
        _, t, typ, _lvl, _stage, part, task, _stream, _job, _aux = rec
        if typ == RELEASE:
            model.release(t, task, t - _aux)
        elif typ == CMD_MIGRATE:
            model.migrate_command(t, task, part)
        elif typ == STAGE_DONE:
            jb = model.tasks[task].active
            if jb is None or not jb.running:
                break  # recording inconsistent with the model: stop, the comparison shows where
            model.stage_done(t, task)
        else:
            continue
        model.dispatch(t, time_of=next_dispatch_time)
    return model.trace
