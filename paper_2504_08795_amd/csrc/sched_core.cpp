#include "sched_core.h"

#include <algorithm>

namespace daris {

typedef unsigned __int128 u128;
static const u128 kOne = (u128)1 << 32;  // utilisation 1.0 in Q32

int64_t ceil_even(int64_t num, int64_t den) {
  // 2 * ceil(num / (2 den)) for positive arguments
  int64_t d2 = 2 * den;
  return 2 * ((num + d2 - 1) / d2);
}

int SchedCore::add_partition(int n_streams) {
  Part p;
  p.n_streams = n_streams;
  p.running.assign(n_streams, -1);
  parts_.push_back(p);
  return (int)parts_.size() - 1;
}

void SchedCore::set_streams(int part, int n_streams) {
  parts_[part].n_streams = n_streams;
  parts_[part].running.assign(n_streams, -1);
}

int SchedCore::add_task(int64_t period, int64_t deadline, int prio, int n_stages) {
  Task t;
  t.period = period;
  t.deadline = deadline;
  t.prio = prio;
  tasks_.push_back(t);
  set_stage_count((int)tasks_.size() - 1, n_stages);
  return (int)tasks_.size() - 1;
}

void SchedCore::set_stage_count(int task, int n_stages) {
  Task& t = tasks_[task];
  t.afet.assign(n_stages, 1);
  t.ring.assign(n_stages, std::deque<int64_t>());
}

void SchedCore::set_afet(int task, int stage, int64_t ns) { tasks_[task].afet[stage] = ns; }

void SchedCore::rec(int64_t t, uint8_t type, int level, int stage, int part, int task, int stream, uint32_t job,
                    uint32_t aux) {
  // an unread trace is capped at 4 Mi records (128 MiB): the older half is dropped and counted
  if (trace_.size() >= (size_t)4 << 20) {
    const size_t half = trace_.size() / 2;
    trace_.erase(trace_.begin(), trace_.begin() + half);
    dropped_ += half;
  }
  TraceRec r;
  r.seq = seq_++;
  r.t_ns = t;
  r.type = type;
  r.level = (uint8_t)level;
  r.stage = (uint8_t)stage;
  r.partition = (uint8_t)part;
  r.task = (uint16_t)task;
  r.stream = (uint16_t)stream;
  r.job = job;
  r.aux = aux;
  trace_.push_back(r);
}

// eq. (1): maximum of the recorded window; the AFET stands in until the stage has run once.
int64_t SchedCore::mret_stage(int task, int stage) const {
  const Task& t = tasks_[task];
  const std::deque<int64_t>& w = t.ring[stage];
  if (w.empty()) return t.afet[stage];
  return *std::max_element(w.begin(), w.end());
}

// eq. (2)
int64_t SchedCore::mret_task(int task) const {
  int64_t s = 0;
  for (int j = 0; j < n_stages(task); ++j) s += mret_stage(task, j);
  return s;
}

// eq. (3), Q32
u128 SchedCore::u_task(int task) const { return ((u128)mret_task(task) << 32) / (u128)tasks_[task].period; }

// eq. (4): every HP task whose context is `part`, active or not
u128 SchedCore::u_high_total(int part) const {
  u128 s = 0;
  for (int i = 0; i < n_tasks(); ++i)
    if (tasks_[i].prio == 1 && tasks_[i].ctx == part) s += u_task(i);
  return s;
}

// eq. (11)-(12): U^{l,a}_k + u < N_s - U^{h,t}_k, rearranged so that nothing goes negative
bool SchedCore::admission_ok(int part, u128 u) const {
  return parts_[part].ula + u + u_high_total(part) < (u128)parts_[part].n_streams * kOne;
}

// Work still booked in a partition: current MRET of every unfinished stage of the jobs placed there.
int64_t SchedCore::backlog(int part) const {
  int64_t s = 0;
  for (int i = 0; i < n_tasks(); ++i) {
    const Task& t = tasks_[i];
    if (!t.active || t.job.part != part) continue;
    for (int j = t.job.stage; j < n_stages(i); ++j) s += mret_stage(i, j);
  }
  return s;
}

void SchedCore::commit() {
  if (committed_) return;
  std::vector<u128> total(parts_.size(), 0);
  for (int prio = 1; prio >= 0; --prio) {
    for (int i = 0; i < n_tasks(); ++i) {
      Task& t = tasks_[i];
      if (t.prio != prio) continue;
      int best = 0;
      for (int k = 1; k < n_parts(); ++k)
        if (total[k] < total[best]) best = k;
      t.ctx = best;
      int64_t afet = 0;
      for (int64_t a : t.afet) afet += a;
      total[best] += ((u128)afet << 32) / (u128)t.period;
    }
  }
  committed_ = true;
}

Decision SchedCore::release(int64_t t, int task, int64_t r, uint32_t* job_out) {
  commit();
  if (r > t) r = t;
  Task& tk = tasks_[task];
  uint32_t m = tk.n_released++;
  if (job_out) *job_out = m;
  tk.st.released++;
  if (tk.st.first_release < 0) tk.st.first_release = r;
  rec(t, T_RELEASE, 0, 0, tk.ctx, task, 0, m, (uint32_t)(t - r));
  if (tk.active) {
    if (tk.prio == 1 && !(flags_ & CF_HP_ADMISSION)) {
      tk.fifo.push_back(std::make_pair(m, r));
      rec(t, T_QUEUED, 0, 0, tk.ctx, task, 0, m, 0);
      return D_QUEUED;
    }
    tk.st.rej_over++;
    rec(t, T_REJECT, 0, 0, tk.ctx, task, 0, m, 2);
    return D_REJECT_OVERRUN;
  }
  return start_job(t, task, m, r, false);
}

Decision SchedCore::start_job(int64_t t, int task, uint32_t m, int64_t r, bool queued) {
  Task& tk = tasks_[task];
  const int n = n_stages(task);
  int k = tk.ctx;
  u128 u = 0;
  Decision result = D_ACCEPTED;
  if (tk.prio == 1) {
    if ((flags_ & CF_HP_ADMISSION) && !admission_ok(k, 0)) {
      tk.st.rej_adm++;
      rec(t, T_REJECT, 0, 0, k, task, 0, m, 1);
      return D_REJECT_ADMISSION;
    }
  } else {
    u = u_task(task);
    if (!admission_ok(k, u)) {
      // other contexts that pass; the one whose predicted finish (backlog_k + mret_i) / N_s,k is earliest wins
      int best = -1;
      int64_t best_fin = 0;
      const int64_t mi = mret_task(task);
      for (int c = 0; c < n_parts(); ++c) {
        if (c == tk.ctx || !admission_ok(c, u)) continue;
        int64_t fin = (backlog(c) + mi) / parts_[c].n_streams;
        if (best < 0 || fin < best_fin) {
          best = c;
          best_fin = fin;
        }
      }
      if (best < 0) {
        tk.st.rej_adm++;
        rec(t, T_REJECT, 0, 0, tk.ctx, task, 0, m, 1);
        return D_REJECT_ADMISSION;
      }
      rec(t, T_MIGRATE, 0, 0, best, task, 0, m, (uint32_t)tk.ctx);
      tk.ctx = k = best;
      result = D_MIGRATED;
    }
    parts_[k].ula += u;
  }
  Job& jb = tk.job;
  jb = Job();
  jb.index = m;
  jb.release = r;
  jb.part = k;
  jb.u = u;
  // eq. (8), cumulative from the release, snapshot of the current MRETs
  u128 total = (u128)mret_task(task), run = 0;
  jb.vd.resize(n);
  for (int j = 0; j < n; ++j) {
    run += (u128)mret_stage(task, j);
    jb.vd[j] = r + (int64_t)(((u128)tk.deadline * run) / total);
  }
  tk.active = true;
  tk.st.accepted++;
  rec(t, T_ACCEPT, 0, 0, k, task, 0, m, queued ? 1u : 0u);
  jb.ready = true;
  parts_[k].ready.push_back(task);
  return result;
}

void SchedCore::apply_migration(int64_t t, int task, int target) {
  Task& tk = tasks_[task];
  tk.pending = -1;
  if (target == tk.ctx) return;
  rec(t, T_MIGRATE, 0, 0, target, task, 0, tk.active ? tk.job.index : 0xFFFFFFFFu, (uint32_t)tk.ctx | 256u);
  if (tk.active) {
    Job& jb = tk.job;
    if (jb.ready) {
      std::vector<int>& q = parts_[jb.part].ready;
      q.erase(std::find(q.begin(), q.end(), task));
      parts_[target].ready.push_back(task);
    }
    if (tk.prio == 0) {
      parts_[jb.part].ula -= jb.u;
      parts_[target].ula += jb.u;
    }
    jb.part = target;
  }
  tk.ctx = target;
}

void SchedCore::migrate_command(int64_t t, int task, int target) {
  commit();
  Task& tk = tasks_[task];
  rec(t, T_CMD_MIGRATE, 0, 0, target, task, 0, tk.active ? tk.job.index : 0xFFFFFFFFu, 0);
  if (tk.active && tk.job.running)
    tk.pending = target;
  else
    apply_migration(t, task, target);
}

bool SchedCore::stage_done(int64_t t, int task) {
  Task& tk = tasks_[task];
  Job& jb = tk.job;
  const int j = jb.stage, n = n_stages(task);
  std::deque<int64_t>& w = tk.ring[j];
  w.push_back(t - jb.t_dispatch);
  while ((int)w.size() > ws_) w.pop_front();
  const bool missed = t > jb.vd[j];
  rec(t, T_STAGE_DONE, 0, j, jb.part, task, jb.stream, jb.index, missed ? 1u : 0u);
  parts_[jb.part].running[jb.stream] = -1;
  jb.running = false;
  if (j + 1 < n) {
    jb.stage = j + 1;
    jb.prev_missed = missed;
    if (tk.pending >= 0) apply_migration(t, task, tk.pending);
    jb.ready = true;
    parts_[jb.part].ready.push_back(task);
    return false;
  }
  const bool late = t > jb.release + tk.deadline;
  const int64_t resp = t - jb.release;
  TaskStats& st = tk.st;
  if (st.completed == 0 || resp < st.resp_min) st.resp_min = resp;
  if (st.completed == 0 || resp > st.resp_max) st.resp_max = resp;
  st.resp_sum += resp;
  st.completed++;
  st.missed += late ? 1 : 0;
  st.last_finish = t;
  rec(t, T_JOB_DONE, 0, j, jb.part, task, jb.stream, jb.index, late ? 1u : 0u);
  if (tk.prio == 0) parts_[jb.part].ula -= jb.u;
  tk.active = false;
  if (tk.pending >= 0) apply_migration(t, task, tk.pending);
  if (!tk.fifo.empty()) {
    std::pair<uint32_t, int64_t> q = tk.fifo.front();
    tk.fifo.pop_front();
    start_job(t, task, q.first, q.second, true);
  }
  return true;
}

// Sec. IV-B2: HP over LP, then last stage, then "predecessor missed its virtual deadline".
int SchedCore::level_of(const Task& tk) const {
  if (flags_ & CF_NO_FIXED) return 0;
  int lvl = tk.prio == 1 ? 4 : 0;
  if (tk.job.stage == (int)tk.afet.size() - 1 && !(flags_ & CF_NO_LAST)) lvl += 2;
  if (tk.job.prev_missed && !(flags_ & CF_NO_PRIOR)) lvl += 1;
  return lvl;
}

void SchedCore::dispatch(int64_t t, std::vector<Launch>* out) {
  for (int k = 0; k < n_parts(); ++k) {
    Part& p = parts_[k];
    for (int s = 0; s < p.n_streams; ++s) {
      if (p.running[s] >= 0 || p.ready.empty()) continue;
      // best = highest level, then earliest absolute virtual deadline, then lowest task id (one job per task)
      size_t bi = 0;
      for (size_t q = 1; q < p.ready.size(); ++q) {
        const Task& a = tasks_[p.ready[q]];
        const Task& b = tasks_[p.ready[bi]];
        const int la = level_of(a), lb = level_of(b);
        const int64_t da = a.job.vd[a.job.stage], db = b.job.vd[b.job.stage];
        if (la > lb || (la == lb && (da < db || (da == db && p.ready[q] < p.ready[bi])))) bi = q;
      }
      const int task = p.ready[bi];
      p.ready.erase(p.ready.begin() + bi);
      Task& tk = tasks_[task];
      Job& jb = tk.job;
      jb.ready = false;
      jb.running = true;
      jb.stream = s;
      jb.t_dispatch = t;
      p.running[s] = task;
      rec(t, T_DISPATCH, level_of(tk), jb.stage, k, task, s, jb.index, (uint32_t)(jb.vd[jb.stage] - jb.release));
      if (out) {
        Launch l;
        l.task = task;
        l.stage = jb.stage;
        l.part = k;
        l.stream = s;
        l.job = jb.index;
        out->push_back(l);
      }
    }
  }
}

bool SchedCore::idle() const {
  for (const Task& t : tasks_)
    if (t.active || !t.fifo.empty()) return false;
  return true;
}

}  // namespace daris
