// Host decision core of the DARIS scheduler: a pure integer function of an ordered stream of input events
// (job releases, forced-migration commands, stage completions).  It owns no clock and no GPU object; the
// virtual-time and real-time drivers feed it and act on what dispatch() returns.
//
// Follows Sec. III (task model, MRET eq. 1-2, utilisation eq. 3-7, virtual deadlines eq. 8) and Sec. IV
// (Algorithm 1, admission test eq. 11-12, the eight-level stage scheduler with EDF inside a level).
#pragma once
#include <cstdint>
#include <deque>
#include <vector>

namespace daris {

enum RecType : uint8_t {
  T_RELEASE = 1, T_ACCEPT, T_REJECT, T_MIGRATE, T_DISPATCH, T_STAGE_DONE, T_JOB_DONE, T_QUEUED, T_CMD_MIGRATE
};
enum Decision : int32_t { D_ACCEPTED = 1, D_MIGRATED, D_REJECT_ADMISSION, D_REJECT_OVERRUN, D_QUEUED };
enum CoreFlags : int { CF_NO_LAST = 1, CF_NO_PRIOR = 2, CF_NO_FIXED = 4, CF_HP_ADMISSION = 8 };

struct TraceRec {  // 32 bytes, little-endian
  uint64_t seq;
  int64_t t_ns;
  uint8_t type, level, stage, partition;
  uint16_t task, stream;
  uint32_t job;
  uint32_t aux;
};
static_assert(sizeof(TraceRec) == 32, "trace record must be 32 bytes");

struct Launch {  // one stage handed to a stream by dispatch()
  int task, stage, part, stream;
  uint32_t job;
};

struct TaskStats {
  int64_t released = 0, accepted = 0, completed = 0, missed = 0, rej_adm = 0, rej_over = 0;
  int64_t resp_min = 0, resp_max = 0, resp_sum = 0, first_release = -1, last_finish = -1;
};

class SchedCore {
 public:
  int add_partition(int n_streams);
  void set_streams(int part, int n_streams);
  int add_task(int64_t period, int64_t deadline, int prio, int n_stages);
  void set_stage_count(int task, int n_stages);  // resets AFET / history of the task
  void set_afet(int task, int stage, int64_t ns);
  void set_window(int ws) { ws_ = ws; }
  void set_flags(int f) { flags_ = f; }

  void commit();  // Algorithm 1
  bool committed() const { return committed_; }

  // Input events.  `t` must not decrease between calls.
  // `t` is the instant the release is processed, `r` (<= t) the nominal release the deadlines count from.
  Decision release(int64_t t, int task, int64_t r, uint32_t* job_out);
  void migrate_command(int64_t t, int task, int target);
  // Completion of the running stage of `task`; returns true when this ended the job.
  bool stage_done(int64_t t, int task);
  // Dispatch pass: every idle stream takes the best ready stage of its partition.  `t` stamps the records.
  void dispatch(int64_t t, std::vector<Launch>* out);

  int n_parts() const { return (int)parts_.size(); }
  int n_tasks() const { return (int)tasks_.size(); }
  int n_streams(int part) const { return parts_[part].n_streams; }
  int context(int task) const { return tasks_[task].ctx; }
  int64_t period(int task) const { return tasks_[task].period; }
  int n_stages(int task) const { return (int)tasks_[task].afet.size(); }
  bool has_active(int task) const { return tasks_[task].active; }
  int64_t active_release(int task) const { return tasks_[task].job.release; }
  uint32_t active_job(int task) const { return tasks_[task].job.index; }
  int64_t mret_stage(int task, int stage) const;
  int64_t mret_task(int task) const;
  bool idle() const;  // no active and no queued job anywhere
  const TaskStats& stats(int task) const { return tasks_[task].st; }
  std::vector<TraceRec>& trace() { return trace_; }  // records not yet consumed by the reader; `seq` keeps counting
  uint64_t dropped() const { return dropped_; }       // records discarded because nobody read the trace

 private:
  struct Job {
    uint32_t index = 0;
    int64_t release = 0;
    std::vector<int64_t> vd;  // absolute virtual deadline per stage
    int part = 0, stage = 0, stream = -1;
    bool prev_missed = false, running = false, ready = false;
    unsigned __int128 u = 0;  // utilisation booked in U^{l,a} of `part`
    int64_t t_dispatch = 0;
  };
  struct Task {
    int64_t period, deadline;
    int prio;
    std::vector<int64_t> afet;
    std::vector<std::deque<int64_t>> ring;  // last ws execution times per stage
    int ctx = 0, pending = -1;
    bool active = false;
    Job job;
    std::deque<std::pair<uint32_t, int64_t>> fifo;  // queued HP releases (job index, release time)
    uint32_t n_released = 0;
    TaskStats st;
  };
  struct Part {
    int n_streams = 1;
    std::vector<int> running;  // per stream: task id or -1
    std::vector<int> ready;    // task ids whose active job waits here
    unsigned __int128 ula = 0; // U^{l,a}_k
  };

  void rec(int64_t t, uint8_t type, int level, int stage, int part, int task, int stream, uint32_t job, uint32_t aux);
  unsigned __int128 u_task(int task) const;
  unsigned __int128 u_high_total(int part) const;
  bool admission_ok(int part, unsigned __int128 u) const;
  int64_t backlog(int part) const;
  int level_of(const Task& tk) const;
  Decision start_job(int64_t t, int task, uint32_t m, int64_t r, bool queued);
  void apply_migration(int64_t t, int task, int target);

  std::vector<Part> parts_;
  std::vector<Task> tasks_;
  std::vector<TraceRec> trace_;
  uint64_t seq_ = 0, dropped_ = 0;
  int ws_ = 5, flags_ = 0;
  bool committed_ = false;
};

// Smallest even integer >= num/den (Sec. III-C2).
int64_t ceil_even(int64_t num, int64_t den);

}  // namespace daris
