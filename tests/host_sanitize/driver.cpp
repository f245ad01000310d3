// Drives the library's host logic through its C ABI from a plain text script, so that it can run as an executable
// built with AddressSanitizer and UndefinedBehaviorSanitizer (DARIS_NO_DEVICE | DARIS_VIRTUAL_TIME: no GPU call is made).
// The script and the expected results come from the Python test next to this file; see its docstring for the format.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <sstream>
#include <string>
#include <vector>

#include "../../include/daris.h"
#include "../../include/daris_debug.h"

static void die(const char* what) {
  std::fprintf(stderr, "driver: %s: %s\n", what, daris_last_error());
  std::exit(2);
}

int main(int argc, char** argv) {
  if (argc != 2) return 64;
  FILE* f = std::fopen(argv[1], "r");
  if (!f) return 65;
  char* line = nullptr;
  size_t cap = 0;
  std::vector<daris_layer> layers;
  while (getline(&line, &cap, f) > 0) {
    std::istringstream in(line);
    std::string cmd;
    if (!(in >> cmd) || cmd[0] == '#') continue;
    if (cmd == "init") {
      int flags;
      in >> flags;
      if (daris_init(0, 7, flags) != DARIS_OK) die("init");
    } else if (cmd == "partition") {
      int n_cu, ns;
      in >> n_cu >> ns;
      const daris_part p = daris_create_partition(n_cu);
      if (p < 0) die("partition");
      if (ns != 1 && daris_partition_set_streams(p, ns) != DARIS_OK) die("streams");
    } else if (cmd == "layer") {
      daris_layer L;
      std::memset(&L, 0, sizeof L);
      in >> L.op >> L.c_in >> L.c_out >> L.k >> L.stride >> L.pad >> L.groups >> L.act >> L.in_from >> L.res_from;
      layers.push_back(L);
    } else if (cmd == "task") {  // task period deadline prio dtype c h w k afet_0 .. afet_{k-1}   (uses the layers given so far)
      int64_t period, deadline;
      int prio, dtype, c, h, w, k;
      in >> period >> deadline >> prio >> dtype >> c >> h >> w >> k;
      daris_dnn d;
      d.n_layers = (int32_t)layers.size();
      d.in_c = c; d.in_h = h; d.in_w = w; d.dtype = dtype;
      d.layers = layers.data();
      const daris_task t = daris_register_task(&d, period, deadline, prio);
      if (t < 0) die("register");
      if (daris_split_stages(t, k) != DARIS_OK) die("split");
      for (int j = 0; j < k; ++j) {
        int64_t a;
        if (in >> a && a > 0 && daris_set_afet(t, j, a) != DARIS_OK) die("afet");
      }
      std::vector<int32_t> cuts(k);
      const int n = daris_get_stage_cuts(t, cuts.data(), k);
      std::printf("cuts %d", t);
      for (int j = 0; j < n; ++j) std::printf(" %d", cuts[j]);
      std::printf("\n");
      for (int l = 0; l < d.n_layers; ++l) {
        int64_t pl[27];
        if (daris_get_launch_plan(t, l, pl, 27) != 27) die("plan");
        std::printf("plan %d %d", t, l);
        for (int i = 0; i < 27; ++i) std::printf(" %" PRId64, pl[i]);
        std::printf("\n");
      }
      layers.clear();
    } else if (cmd == "et") {  // et task stage partition n v...
      int t, s, p, n;
      in >> t >> s >> p >> n;
      std::vector<int64_t> v(n);
      for (int i = 0; i < n; ++i) in >> v[i];
      if (daris_set_virtual_time(t, s, p, 0, n, v.data()) != DARIS_OK) die("et");
    } else if (cmd == "release") {
      int64_t t;
      int task;
      in >> t >> task;
      int32_t dec = 0;
      if (daris_release_job(task, nullptr, nullptr, t, &dec) != DARIS_OK) die("release");
      std::printf("decision %d %d\n", task, dec);
    } else if (cmd == "migrate") {
      int task, p;
      in >> task >> p;
      if (daris_migrate(task, p) != DARIS_OK) die("migrate");
    } else if (cmd == "run") {
      if (daris_run_until_idle() != DARIS_OK) die("run");
      std::vector<daris_trace_rec> buf(1 << 14);
      for (;;) {
        const int64_t got = daris_trace_read(buf.data(), (int64_t)(buf.size() * sizeof(daris_trace_rec)));
        if (got < 0) die("trace");
        if (got == 0) break;
        for (int64_t i = 0; i < got / (int64_t)sizeof(daris_trace_rec); ++i) {
          const daris_trace_rec& r = buf[i];
          std::printf("rec %" PRIu64 " %" PRId64 " %u %u %u %u %u %u %u %u\n", r.seq, r.t_ns, r.type, r.level, r.stage, r.partition, r.task, r.stream, r.job, r.aux);
        }
      }
    } else if (cmd == "stats") {
      int t;
      in >> t;
      daris_task_stats s;
      if (daris_get_stats(t, &s) != DARIS_OK) die("stats");
      std::printf("stats %d %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %d\n", t, s.released, s.accepted, s.completed, s.missed,
                  s.rejected_admission, s.rejected_overrun, s.partition);
    } else if (cmd == "shutdown") {
      if (daris_shutdown() != DARIS_OK) die("shutdown");
    } else {
      std::fprintf(stderr, "driver: unknown command %s\n", cmd.c_str());
      return 66;
    }
  }
  std::free(line);
  std::fclose(f);
  return 0;
}
