// C ABI of the library: global state, partitions as CU-masked hardware queues, task registration, and the two
// drivers around the decision core -- a virtual-time event loop and the real-time driver (API thread + one worker
// thread per stream) in which a stage boundary is a completion signal observed by the host (Sec. III-B1).
//
// HIP serves for device memory and copies only.  Kernels are dispatched as AQL packets on the library's own queues
// (aql.h); every layer's argument block is encoded when the task is registered and lives in device memory.
#include <dlfcn.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <queue>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include "../../include/daris.h"
#include "../../include/daris_debug.h"
#include "aql.h"
#include "kernels.h"
#include "net_plan.h"
#include "sched_core.h"
#include "static_scratch.h"

using namespace daris;

// the device code object (every kernel, built from kernels.hip), linked into the library as data
extern "C" const char daris_kernels_co[];
extern "C" const char daris_kernels_co_end[];

namespace {

thread_local std::string tl_error;

daris_status fail(daris_status code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  tl_error = buf;
  return code;
}

#define HIP_TRY(expr)                                                                                       \
  do {                                                                                                      \
    hipError_t e_ = (expr);                                                                                 \
    if (e_ != hipSuccess) return fail(DARIS_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

struct JobIo {
  const void* in = nullptr;
  void* out = nullptr;
  // device-resident argument blocks of the two launches that touch these buffers, prepared ahead (I/O pools); nullptr:
  // the block is patched at launch time and travels through the queue's host-coherent ring
  const void* in_args = nullptr;
  const void* out_args = nullptr;
};

struct LaunchRt {
  KernelLaunch kl;
  const void* dev = nullptr;  // the launch's argument block inside the task's device buffer
  double flops = 0;           // arithmetic of the layer(s) a dense-convolution launch computes, else 0
};

// Argument blocks of the input-reading and the logits-writing launch, one per buffer of a set of I/O buffers.
struct IoVariants {
  char* dev = nullptr;
  std::vector<const void*> in, out;
};

struct TaskRt {
  NetPlan net;
  std::vector<void*> slots;
  float* ws = nullptr;
  int prio = 0;  // DARIS_HP / DARIS_LP
  std::vector<void*> owned;  // every device allocation of the task
  // I/O
  const void* pool_in = nullptr;
  void* pool_out = nullptr;
  int32_t n_inputs = 0, n_slots = 0;
  std::unordered_map<uint32_t, JobIo> io;  // per released job
  // the whole network as launches in execution order, encoded at registration; layer l issues launches
  // [layer_lo[l], layer_lo[l + 1]) (none for the earlier member of a launch pair)
  std::vector<LaunchRt> launches;
  std::vector<int> layer_lo;
  int in_launch = -1, out_launch = -1;  // the launches that read the job's input / write its logits
  uint32_t in_off = 0, out_off = 0;     // byte offset of that pointer inside the argument block
  IoVariants pool;                      // argument blocks for the buffers of daris_task_set_io
  // the same network encoded on the static device scratch (daris_forward_static), built at its first call; host memory only
  std::vector<LaunchRt> static_launches;
  std::vector<int> static_layer_lo;
  int static_in = -1, static_out = -1;
  uint32_t static_in_off = 0, static_out_off = 0;
  // virtual execution times: (stage, partition) -> (job_lo, values)
  std::map<std::pair<int, int>, std::pair<int64_t, std::vector<int64_t>>> vt;
  // library-driven runs
  int32_t closed_left = 0;
};

struct StreamRt {  // one CU-masked queue and, in real-time mode, the worker thread that feeds and watches it
  struct HwQueue {
    AqlQueue q;
    std::mutex mu;  // one producer at a time (the streams' workers; direct calls of the API thread)
  };
  // the hardware queue the stream's packets go to: its own, or (DARIS_SHARED_QUEUE) one for all streams of the partition
  std::shared_ptr<HwQueue> hw;
  hsa_signal_t done{0};            // completion of the last launch of a stage
  hsa_signal_t begin{0};           // driver profile: completion of a stage's first launch (its start time stamp)
  std::vector<hsa_signal_t> tsig;  // kernel timing: one signal per launch of a sampled stage
  // what enqueue_stage left for finish_stage
  int pend_lo = 0, pend_hi = 0;
  bool pend_sample = false, pend_prof = false;
  std::thread thr;
  std::condition_variable cv;
  std::atomic<bool> has_work{false};  // a stage handed over by a dispatch pass, not yet picked up by the worker
  Launch work;
  JobIo work_io;
  bool work_sample = false;
  int64_t work_t = 0;  // host clock at the hand-over
};

struct PartRt {
  int n_cu = 0, start = 0, n_streams = 1;
  uint32_t mask[8] = {0};
  std::vector<std::shared_ptr<StreamRt>> streams;
};

struct VtEvent {
  int64_t t;
  int task;
  uint32_t job;
  bool operator>(const VtEvent& o) const {
    if (t != o.t) return t > o.t;
    if (task != o.task) return task > o.task;
    return job > o.job;
  }
};

struct Global {
  bool inited = false;
  int device = 0, flags = 0;
  uint64_t seed = 0;
  bool vt = false, nodev = false;
  SchedCore core;
  std::vector<PartRt> parts;
  std::vector<std::unique_ptr<TaskRt>> tasks;
  int cu_cursor = 0;
  int plan_cus = 128;      // partition size the launch plans of tasks registered from now on are balanced for
  bool committed = false;  // Algorithm 1 has run, the online phase has begun
  bool frozen = false;     // streams exist, the partition set can no longer change
  // virtual time
  int64_t vt_now = -1;
  bool vt_dirty = false;
  std::priority_queue<VtEvent, std::vector<VtEvent>, std::greater<VtEvent>> heap;
  // real time
  std::mutex mu;
  std::condition_variable cv_idle;
  bool stop = false;
  std::atomic<bool> stop_flag{false};  // mirrors `stop` for the workers' lock-free spin
  std::chrono::steady_clock::time_point epoch;
  std::string async_error;
  // A wait for the GPU ran into the limit, or a queue reported an error: what the GPU still does with the buffers is
  // unknown, so every later call but daris_shutdown (and the read-only accessors) is refused.
  std::atomic<bool> failed{false};
  std::string failed_why;
  int tm_every = 0;                 // kernel timing: sample every n-th job of a task, 0 = off
  int64_t tm_left = 0;              // samples still to take
  int64_t tm_launches[K_COUNT] = {0};
  double tm_ms[K_COUNT] = {0}, tm_flops[K_COUNT] = {0};
  hsa_signal_t util_sig{0};         // completion signal of the API thread's direct launches (under mu)
  int64_t closed_total_left = -1;  // closed-loop runs: releases left over all tasks, -1 = no common budget
  bool prof = false;                // driver profile: where a stage's wall time goes (host clock and GPU markers)
  int64_t prof_acc[8] = {0};
};

Global* G = nullptr;

int64_t now_ns() {
  return std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - G->epoch).count();
}

// ---- stage execution ----------------------------------------------------------------------------------------------

// The loaded code object and its kernels: set up by the first daris_init with a device and kept until the process ends.
AqlRuntime g_rt;
KernelTable g_kt;
int g_rt_device = -1;

ConvArgs conv_args(TaskRt& T, int l, void* y, const std::vector<void*>& slots, float* ws) {
  NetPlan& net = T.net;
  LayerPlan& L = net.layers[l];
  const TensorInfo& in = net.tensor(L.in_t);
  ConvArgs a;
  a.x = slots[in.slot]; a.w = L.w_dev; a.bias = L.b_dev; a.y = y; a.ws = ws; a.wave_prio = (T.prio == DARIS_HP && (G->flags & DARIS_WAVE_PRIORITY)) ? 1 : 0;
  a.res = L.res_t >= 0 ? slots[net.tensor(L.res_t).slot] : nullptr;
  a.H = in.H; a.W = in.W; a.Cin = in.Cs; a.Ho = L.out.H; a.Wo = L.out.W; a.Cout = L.out.Cs;
  a.kh = a.kw = L.d.k; a.stride = L.d.stride; a.pad = L.d.pad;
  a.K = L.K; a.Kpad = L.Kpad; a.M = L.out.H * L.out.W; a.act = L.d.act;
  a.splitk = L.cp.splitk; a.S = L.cp.S; a.sz = L.cp.sz; a.sw = L.cp.sw;
  a.MT = L.cp.MT; a.NTn = L.cp.NTn; a.G = L.cp.G; a.xmode = L.cp.xmode;
  a.mg_wo = div_magic((uint32_t)a.Wo); a.mg_cin = div_magic((uint32_t)a.Cin); a.mg_kw = div_magic((uint32_t)a.kw);
  a.c_real = 0;
  if (l == 0 && net.fuse_ingest) {  // layer 0 gathers from the job's fp32 [C][H][W] input: the pointer is filled in per job
    a.x = nullptr;
    a.c_real = net.in_c;
  }
  return a;
}

// Where the launch sequence of a network reads a job's input and writes its logits.
struct IoLaunches {
  int in_launch = -1, out_launch = -1;  // indices into the launch sequence
  uint32_t in_off = 0, out_off = 0;     // byte offset of that pointer inside the argument block
};

// Encodes the whole network of T as launches in execution order, with its activation tensors in `slots` (one device
// buffer per slot of the plan) and its split-K partial sums in `ws`; the weights must be on the device.  The two pointers
// that change from job to job (the input of the first launch, the logits of the last) stay null in the argument blocks.
// Returns "" or an error text.
std::string encode_network(TaskRt& T, const std::vector<void*>& slots, float* ws, std::vector<LaunchRt>* launches, std::vector<int>* layer_lo,
                           IoLaunches* iol) {
  NetPlan& net = T.net;
  const int n = (int)net.layers.size();
  const int bf16 = net.bf16;
  std::vector<KernelLaunch> ks;
  launches->clear();
  layer_lo->assign(n + 1, 0);
  *iol = IoLaunches();
  auto take = [&](double flops) {
    for (size_t i = 0; i < ks.size(); ++i) {
      LaunchRt r;
      r.kl = ks[i];
      r.flops = i == 0 ? flops : 0;
      launches->push_back(r);
    }
    ks.clear();
  };
  if (!net.fuse_ingest) {
    if (!encode_ingest(g_kt, nullptr, slots[net.ingest.slot], net.ingest.C, net.ingest.Cs, net.ingest.H, net.ingest.W, bf16, &ks))
      return "input conversion launch";
    iol->in_launch = 0;
    iol->in_off = kIngestInputOffset;
    take(0);
  }
  for (int l = 0; l < n; ++l) {
    (*layer_lo)[l] = (int)launches->size();
    LayerPlan& L = net.layers[l];
    const TensorInfo& in = net.tensor(L.in_t);
    const void* x = slots[in.slot];
    const bool direct = l == n - 1 && net.final_direct;  // writes the job's logits
    void* y = direct ? nullptr : slots[L.out.slot];
    bool ok = false;
    double flops = 0;
    switch (L.d.op) {
      case DARIS_OP_CONV:
        if (L.depthwise && L.fused_dw) {
          ok = true;  // computed inside the next layer's launch
        } else if (L.depthwise) {
          DwArgs a;
          a.x = x; a.w = L.w_dev; a.bias = L.b_dev; a.y = y;
          a.H = in.H; a.W = in.W; a.C = in.Cs; a.Ho = L.out.H; a.Wo = L.out.W;
          a.k = L.d.k; a.stride = L.d.stride; a.pad = L.d.pad; a.act = L.d.act;
          ok = encode_dwconv(g_kt, a, bf16, &ks);
        } else if (L.pair_with >= 0 && !L.pair_lead) {
          ok = true;  // issued together with the next layer
        } else {
          const ConvArgs a = conv_args(T, l, y, slots, ws);
          flops = 2.0 * (double)L.macs;
          if (L.fused_dw) {
            LayerPlan& O = net.layers[L.pair_with];  // the depthwise layer: this launch reads ITS input
            const TensorInfo& din = net.tensor(O.in_t);
            ConvArgs b = a;
            b.x = slots[din.slot];
            DwFusedArgs d;
            d.w = O.w_dev; d.bias = O.b_dev; d.H = din.H; d.W = din.W; d.stride = O.d.stride; d.act = O.d.act;
            flops += 2.0 * (double)O.macs;
            ok = encode_conv_dw(g_kt, L.cp, b, d, bf16, &ks);
          } else if (L.pair_with >= 0) {
            LayerPlan& O = net.layers[L.pair_with];
            const ConvArgs b = conv_args(T, L.pair_with, slots[O.out.slot], slots, ws);
            flops += 2.0 * (double)O.macs;
            // the heavier convolution is the first problem (its plan was kept)
            ok = L.macs >= O.macs ? encode_conv_pair(g_kt, L.cp, a, O.cp, b, bf16, &ks) : encode_conv_pair(g_kt, O.cp, b, L.cp, a, bf16, &ks);
          } else {
            if (l == 0 && net.fuse_ingest) {
              iol->in_launch = (int)launches->size();
              iol->in_off = kConvInputOffset;
            }
            ok = encode_conv(g_kt, L.cp, a, bf16, &ks);
          }
        }
        break;
      case DARIS_OP_MAXPOOL:
      case DARIS_OP_GAVGPOOL: {
        PoolArgs a;
        a.x = x; a.y = y; a.H = in.H; a.W = in.W; a.C = in.Cs; a.Ho = L.out.H; a.Wo = L.out.W;
        a.k = L.d.k; a.stride = L.d.stride; a.pad = L.d.pad;
        ok = L.d.op == DARIS_OP_MAXPOOL ? encode_maxpool(g_kt, a, bf16, &ks) : encode_gavgpool(g_kt, a, bf16, &ks);
        break;
      }
      case DARIS_OP_FC: {
        FcArgs a;
        a.x = x; a.w = L.w_dev; a.bias = L.b_dev; a.y = y;
        a.K = L.K; a.N = L.d.c_out; a.Ns = direct ? L.d.c_out : L.out.Cs;
        a.act = L.d.act; a.out_f32 = direct ? 1 : 0;
        if (direct) {
          iol->out_launch = (int)launches->size();
          iol->out_off = kFcOutputOffset;
        }
        ok = encode_fc(g_kt, a, bf16, &ks);
        break;
      }
    }
    if (!ok) return "launch of layer " + std::to_string(l) + " (" + kernel_name(L.kernel_id) + ")";
    take(flops);
  }
  (*layer_lo)[n] = (int)launches->size();
  if (!net.final_direct) {
    const TensorInfo& o = net.layers[n - 1].out;
    if (!encode_egress(g_kt, slots[o.slot], nullptr, o.C, o.Cs, o.H, o.W, bf16, &ks)) return "output conversion launch";
    iol->out_launch = (int)launches->size();
    iol->out_off = kEgressOutputOffset;
    take(0);
  }
  return "";
}

// Encodes T's network on its own buffers and uploads the argument blocks into one device buffer; a job brings its own
// copies of the two job-dependent blocks (JobIo).  Returns "" or an error text.
std::string build_launches(TaskRt& T) {
  IoLaunches iol;
  std::string err = encode_network(T, T.slots, T.ws, &T.launches, &T.layer_lo, &iol);
  if (!err.empty()) return err;
  T.in_launch = iol.in_launch;
  T.out_launch = iol.out_launch;
  T.in_off = iol.in_off;
  T.out_off = iol.out_off;
  // one device buffer for all argument blocks, 64 bytes apart at least
  std::vector<unsigned char> img;
  std::vector<size_t> off;
  for (LaunchRt& r : T.launches) {
    off.push_back(img.size());
    img.insert(img.end(), r.kl.args, r.kl.args + r.kl.nbytes);
    img.resize((img.size() + 63) / 64 * 64, 0);
  }
  void* dev = nullptr;
  hipError_t e = hipMalloc(&dev, img.size());
  if (e != hipSuccess) return std::string("argument buffer: ") + hipGetErrorString(e);
  T.owned.push_back(dev);
  e = hipMemcpy(dev, img.data(), img.size(), hipMemcpyHostToDevice);
  if (e != hipSuccess) return std::string("argument upload: ") + hipGetErrorString(e);
  for (size_t i = 0; i < T.launches.size(); ++i) T.launches[i].dev = (const char*)dev + off[i];
  return "";
}

void free_variants(IoVariants* v) {
  if (v->dev) (void)hipFree(v->dev);
  v->dev = nullptr;
  v->in.clear();
  v->out.clear();
}

// Argument blocks of T's input-reading launch for n_in input buffers (in_stride bytes apart) and of its logits-writing
// launch for n_out output buffers.  Leaves v empty when one launch does both (then jobs patch at launch time).
hipError_t build_variants(TaskRt& T, const void* in_base, int n_in, size_t in_stride, void* out_base, int n_out, size_t out_stride,
                          IoVariants* v) {
  free_variants(v);
  if (T.in_launch < 0 || T.out_launch < 0 || T.in_launch == T.out_launch) return hipSuccess;
  const KernelLaunch& ki = T.launches[T.in_launch].kl;
  const KernelLaunch& ko = T.launches[T.out_launch].kl;
  const size_t bi = (ki.nbytes + 63) / 64 * 64, bo = (ko.nbytes + 63) / 64 * 64;
  std::vector<unsigned char> img((size_t)n_in * bi + (size_t)n_out * bo, 0);
  for (int i = 0; i < n_in; ++i) {
    unsigned char* blk = img.data() + (size_t)i * bi;
    std::memcpy(blk, ki.args, ki.nbytes);
    const void* ptr = (const char*)in_base + (size_t)i * in_stride;
    std::memcpy(blk + T.in_off, &ptr, sizeof(ptr));
  }
  for (int i = 0; i < n_out; ++i) {
    unsigned char* blk = img.data() + (size_t)n_in * bi + (size_t)i * bo;
    std::memcpy(blk, ko.args, ko.nbytes);
    void* ptr = (char*)out_base + (size_t)i * out_stride;
    std::memcpy(blk + T.out_off, &ptr, sizeof(ptr));
  }
  hipError_t e = hipMalloc((void**)&v->dev, img.size());
  if (e != hipSuccess) {
    v->dev = nullptr;
    return e;
  }
  e = hipMemcpy(v->dev, img.data(), img.size(), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    free_variants(v);
    return e;
  }
  for (int i = 0; i < n_in; ++i) v->in.push_back(v->dev + (size_t)i * bi);
  for (int i = 0; i < n_out; ++i) v->out.push_back(v->dev + (size_t)n_in * bi + (size_t)i * bo);
  return hipSuccess;
}

struct EnqueueOpts {
  hsa_signal_t done{0};   // completes with the last launch
  hsa_signal_t first{0};  // completes with the first launch (ignored when that launch carries `done`, or when sampling)
  bool release_system = false;  // the last launch makes its writes visible to the host and to other processes' copies
  bool acquire_system = false;  // the first launch sees what copies and other queues of the system wrote before
  bool sample = false;          // every launch completes a signal of S.tsig, so that its time stamps can be read
};

// Appends launches [lo, hi) of T to S's queue (S.hw->mu held).  Returns nullptr or an error text.
const char* enqueue_range(TaskRt& T, int lo, int hi, const JobIo& io, StreamRt& S, const EnqueueOpts& o) {
  if (lo < 0 || hi > (int)T.launches.size() || lo >= hi) return "empty launch range";
  if (o.sample) {
    while ((int)S.tsig.size() < hi - lo - 1) {
      hsa_signal_t sg = g_rt.new_signal(1);
      if (!sg.handle) return "signal creation failed";
      S.tsig.push_back(sg);
    }
  }
  for (int i = lo; i < hi; ++i) {
    const LaunchRt& r = T.launches[i];
    hsa_signal_t sig{0};
    if (i == hi - 1 && o.done.handle) sig = o.done;
    else if (o.sample && i < hi - 1) sig = S.tsig[i - lo];
    else if (i == lo) sig = o.first;
    const unsigned fl = ((i == hi - 1 && o.release_system) ? AqlQueue::kReleaseSystem : 0u) | ((i == lo && o.acquire_system) ? AqlQueue::kAcquireSystem : 0u);
    const void* dev = r.dev;
    const bool is_in = i == T.in_launch, is_out = i == T.out_launch;
    if (is_in || is_out) {
      if (is_in && !is_out && io.in_args) dev = io.in_args;
      else if (is_out && !is_in && io.out_args) dev = io.out_args;
      else {
        if ((is_in && !io.in) || (is_out && !io.out)) return "job without I/O buffers";
        alignas(8) unsigned char blk[sizeof(KernelLaunch::args)];
        std::memcpy(blk, r.kl.args, r.kl.nbytes);
        if (is_in) std::memcpy(blk + T.in_off, &io.in, sizeof(void*));
        if (is_out) std::memcpy(blk + T.out_off, &io.out, sizeof(void*));
        if (!S.hw->q.dispatch_copy(*r.kl.k, r.kl.groups, r.kl.threads, blk, r.kl.nbytes, sig, fl)) return "packet rejected";
        continue;
      }
    }
    if (!S.hw->q.dispatch(*r.kl.k, r.kl.groups, r.kl.threads, dev, sig, fl)) return "packet rejected";
  }
  return nullptr;
}

void stage_range(const TaskRt& T, int stage, int* lo, int* hi) {
  const NetPlan& net = T.net;
  const int n = (int)net.layers.size();
  const int first = net.stage_first[stage];
  const int end = stage + 1 < (int)net.stage_first.size() ? net.stage_first[stage + 1] : n;
  *lo = stage == 0 ? 0 : T.layer_lo[first];
  *hi = end == n ? (int)T.launches.size() : T.layer_lo[end];
}

// Enqueues one stage of a job on S (S.hw->mu held); S.done completes with it.  Inside a job the next stage runs on this
// device whichever queue it gets, so its boundary releases at device scope; the last stage's boundary makes the logits
// visible to the host.
const char* enqueue_stage(TaskRt& T, int stage, const JobIo& io, StreamRt& S, bool sample, bool prof) {
  int lo, hi;
  stage_range(T, stage, &lo, &hi);
  EnqueueOpts o;
  o.done = S.done;
  o.first = prof ? S.begin : hsa_signal_t{0};
  o.release_system = stage + 1 == (int)T.net.stage_first.size();
  o.acquire_system = stage == 0;
  o.sample = sample;
  S.pend_lo = lo;
  S.pend_hi = hi;
  S.pend_sample = sample;
  S.pend_prof = prof;
  return enqueue_range(T, lo, hi, io, S, o);
}

// After S.done was seen complete: reads the time stamps the stage asked for (kernel timing into the global sums; the
// span from the first kernel's start to the last kernel's end is returned in nanoseconds, 0 if not profiled) and
// re-arms the signals.  The global sums need G->mu in real-time mode.
int64_t finish_stage(TaskRt& T, StreamRt& S) {
  const int lo = S.pend_lo, hi = S.pend_hi;
  int64_t span_ns = 0;
  double t_first = 0, t_last_end = 0, a = 0, b = 0;
  if (S.pend_sample) {
    for (int i = lo; i < hi; ++i) {
      const hsa_signal_t sg = i == hi - 1 ? S.done : S.tsig[i - lo];
      if (!g_rt.dispatch_time_us(sg, &a, &b)) continue;
      const LaunchRt& r = T.launches[i];
      const int k = r.kl.kernel_id;
      if (k > K_NONE && k < K_COUNT) {
        G->tm_launches[k]++;
        G->tm_ms[k] += (b - a) * 1e-3;
        G->tm_flops[k] += r.flops;
      }
      if (i == lo) t_first = a;
      if (i == hi - 1) t_last_end = b;
      if (i < hi - 1) hsa_signal_store_relaxed(sg, 1);
    }
    span_ns = (int64_t)((t_last_end - t_first) * 1e3);
  } else if (S.pend_prof) {
    if (g_rt.dispatch_time_us(S.done, &a, &b)) {
      t_first = a;
      t_last_end = b;
      if (hi - lo > 1) {
        double a0 = 0, b0 = 0;
        if (g_rt.dispatch_time_us(S.begin, &a0, &b0)) t_first = a0;
      }
      span_ns = (int64_t)((t_last_end - t_first) * 1e3);
    }
    if (hi - lo > 1) hsa_signal_store_relaxed(S.begin, 1);
  }
  hsa_signal_store_relaxed(S.done, 1);
  return span_ns;
}

// Marks the library failed (under G->mu or from the API thread) and returns the status for the caller.
daris_status gpu_wait_failed(const StreamRt& S, const char* what) {
  const bool dead = S.hw && S.hw->q.dead();
  char buf[256];
  snprintf(buf, sizeof buf, "%s: %s; the library accepts no further work (daris_shutdown only)", what,
           dead ? "the queue reported an error" : "the GPU did not complete it within the wait limit (daris_set_timeout)");
  if (!G->failed.exchange(true)) G->failed_why = buf;
  return fail(DARIS_EHIP, "%s", buf);
}

// API thread, G->mu held: runs launches [lo, hi) of T on S and waits for them.
daris_status run_direct(TaskRt& T, int lo, int hi, const JobIo& io, StreamRt& S) {
  EnqueueOpts o;
  o.done = G->util_sig;
  o.release_system = o.acquire_system = true;
  const char* err;
  {
    std::lock_guard<std::mutex> ql(S.hw->mu);
    err = enqueue_range(T, lo, hi, io, S, o);
  }
  if (err) return fail(DARIS_EHIP, "%s", err);
  if (!aql_wait(G->util_sig, &S.hw->q)) return gpu_wait_failed(S, "direct execution");
  return DARIS_OK;
}

// API thread, G->mu held: one launch with arguments built just now.
daris_status run_one(const std::vector<KernelLaunch>& ks, StreamRt& S) {
  for (size_t i = 0; i < ks.size(); ++i) {
    bool ok;
    {
      std::lock_guard<std::mutex> ql(S.hw->mu);
      ok = S.hw->q.dispatch_copy(*ks[i].k, ks[i].groups, ks[i].threads, ks[i].args, ks[i].nbytes, G->util_sig, AqlQueue::kReleaseSystem | AqlQueue::kAcquireSystem);
    }
    if (!ok) return fail(DARIS_EHIP, "packet rejected");
    if (!aql_wait(G->util_sig, &S.hw->q)) return gpu_wait_failed(S, "direct launch");
  }
  return DARIS_OK;
}

// Acts on the launches a dispatch pass produced.  Virtual time: schedule the completion from the table and (with a
// device) run the kernels now, waiting for them, so that a task's stages execute in order whichever queues they get.
// Real time: hand the stage to the worker of its stream.
daris_status issue(const std::vector<Launch>& ls, int64_t t) {
  for (const Launch& l : ls) {
    TaskRt& T = *G->tasks[l.task];
    if (G->vt) {
      auto it = T.vt.find(std::make_pair(l.stage, l.part));
      if (it == T.vt.end()) return fail(DARIS_ESTATE, "no virtual execution time for task %d stage %d partition %d", l.task, l.stage, l.part);
      const int64_t idx = (int64_t)l.job - it->second.first;
      if (idx < 0 || idx >= (int64_t)it->second.second.size())
        return fail(DARIS_ESTATE, "virtual execution time table of task %d stage %d partition %d has no job %u", l.task, l.stage, l.part, l.job);
      G->heap.push(VtEvent{t + it->second.second[idx], l.task, l.job});
    }
    if (!G->nodev) {
      StreamRt& S = *G->parts[l.part].streams[l.stream];
      auto io = T.io.find(l.job);
      if (io == T.io.end()) return fail(DARIS_ESTATE, "job %u of task %d has no I/O buffers", l.job, l.task);
      bool sample = G->tm_every > 0 && l.job % (uint32_t)G->tm_every == 0 && G->tm_left > 0;
      if (sample) {
        int lo, hi;
        stage_range(T, l.stage, &lo, &hi);
        G->tm_left -= hi - lo;
      }
      if (G->vt) {
        const char* err;
        {
          std::lock_guard<std::mutex> ql(S.hw->mu);
          err = enqueue_stage(T, l.stage, io->second, S, sample, false);
        }
        if (err) return fail(DARIS_EHIP, "stage execution: %s", err);
        if (!aql_spin(S.done, &S.hw->q)) return gpu_wait_failed(S, "stage execution");
        finish_stage(T, S);
      } else {
        // real time: the stream's own worker enqueues the kernels and watches the boundary signal
        S.work = l;
        S.work_io = io->second;
        S.work_sample = sample;
        S.work_t = G->prof ? now_ns() : 0;
        S.has_work = true;
        S.cv.notify_one();
      }
    }
  }
  return DARIS_OK;
}

daris_status dispatch_and_issue(int64_t t) {
  std::vector<Launch> ls;
  G->core.dispatch(t, &ls);
  return issue(ls, t);
}

// ---- virtual-time driver -------------------------------------------------------------------------------------------

// Process every completion due at exactly G->vt_now (ordered by task, job).
void vt_completions_now() {
  while (!G->heap.empty() && G->heap.top().t == G->vt_now) {
    VtEvent ev = G->heap.top();
    G->heap.pop();
    if (G->core.stage_done(ev.t, ev.task)) G->tasks[ev.task]->io.erase(ev.job);
    G->vt_dirty = true;
  }
}

// Advance the virtual clock up to `limit` (exclusive): dispatch what is pending, then event by event.
daris_status vt_advance(int64_t limit, bool unbounded) {
  for (;;) {
    if (G->vt_dirty) {
      G->vt_dirty = false;
      daris_status st = dispatch_and_issue(G->vt_now);
      if (st != DARIS_OK) return st;
    }
    if (G->heap.empty()) return DARIS_OK;
    const int64_t t = G->heap.top().t;
    if (!unbounded && t >= limit) return DARIS_OK;
    G->vt_now = t;
    vt_completions_now();
  }
}

// ---- real-time driver ----------------------------------------------------------------------------------------------

daris_status rt_release_locked(int task, const JobIo& io, int64_t now, int64_t r, int32_t* decision) {
  uint32_t job = 0;
  Decision d = G->core.release(now, task, r, &job);
  if (decision) *decision = (int32_t)d;
  if (d == D_ACCEPTED || d == D_MIGRATED || d == D_QUEUED) G->tasks[task]->io[job] = io;
  return dispatch_and_issue(now);
}

JobIo pool_io(TaskRt& T, uint32_t job) {
  JobIo io;
  const NetPlan& n = T.net;
  const size_t in_elems = (size_t)n.in_c * n.in_h * n.in_w;
  const uint32_t i = job % (uint32_t)T.n_inputs, j = job % (uint32_t)T.n_slots;
  io.in = (const float*)T.pool_in + (size_t)i * in_elems;
  io.out = (float*)T.pool_out + (size_t)j * n.n_out;
  if (i < T.pool.in.size()) io.in_args = T.pool.in[i];
  if (j < T.pool.out.size()) io.out_args = T.pool.out[j];
  return io;
}

// Worker of one stream (real-time mode).  It enqueues the kernels of the stage a dispatch pass gave to its stream,
// spins on the completion signal of the last one, and then -- under the scheduler lock -- feeds the completion into the
// decision core and runs the dispatch pass that follows every input event.  The enqueue and the wait happen
// outside the lock, so the partitions' launch paths do not serialise.
void worker_loop(StreamRt* S) {
  std::unique_lock<std::mutex> lk(G->mu);
  for (;;) {
    if (!G->stop && !S->has_work) {
      // A stage usually follows within microseconds (another stream's boundary hands it over): spin for a while
      // outside the lock before sleeping, a wake-up through the condition variable costs ~10 us.
      lk.unlock();
      for (int i = 0; i < 20000 && !S->has_work.load(std::memory_order_acquire) && !G->stop_flag.load(std::memory_order_relaxed); ++i)
        __builtin_ia32_pause();
      lk.lock();
    }
    S->cv.wait(lk, [&] { return G->stop || S->has_work; });
    if (G->stop) return;
    const Launch l = S->work;
    const JobIo io = S->work_io;
    const bool sample = S->work_sample;
    S->has_work = false;
    TaskRt& T = *G->tasks[l.task];
    const bool prof = G->prof;
    const int64_t t_handed = S->work_t;
    lk.unlock();
    const int64_t t0 = prof ? now_ns() : 0;
    const char* err;
    {
      std::lock_guard<std::mutex> ql(S->hw->mu);
      err = enqueue_stage(T, l.stage, io, *S, sample, prof);
    }
    const int64_t t1 = prof ? now_ns() : 0;
    const bool completed = !err && aql_spin(S->done, &S->hw->q, &G->stop_flag);
    const int64_t t2 = prof ? now_ns() : 0;
    lk.lock();
    if (G->stop) return;
    int64_t gpu_ns = 0;
    if (err || !completed) {
      // The stage did not run to its boundary: the decision core keeps it as running, nothing more is dispatched, and
      // whoever waits for idleness gets the error.  This worker ends here.
      if (err) {
        if (G->async_error.empty()) G->async_error = std::string("stage execution: ") + err;
        if (!G->failed.exchange(true)) G->failed_why = G->async_error;
      } else {
        gpu_wait_failed(*S, "stage execution");
        if (G->async_error.empty()) G->async_error = G->failed_why;
      }
      G->cv_idle.notify_all();
      return;
    }
    gpu_ns = finish_stage(T, *S);
    const int64_t now = now_ns();
    if (prof) {
      G->prof_acc[0] += 1;
      G->prof_acc[1] += t1 - t0;
      G->prof_acc[2] += t2 - t1;
      G->prof_acc[3] += now - t2;
      G->prof_acc[5] += gpu_ns;
      G->prof_acc[6] += t0 - t_handed;
    }
    const int task = l.task;
    const uint32_t job = G->core.active_job(task);
    const bool job_done = G->core.stage_done(now, task);
    if (job_done) T.io.erase(job);
    // a dispatch pass follows every input event (completion, release, migration command)
    if (dispatch_and_issue(now) != DARIS_OK && G->async_error.empty()) G->async_error = tl_error;
    if (job_done) {
      // closed loop: the next job of the task is released the instant this one ends
      while (T.closed_left > 0 && G->closed_total_left != 0 && !G->core.has_active(task)) {
        T.closed_left--;
        if (G->closed_total_left > 0) G->closed_total_left--;
        const uint32_t next = (uint32_t)G->core.stats(task).released;
        int32_t dec = 0;
        if (rt_release_locked(task, pool_io(T, next), now, now, &dec) != DARIS_OK && G->async_error.empty())
          G->async_error = tl_error;
      }
    }
    if (prof) G->prof_acc[4] += now_ns() - now;
    if (G->core.idle()) G->cv_idle.notify_all();
  }
}

daris_status check_failed() {
  if (G && G->failed.load()) return fail(DARIS_EHIP, "%s", G->failed_why.c_str());
  return DARIS_OK;
}

// `observe`: a read-only accessor, allowed in the failed state too
daris_status check_task(daris_task t, bool observe = false) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (!observe && check_failed() != DARIS_OK) return DARIS_EHIP;
  if (t < 0 || t >= (int)G->tasks.size()) return fail(DARIS_ERANGE, "task handle %d out of range", t);
  return DARIS_OK;
}
daris_status check_part(daris_part p, bool observe = false) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (!observe && check_failed() != DARIS_OK) return DARIS_EHIP;
  if (p < 0 || p >= (int)G->parts.size()) return fail(DARIS_ERANGE, "partition handle %d out of range", p);
  return DARIS_OK;
}

daris_status wait_idle() {
  std::unique_lock<std::mutex> lk(G->mu);
  while (!G->core.idle()) {
    if (!G->async_error.empty() || G->failed.load()) break;
    G->cv_idle.wait_for(lk, std::chrono::milliseconds(1));
  }
  if (G->failed.load() && G->async_error.empty()) G->async_error = G->failed_why;
  if (!G->async_error.empty()) {
    daris_status st = fail(DARIS_EHIP, "%s", G->async_error.c_str());
    G->async_error.clear();
    return st;
  }
  return DARIS_OK;
}

void free_task(TaskRt& T) {
  for (void* p : T.owned) (void)hipFree(p);
  T.owned.clear();
  free_variants(&T.pool);
}

}  // namespace

extern "C" {

const char* daris_last_error(void) { return tl_error.c_str(); }

int32_t daris_cu_per_partition(int32_t os_num, int32_t os_den, int32_t n_cu_max, int32_t n_c) {
  if (os_num < 1 || os_den < 1 || n_cu_max < 1 || n_c < 1) return fail(DARIS_EINVAL, "arguments must be positive");
  return (int32_t)ceil_even((int64_t)os_num * n_cu_max, (int64_t)os_den * n_c);
}

daris_status daris_init(int device, uint64_t seed, int flags) {
  if (G && G->inited) return fail(DARIS_ESTATE, "already initialised");
  if ((flags & DARIS_NO_DEVICE) && !(flags & DARIS_VIRTUAL_TIME)) return fail(DARIS_EINVAL, "DARIS_NO_DEVICE needs DARIS_VIRTUAL_TIME");
  delete G;
  G = new Global();
  G->device = device;
  G->seed = seed;
  G->flags = flags;
  G->vt = flags & DARIS_VIRTUAL_TIME;
  G->nodev = flags & DARIS_NO_DEVICE;
  int cf = 0;
  if (flags & DARIS_NO_LAST) cf |= CF_NO_LAST;
  if (flags & DARIS_NO_PRIOR) cf |= CF_NO_PRIOR;
  if (flags & DARIS_NO_FIXED) cf |= CF_NO_FIXED;
  if (flags & DARIS_HP_ADMISSION) cf |= CF_HP_ADMISSION;
  G->core.set_flags(cf);
  if (!G->nodev) {
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || device < 0 || device >= n) {
      delete G;
      G = nullptr;
      return fail(DARIS_EHIP, "no usable HIP device %d (%s)", device, e == hipSuccess ? "index out of range" : hipGetErrorString(e));
    }
    e = hipSetDevice(device);
    if (e == hipSuccess) e = hipFree(nullptr);  // HIP's context (and with it the HSA runtime) exists from here on
    if (e != hipSuccess) {
      delete G;
      G = nullptr;
      return fail(DARIS_EHIP, "hipSetDevice failed: %s", hipGetErrorString(e));
    }
    std::string err;
    if (!g_rt.ready()) {
      err = g_rt.init(device, daris_kernels_co, (size_t)(daris_kernels_co_end - daris_kernels_co));
      if (err.empty()) {
        err = g_kt.resolve(g_rt);
        if (!err.empty()) err = "kernel " + err;
      }
      if (err.empty()) g_rt_device = device;
    } else if (device != g_rt_device) {
      err = "the kernels are loaded on device " + std::to_string(g_rt_device) + "; one device per process";
    }
    if (err.empty()) err = static_scratch_init(device);  // this GPU's copy of the static scratch array (device is current)
    if (err.empty()) {
      G->util_sig = g_rt.new_signal(1);
      if (!G->util_sig.handle) err = "signal creation failed";
    }
    if (!err.empty()) {
      delete G;
      G = nullptr;
      return fail(DARIS_EHIP, "%s", err.c_str());
    }
  }
  G->inited = true;
  return DARIS_OK;
}

daris_status daris_set_timeout(int64_t ns) {
  if (ns < 1) return fail(DARIS_EINVAL, "the wait limit must be positive");
  aql_set_wait_limit_ns(ns);
  return DARIS_OK;
}

daris_status daris_set_plan_cus(int n_cu) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (n_cu < 8 || n_cu > 256) return fail(DARIS_EINVAL, "the nominal partition size must be in 8..256, got %d", n_cu);
  G->plan_cus = n_cu;
  return DARIS_OK;
}

daris_status daris_shutdown(void) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  {
    std::lock_guard<std::mutex> lk(G->mu);
    G->stop = true;
    G->stop_flag = true;
  }
  for (PartRt& P : G->parts)
    for (auto& S : P.streams) {
      S->cv.notify_all();
      if (S->thr.joinable()) S->thr.join();
    }
  if (!G->nodev) {
    // Work that a failed wait left behind may still be executing: let every queue run dry (bounded) before its buffers
    // are freed; destroying the queue afterwards stops whatever is left on it.
    if (G->failed.load()) {
      for (PartRt& P : G->parts)
        for (auto& S : P.streams)
          if (S->hw && S->hw->q.valid()) (void)S->hw->q.drain(g_rt.new_signal(1), 5ll * 1000 * 1000 * 1000);
    }
    (void)hipDeviceSynchronize();
    for (auto& T : G->tasks) free_task(*T);
    for (PartRt& P : G->parts)
      for (auto& S : P.streams) {
        if (S->hw) S->hw->q.destroy();  // destroying a shared queue again is a no-op
        g_rt.free_signal(S->done);
        g_rt.free_signal(S->begin);
        for (hsa_signal_t sg : S->tsig) g_rt.free_signal(sg);
      }
    g_rt.free_signal(G->util_sig);
  }
  delete G;
  G = nullptr;
  return DARIS_OK;
}

daris_part daris_create_partition(int n_cu) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (G->frozen) return fail(DARIS_ESTATE, "partitions must be created before the first execution or daris_commit");
  if (n_cu < 1 || n_cu > 256) return fail(DARIS_EINVAL, "n_cu must be in 1..256, got %d", n_cu);
  if (G->parts.size() >= 255) return fail(DARIS_ERANGE, "too many partitions");
  PartRt P;
  P.n_cu = n_cu;
  P.start = G->cu_cursor;
  for (int i = 0; i < n_cu; ++i) {
    const int cu = (P.start + i) % 256;
    P.mask[cu / 32] |= 1u << (cu % 32);
  }
  G->cu_cursor = (G->cu_cursor + n_cu) % 256;
  G->parts.push_back(P);
  return G->core.add_partition(1);
}

daris_status daris_partition_set_streams(daris_part p, int n_s) {
  daris_status st = check_part(p);
  if (st != DARIS_OK) return st;
  if (G->frozen) return fail(DARIS_ESTATE, "stream count must be set before the first execution or daris_commit");
  if (n_s < 1 || n_s > 8) return fail(DARIS_EINVAL, "n_s must be in 1..8");
  G->parts[p].n_streams = n_s;
  G->core.set_streams(p, n_s);
  return DARIS_OK;
}

daris_status daris_partition_get_mask(daris_part p, uint32_t mask_out[8]) {
  daris_status st = check_part(p, true);
  if (st != DARIS_OK) return st;
  if (!mask_out) return fail(DARIS_EINVAL, "mask_out is NULL");
  std::memcpy(mask_out, G->parts[p].mask, sizeof(uint32_t) * 8);
  return DARIS_OK;
}

daris_task daris_register_task(const daris_dnn* dnn, int64_t period_ns, int64_t deadline_ns, int priority) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (check_failed() != DARIS_OK) return DARIS_EHIP;
  if (G->committed) return fail(DARIS_ESTATE, "tasks must be registered before daris_commit");
  if (!dnn) return fail(DARIS_EINVAL, "dnn is NULL");
  if (period_ns <= 0 || deadline_ns <= 0) return fail(DARIS_EINVAL, "period and deadline must be positive");
  if (priority != DARIS_HP && priority != DARIS_LP) return fail(DARIS_EINVAL, "priority must be DARIS_HP or DARIS_LP");
  if (G->tasks.size() >= 65535) return fail(DARIS_ERANGE, "too many tasks");
  std::unique_ptr<TaskRt> T(new TaskRt());
  std::string err = build_plan(*dnn, G->flags & DARIS_KEEP_ACTIVATIONS, !(G->flags & DARIS_NO_PAIR), !(G->flags & DARIS_NO_FUSED_INGEST), !(G->flags & DARIS_NO_STAGED_ROWS), !(G->flags & DARIS_NO_SMALL_TILES), !(G->flags & DARIS_NO_FUSED_DW), G->plan_cus, &T->net);
  if (!err.empty()) return fail(DARIS_EINVAL, "%s", err.c_str());
  if (!G->nodev) {
    NetPlan& net = T->net;
    auto dev_alloc = [&](size_t bytes, void** out) -> hipError_t {
      hipError_t e = hipMalloc(out, bytes ? bytes : 16);
      if (e == hipSuccess) T->owned.push_back(*out);
      return e;
    };
    for (size_t i = 0; i < net.layers.size(); ++i) {
      LayerPlan& L = net.layers[i];
      const daris_layer& src = dnn->layers[i];
      if (L.d.op != DARIS_OP_CONV && L.d.op != DARIS_OP_FC) continue;
      if (!src.w) {
        free_task(*T);
        return fail(DARIS_EINVAL, "layer %zu has no weights", i);
      }
      std::vector<unsigned char> wp;
      std::vector<float> bp;
      if (L.d.op == DARIS_OP_CONV) pack_conv(net, L, src.w, src.b, &wp, &bp);
      else pack_fc(net, L, src.w, src.b, &wp, &bp);
      hipError_t e = dev_alloc(wp.size(), &L.w_dev);
      if (e == hipSuccess) e = dev_alloc(bp.size() * sizeof(float), (void**)&L.b_dev);
      if (e == hipSuccess) e = hipMemcpy(L.w_dev, wp.data(), wp.size(), hipMemcpyHostToDevice);
      if (e == hipSuccess) e = hipMemcpy(L.b_dev, bp.data(), bp.size() * sizeof(float), hipMemcpyHostToDevice);
      if (e != hipSuccess) {
        free_task(*T);
        return fail(e == hipErrorOutOfMemory ? DARIS_ENOMEM : DARIS_EHIP, "weight upload of layer %zu: %s", i, hipGetErrorString(e));
      }
    }
    T->slots.resize(net.slot_bytes.size());
    for (size_t i = 0; i < net.slot_bytes.size(); ++i) {
      hipError_t e = dev_alloc(net.slot_bytes[i], &T->slots[i]);
      if (e == hipSuccess) e = hipMemset(T->slots[i], 0, net.slot_bytes[i]);
      if (e != hipSuccess) {
        free_task(*T);
        return fail(DARIS_ENOMEM, "activation buffer: %s", hipGetErrorString(e));
      }
    }
    if (net.ws_bytes) {
      hipError_t e = dev_alloc(net.ws_bytes, (void**)&T->ws);
      if (e != hipSuccess) {
        free_task(*T);
        return fail(DARIS_ENOMEM, "split-K workspace: %s", hipGetErrorString(e));
      }
    }
    T->prio = priority;
    err = build_launches(*T);
    if (!err.empty()) {
      free_task(*T);
      return fail(DARIS_EHIP, "%s", err.c_str());
    }
  }
  T->prio = priority;
  G->tasks.push_back(std::move(T));
  return G->core.add_task(period_ns, deadline_ns, priority, 1);
}

daris_status daris_split_stages(daris_task t, int k) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  if (G->committed) return fail(DARIS_ESTATE, "stages must be chosen before daris_commit");
  NetPlan& net = G->tasks[t]->net;
  if (k < 1) return fail(DARIS_EINVAL, "k must be >= 1");
  if (k > 255) return fail(DARIS_ERANGE, "k must be <= 255");
  if (!split_stages(&net, k)) return fail(DARIS_ERANGE, "k = %d exceeds the %zu legal cut points + 1", k, net.legal_cuts.size());
  // A depthwise layer is computed inside the next layer's launch only while both lie in one stage: a cut between them makes
  // the depthwise layer's output the tensor that crosses the boundary (and a stage of that layer alone would have no launch).
  bool refused = false;
  for (size_t l = 0; l + 1 < net.layers.size(); ++l) {
    LayerPlan& A = net.layers[l];
    LayerPlan& B = net.layers[l + 1];
    if (!A.fusable_dw || !A.depthwise) continue;
    const bool cut = std::find(net.stage_first.begin(), net.stage_first.end(), (int)l + 1) != net.stage_first.end();
    if (A.fused_dw == !cut) continue;
    A.fused_dw = B.fused_dw = !cut;
    A.pair_with = cut ? -1 : (int)l + 1;
    B.pair_with = cut ? -1 : (int)l;
    B.pair_lead = !cut;
    refused = true;
  }
  if (refused && !G->nodev) {
    TaskRt& T = *G->tasks[t];
    T.static_launches.clear();
    const std::string err = build_launches(T);
    if (!err.empty()) return fail(DARIS_EHIP, "%s", err.c_str());
  }
  G->core.set_stage_count(t, k);
  G->tasks[t]->vt.clear();
  return DARIS_OK;
}

int32_t daris_get_stage_cuts(daris_task t, int32_t* first_layer, int32_t cap) {
  daris_status st = check_task(t, true);
  if (st != DARIS_OK) return st;
  const std::vector<int>& f = G->tasks[t]->net.stage_first;
  for (int i = 0; i < (int)f.size() && i < cap && first_layer; ++i) first_layer[i] = f[i];
  return (int32_t)f.size();
}

int32_t daris_get_launch_plan(daris_task t, int layer, int64_t* out, int32_t cap) {
  daris_status st = check_task(t, true);
  if (st != DARIS_OK) return st;
  const NetPlan& net = G->tasks[t]->net;
  if (layer < 0 || layer >= (int)net.layers.size()) return fail(DARIS_ERANGE, "layer %d out of range", layer);
  if (!out || cap < 27) return fail(DARIS_EINVAL, "out must hold 27 entries");
  const LayerPlan& L = net.layers[layer];
  const ConvPlan& c = L.cp;
  const bool conv = L.d.op == DARIS_OP_CONV && !L.depthwise;
  const int64_t v[27] = {L.kernel_id, conv ? 1 : 0, conv ? c.rows : 0, (int64_t)L.out.H * L.out.W, L.out.Cs, L.K, L.Kpad,
                         c.tn, c.nw, c.S, c.sz, c.sw, c.splitk, c.MT, c.NTn, c.G, c.xmode, (int64_t)c.grid_x, 1, 1,
                         c.threads, (int64_t)c.ws_bytes, L.pair_with, L.pair_lead ? 1 : 0,
                         L.out.slot, net.tensor(L.in_t).slot, L.res_t >= 0 ? net.tensor(L.res_t).slot : -1};
  for (int i = 0; i < 27; ++i) out[i] = v[i];
  return 27;
}

daris_status daris_set_afet(daris_task t, int stage, int64_t ns) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  if (stage < 0 || stage >= G->core.n_stages(t)) return fail(DARIS_ERANGE, "stage %d out of range", stage);
  if (ns <= 0) return fail(DARIS_EINVAL, "AFET must be positive");
  if (G->committed) return fail(DARIS_ESTATE, "AFET must be set before daris_commit");
  G->core.set_afet(t, stage, ns);
  return DARIS_OK;
}

daris_status daris_set_window(int ws) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (ws < 1) return fail(DARIS_EINVAL, "ws must be >= 1");
  G->core.set_window(ws);
  return DARIS_OK;
}

daris_status daris_set_virtual_time(daris_task t, int stage, daris_part p, int64_t job_lo, int64_t job_hi, const int64_t* et_ns) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  st = check_part(p);
  if (st != DARIS_OK) return st;
  if (stage < 0 || stage >= G->core.n_stages(t)) return fail(DARIS_ERANGE, "stage %d out of range", stage);
  if (job_lo < 0 || job_hi < job_lo || !et_ns) return fail(DARIS_EINVAL, "bad job range or NULL table");
  std::vector<int64_t> v(et_ns, et_ns + (job_hi - job_lo));
  for (int64_t x : v)
    if (x < 1) return fail(DARIS_EINVAL, "execution times must be >= 1 ns");
  G->tasks[t]->vt[std::make_pair(stage, (int)p)] = std::make_pair(job_lo, std::move(v));
  return DARIS_OK;
}

// Creates the CU-masked queues of every partition; after this the partition set is frozen.
static daris_status make_streams(void) {
  if (G->frozen) return DARIS_OK;
  if (G->parts.empty()) return fail(DARIS_ESTATE, "no partition");
  if (!G->nodev) {
    for (PartRt& P : G->parts) {
      for (int i = 0; i < P.n_streams; ++i) {
        P.streams.emplace_back(new StreamRt());
        StreamRt& S = *P.streams.back();
        if (i > 0 && (G->flags & DARIS_SHARED_QUEUE)) {
          S.hw = P.streams[0]->hw;
        } else {
          S.hw = std::make_shared<StreamRt::HwQueue>();
          const std::string err = S.hw->q.create(&g_rt, P.mask);
          if (!err.empty()) return fail(DARIS_EHIP, "queue of partition with %d CUs: %s", P.n_cu, err.c_str());
          // completion signals receive the start and end time stamps of their dispatch; switched on before the first
          // packet and left on (a stage carries one signal, so the cost is one record per stage)
          S.hw->q.set_profiling(true);
        }
        S.done = g_rt.new_signal(1);
        S.begin = g_rt.new_signal(1);
        if (!S.done.handle || !S.begin.handle) return fail(DARIS_EHIP, "signal creation failed");
      }
    }
  }
  G->frozen = true;
  return DARIS_OK;
}

daris_status daris_commit(void) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (check_failed() != DARIS_OK) return DARIS_EHIP;
  if (G->committed) return DARIS_OK;
  if (G->tasks.empty()) return fail(DARIS_ESTATE, "no task");
  daris_status st0 = make_streams();
  if (st0 != DARIS_OK) return st0;
  G->core.commit();
  G->committed = true;
  G->epoch = std::chrono::steady_clock::now();
  if (!G->vt)
    for (PartRt& P : G->parts)
      for (auto& S : P.streams) S->thr = std::thread(worker_loop, S.get());
  return DARIS_OK;
}

daris_part daris_get_partition(daris_task t) {
  daris_status st = check_task(t, true);
  if (st != DARIS_OK) return st;
  if (!G->committed) return fail(DARIS_ESTATE, "not committed");
  std::lock_guard<std::mutex> lk(G->mu);
  return G->core.context(t);
}

daris_status daris_release_job(daris_task t, const void* d_input, void* d_logits, int64_t release_ns, int32_t* decision) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  if (!G->nodev && (!d_input || !d_logits)) return fail(DARIS_EINVAL, "NULL device buffer");
  st = daris_commit();
  if (st != DARIS_OK) return st;
  JobIo io;
  io.in = d_input;
  io.out = d_logits;
  if (G->vt) {
    if (release_ns < 0 || release_ns < G->vt_now) return fail(DARIS_ESTATE, "virtual release times must not decrease");
    if (release_ns > G->vt_now) {
      st = vt_advance(release_ns, false);
      if (st != DARIS_OK) return st;
      G->vt_now = release_ns;
      vt_completions_now();
    }
    uint32_t job = 0;
    Decision d = G->core.release(release_ns, t, release_ns, &job);
    if (decision) *decision = (int32_t)d;
    if (d == D_ACCEPTED || d == D_MIGRATED || d == D_QUEUED) G->tasks[t]->io[job] = io;
    G->vt_dirty = true;
    return DARIS_OK;
  }
  {
    std::lock_guard<std::mutex> lk(G->mu);
    const int64_t now = now_ns();
    st = rt_release_locked(t, io, now, release_ns < 0 ? now : release_ns, decision);
  }
  return st;
}

daris_status daris_migrate(daris_task t, daris_part p) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  st = check_part(p);
  if (st != DARIS_OK) return st;
  st = daris_commit();
  if (st != DARIS_OK) return st;
  if (G->vt) {
    G->core.migrate_command(G->vt_now < 0 ? 0 : G->vt_now, t, p);
    G->vt_dirty = true;
    return DARIS_OK;
  }
  std::lock_guard<std::mutex> lk(G->mu);
  const int64_t now = now_ns();
  G->core.migrate_command(now, t, p);
  return dispatch_and_issue(now);
}

daris_status daris_run_until_idle(void) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (check_failed() != DARIS_OK) return DARIS_EHIP;
  if (!G->committed) return DARIS_OK;
  if (G->vt) {
    daris_status st = vt_advance(0, true);
    if (st != DARIS_OK) return st;
    return DARIS_OK;  // with a device every stage was waited for when it was issued
  }
  return wait_idle();
}

daris_status daris_task_set_io(daris_task t, const void* d_inputs, int32_t n_inputs, void* d_logits, int32_t n_slots) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  if (!G->nodev && (!d_inputs || !d_logits)) return fail(DARIS_EINVAL, "NULL device buffer");
  if (n_inputs < 1 || n_slots < 1) return fail(DARIS_EINVAL, "pool sizes must be >= 1");
  TaskRt& T = *G->tasks[t];
  std::lock_guard<std::mutex> lk(G->mu);
  if (G->core.has_active(t)) return fail(DARIS_ESTATE, "task %d has an active job", t);
  T.pool_in = d_inputs;
  T.pool_out = d_logits;
  T.n_inputs = n_inputs;
  T.n_slots = n_slots;
  if (!G->nodev) {
    // The jobs run on queues of the library's own, unordered with the caller's HIP streams: wait here, once, for whatever
    // those streams are still writing into the pools (inputs being uploaded, logits being pre-filled).
    HIP_TRY(hipDeviceSynchronize());
    // argument blocks for every buffer of the two pools, so that a release writes nothing but packets
    free_variants(&T.pool);
    if ((int64_t)n_inputs + n_slots <= (1 << 20)) {
      const NetPlan& n = T.net;
      hipError_t e = build_variants(T, d_inputs, n_inputs, (size_t)n.in_c * n.in_h * n.in_w * sizeof(float), d_logits, n_slots,
                                    (size_t)n.n_out * sizeof(float), &T.pool);
      if (e != hipSuccess) return fail(e == hipErrorOutOfMemory ? DARIS_ENOMEM : DARIS_EHIP, "argument blocks of the I/O pool: %s", hipGetErrorString(e));
    }
  }
  return DARIS_OK;
}

daris_status daris_run_periodic(const int64_t* phase_ns, const int32_t* n_jobs) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (check_failed() != DARIS_OK) return DARIS_EHIP;
  if (!n_jobs) return fail(DARIS_EINVAL, "n_jobs is NULL");
  daris_status st = daris_commit();
  if (st != DARIS_OK) return st;
  struct Rel {
    int64_t t;
    int task;
    uint32_t m;
  };
  std::vector<Rel> rels;
  for (int i = 0; i < (int)G->tasks.size(); ++i) {
    if (n_jobs[i] > 0 && G->tasks[i]->n_inputs < 1) return fail(DARIS_ESTATE, "task %d has no I/O pool (daris_task_set_io)", i);
    const int64_t ph = phase_ns ? phase_ns[i] : 0;
    if (ph < 0) return fail(DARIS_EINVAL, "phases must be >= 0");
    const int64_t period = G->core.period(i);
    for (int32_t m = 0; m < n_jobs[i]; ++m) rels.push_back(Rel{ph + (int64_t)m * period, i, (uint32_t)m});
  }
  std::sort(rels.begin(), rels.end(), [](const Rel& a, const Rel& b) {
    if (a.t != b.t) return a.t < b.t;
    if (a.task != b.task) return a.task < b.task;
    return a.m < b.m;
  });
  const int64_t base = G->vt ? (G->vt_now < 0 ? 0 : G->vt_now + 1) : now_ns() + 200000;  // real time: start 0.2 ms from now
  for (const Rel& r : rels) {
    TaskRt& T = *G->tasks[r.task];
    const int64_t t = base + r.t;
    if (G->vt) {
      const uint32_t job = (uint32_t)G->core.stats(r.task).released;
      st = daris_release_job(r.task, G->nodev ? nullptr : pool_io(T, job).in, G->nodev ? nullptr : pool_io(T, job).out, t, nullptr);
      if (st != DARIS_OK) return st;
      continue;
    }
    // sleep most of the wait, spin the last stretch
    for (;;) {
      const int64_t left = t - now_ns();
      if (left <= 0) break;
      if (left > 150000) std::this_thread::sleep_for(std::chrono::nanoseconds(left - 100000));
    }
    {
      std::lock_guard<std::mutex> lk(G->mu);
      const uint32_t job = (uint32_t)G->core.stats(r.task).released;
      st = rt_release_locked(r.task, pool_io(T, job), now_ns(), t, nullptr);
    }
      if (st != DARIS_OK) return st;
  }
  return daris_run_until_idle();
}

daris_status daris_run_closed_loop(const int32_t* n_jobs, int64_t total_jobs) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (check_failed() != DARIS_OK) return DARIS_EHIP;
  if (G->vt) return fail(DARIS_ESTATE, "closed-loop runs need real-time mode");
  if (!n_jobs) return fail(DARIS_EINVAL, "n_jobs is NULL");
  daris_status st = daris_commit();
  if (st != DARIS_OK) return st;
  for (int i = 0; i < (int)G->tasks.size(); ++i)
    if (n_jobs[i] > 0 && G->tasks[i]->n_inputs < 1) return fail(DARIS_ESTATE, "task %d has no I/O pool (daris_task_set_io)", i);
  {
    std::lock_guard<std::mutex> lk(G->mu);
    const int64_t now = now_ns();
    G->closed_total_left = total_jobs > 0 ? total_jobs : -1;
    for (int i = 0; i < (int)G->tasks.size(); ++i) G->tasks[i]->closed_left = n_jobs[i];
    for (int i = 0; i < (int)G->tasks.size(); ++i) {
      TaskRt& T = *G->tasks[i];
      // a rejected release ends no job, so keep releasing until one is admitted or the budget is spent
      while (T.closed_left > 0 && G->closed_total_left != 0 && !G->core.has_active(i)) {
        T.closed_left--;
        if (G->closed_total_left > 0) G->closed_total_left--;
        const uint32_t job = (uint32_t)G->core.stats(i).released;
        st = rt_release_locked(i, pool_io(T, job), now, now, nullptr);
        if (st != DARIS_OK) return st;
      }
    }
  }
  daris_status st2 = wait_idle();
  {
    std::lock_guard<std::mutex> lk(G->mu);
    for (auto& T : G->tasks) T->closed_left = 0;
    G->closed_total_left = -1;
  }
  return st2;
}

daris_status daris_get_stats(daris_task t, daris_task_stats* out) {
  daris_status st = check_task(t, true);
  if (st != DARIS_OK) return st;
  if (!out) return fail(DARIS_EINVAL, "out is NULL");
  std::lock_guard<std::mutex> lk(G->mu);
  const TaskStats& s = G->core.stats(t);
  out->released = s.released;
  out->accepted = s.accepted;
  out->completed = s.completed;
  out->missed = s.missed;
  out->rejected_admission = s.rej_adm;
  out->rejected_overrun = s.rej_over;
  out->resp_min_ns = s.resp_min;
  out->resp_max_ns = s.resp_max;
  out->resp_sum_ns = s.resp_sum;
  out->first_release_ns = s.first_release;
  out->last_finish_ns = s.last_finish;
  out->partition = G->core.context(t);
  out->n_stages = G->core.n_stages(t);
  return DARIS_OK;
}

int64_t daris_trace_read(void* buf, int64_t cap_bytes) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (!buf || cap_bytes < 0) return fail(DARIS_EINVAL, "bad buffer");
  std::lock_guard<std::mutex> lk(G->mu);
  std::vector<TraceRec>& tr = G->core.trace();
  const size_t n = std::min<size_t>((size_t)cap_bytes / sizeof(TraceRec), tr.size());
  std::memcpy(buf, tr.data(), n * sizeof(TraceRec));
  tr.erase(tr.begin(), tr.begin() + n);  // consumed records are released
  return (int64_t)(n * sizeof(TraceRec));
}

int64_t daris_get_mret(daris_task t, int stage) {
  daris_status st = check_task(t, true);
  if (st != DARIS_OK) return st;
  if (stage < 0 || stage >= G->core.n_stages(t)) return fail(DARIS_ERANGE, "stage %d out of range", stage);
  std::lock_guard<std::mutex> lk(G->mu);
  return G->core.mret_stage(t, stage);
}

// ---- direct execution ---------------------------------------------------------------------------------------------------

static daris_status direct_checks(daris_task t, daris_part p) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  st = check_part(p);
  if (st != DARIS_OK) return st;
  if (G->nodev) return fail(DARIS_ESTATE, "no device in DARIS_NO_DEVICE mode");
  return make_streams();
}

daris_status daris_forward(daris_task t, const void* d_input, void* d_logits, daris_part p) {
  daris_status st = direct_checks(t, p);
  if (st != DARIS_OK) return st;
  if (!d_input || !d_logits) return fail(DARIS_EINVAL, "NULL device buffer");
  std::lock_guard<std::mutex> lk(G->mu);
  if (G->core.has_active(t)) return fail(DARIS_ESTATE, "task %d has an active job", t);
  TaskRt& T = *G->tasks[t];
  HIP_TRY(hipDeviceSynchronize());  // the caller's streams may still be writing the two buffers (see daris_task_set_io)
  JobIo io;
  io.in = d_input;
  io.out = d_logits;
  return run_direct(T, 0, (int)T.launches.size(), io, *G->parts[p].streams[0]);
}

// For callers that cannot allocate device memory.  Nothing below calls hipMalloc, hipFree or any routine that allocates
// device or pinned memory: the queues, signals and argument rings exist already, the network's tensors go into the static
// device array, and each launch's argument block travels through its queue's ring of host-coherent memory.
daris_status daris_forward_static(daris_task t, const void* d_input, void* d_logits, daris_part p) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  st = check_part(p);
  if (st != DARIS_OK) return st;
  if (G->nodev) return fail(DARIS_ESTATE, "no device in DARIS_NO_DEVICE mode");
  if (!G->frozen) return fail(DARIS_ESTATE, "the streams do not exist yet (creating them allocates): call daris_commit, or run anything once, before daris_forward_static");
  if (!d_input || !d_logits) return fail(DARIS_EINVAL, "NULL device buffer");
  std::lock_guard<std::mutex> lk(G->mu);
  if (G->core.has_active(t)) return fail(DARIS_ESTATE, "task %d has an active job", t);
  TaskRt& T = *G->tasks[t];
  unsigned char* base = static_cast<unsigned char*>(static_scratch_ptr(G->device));
  if (!base) return fail(DARIS_EHIP, "the static scratch of device %d was not set up", G->device);
  // layout: the plan's activation slots one after the other, 256 bytes apart at least, then the split-K workspace
  const NetPlan& net = T.net;
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  size_t need = up(net.ws_bytes);
  for (size_t b : net.slot_bytes) need += up(b);
  if (need > (size_t)DARIS_STATIC_SCRATCH_BYTES)
    return fail(DARIS_ERANGE, "task %d needs %zu bytes of activation buffers and split-K workspace; the static scratch holds %u", t, need,
                (unsigned)DARIS_STATIC_SCRATCH_BYTES);
  if (T.static_launches.empty()) {
    std::vector<void*> slots(net.slot_bytes.size());
    size_t off = 0;
    for (size_t i = 0; i < slots.size(); ++i) {
      slots[i] = base + off;
      off += up(net.slot_bytes[i]);
    }
    IoLaunches iol;
    const std::string err = encode_network(T, slots, reinterpret_cast<float*>(base + off), &T.static_launches, &T.static_layer_lo, &iol);
    if (!err.empty()) {
      T.static_launches.clear();
      return fail(DARIS_EHIP, "%s", err.c_str());
    }
    T.static_in = iol.in_launch;
    T.static_out = iol.out_launch;
    T.static_in_off = iol.in_off;
    T.static_out_off = iol.out_off;
  }
  HIP_TRY(hipDeviceSynchronize());  // the caller's streams may still be writing the two buffers (see daris_task_set_io)
  StreamRt& S = *G->parts[p].streams[0];
  const int n = (int)T.static_launches.size();
  {
    std::lock_guard<std::mutex> ql(S.hw->mu);
    for (int i = 0; i < n; ++i) {
      const KernelLaunch& kl = T.static_launches[i].kl;
      alignas(8) unsigned char blk[sizeof(KernelLaunch::args)];
      std::memcpy(blk, kl.args, kl.nbytes);
      if (i == T.static_in) std::memcpy(blk + T.static_in_off, &d_input, sizeof(void*));
      if (i == T.static_out) std::memcpy(blk + T.static_out_off, &d_logits, sizeof(void*));
      const unsigned fl = (i == 0 ? AqlQueue::kAcquireSystem : 0u) | (i == n - 1 ? AqlQueue::kReleaseSystem : 0u);
      if (!S.hw->q.dispatch_copy(*kl.k, kl.groups, kl.threads, blk, kl.nbytes, i == n - 1 ? G->util_sig : hsa_signal_t{0}, fl)) {
        // Launches already queued keep running on the static array; the next call would race with them.
        return gpu_wait_failed(S, "daris_forward_static: packet rejected");
      }
    }
  }
  if (!aql_wait(G->util_sig, &S.hw->q)) return gpu_wait_failed(S, "daris_forward_static");
  return DARIS_OK;
}

daris_status daris_read_layer(daris_task t, int layer, float* host_out, int64_t cap_elems) {
  daris_status st = check_task(t);
  if (st != DARIS_OK) return st;
  if (G->nodev) return fail(DARIS_ESTATE, "no device in DARIS_NO_DEVICE mode");
  if (!(G->flags & DARIS_KEEP_ACTIVATIONS)) return fail(DARIS_ESTATE, "needs DARIS_KEEP_ACTIVATIONS");
  TaskRt& T = *G->tasks[t];
  if (layer < -1 || layer >= (int)T.net.layers.size()) return fail(DARIS_ERANGE, "layer %d out of range", layer);
  const TensorInfo& o = T.net.tensor(layer + 1);
  if (o.slot < 0) return fail(DARIS_ESTATE, "layer %d writes straight to the caller's logits", layer);
  const int64_t n = (int64_t)o.C * o.H * o.W;
  if (!host_out || cap_elems < n) return fail(DARIS_EINVAL, "host buffer too small (%lld needed)", (long long)n);
  st = make_streams();
  if (st != DARIS_OK) return st;
  std::lock_guard<std::mutex> lk(G->mu);
  float* tmp = nullptr;
  HIP_TRY(hipMalloc((void**)&tmp, (size_t)n * sizeof(float)));
  std::vector<KernelLaunch> ks;
  st = encode_egress(g_kt, T.slots[o.slot], tmp, o.C, o.Cs, o.H, o.W, T.net.bf16, &ks) ? run_one(ks, *G->parts[0].streams[0])
                                                                                      : fail(DARIS_EHIP, "read_layer: launch encoding");
  hipError_t e = st == DARIS_OK ? hipMemcpy(host_out, tmp, (size_t)n * sizeof(float), hipMemcpyDeviceToHost) : hipSuccess;
  (void)hipFree(tmp);
  if (e != hipSuccess) return fail(DARIS_EHIP, "read_layer: %s", hipGetErrorString(e));
  return st;
}

daris_status daris_profile_layers(daris_task t, daris_part p, int reps, float* ms_per_layer, int32_t* kernel_id, double* flops) {
  daris_status st = direct_checks(t, p);
  if (st != DARIS_OK) return st;
  if (reps < 1 || !ms_per_layer) return fail(DARIS_EINVAL, "bad arguments");
  std::lock_guard<std::mutex> lk(G->mu);
  if (G->core.has_active(t)) return fail(DARIS_ESTATE, "task %d has an active job", t);
  TaskRt& T = *G->tasks[t];
  StreamRt& S = *G->parts[p].streams[0];
  const int n = (int)T.net.layers.size();
  float* scratch_out = nullptr;
  HIP_TRY(hipMalloc((void**)&scratch_out, (size_t)std::max(T.net.n_out, 4) * sizeof(float)));
  float* scratch_in = nullptr;  // stands in for the caller's input where layer 0 reads it directly
  const size_t in_bytes = (size_t)T.net.in_c * T.net.in_h * T.net.in_w * sizeof(float);
  IoVariants var;
  hipError_t ea = hipMalloc((void**)&scratch_in, in_bytes);
  if (ea == hipSuccess) ea = hipMemset(scratch_in, 0, in_bytes);
  if (ea == hipSuccess) ea = build_variants(T, scratch_in, 1, 0, scratch_out, 1, 0, &var);
  hsa_signal_t first = g_rt.new_signal(1);
  if (ea != hipSuccess || !first.handle) {
    (void)hipFree(scratch_out);
    if (scratch_in) (void)hipFree(scratch_in);
    g_rt.free_signal(first);
    return fail(DARIS_ENOMEM, "profile buffers: %s", ea != hipSuccess ? hipGetErrorString(ea) : "signal creation failed");
  }
  JobIo io;
  io.in = scratch_in;
  io.out = scratch_out;
  if (!var.in.empty()) io.in_args = var.in[0];
  if (!var.out.empty()) io.out_args = var.out[0];
  daris_status result = DARIS_OK;
  std::lock_guard<std::mutex> ql(S.hw->mu);
  for (int l = 0; l < n && result == DARIS_OK; ++l) {
    const int lo = T.layer_lo[l], hi = T.layer_lo[l + 1];
    ms_per_layer[l] = 0.f;
    if (kernel_id) kernel_id[l] = T.net.layers[l].kernel_id;
    if (flops) flops[l] = 2.0 * (double)T.net.layers[l].macs;
    if (lo == hi) continue;  // the earlier member of a launch pair: its work is timed with the later one
    // one warm-up pass, then `reps` passes back to back: from the start of the first kernel to the end of the last
    const bool one = reps == 1 && hi - lo == 1;  // then the only launch carries the completion signal
    const char* err = nullptr;
    for (int r = -1; r < reps && !err; ++r) {
      EnqueueOpts o;
      if (r == 0 && !one) o.first = first;
      if (r == reps - 1) o.done = G->util_sig;
      o.acquire_system = r == -1;
      o.release_system = r == reps - 1;
      err = enqueue_range(T, lo, hi, io, S, o);
    }
    if (err) {
      result = fail(DARIS_EHIP, "profiling layer %d: %s", l, err);
      break;  // nothing was given the completion signal: do not wait
    }
    if (!aql_spin(G->util_sig, &S.hw->q)) {
      result = gpu_wait_failed(S, "layer profile");
      break;
    }
    double a0 = 0, b0 = 0, a1 = 0, b1 = 0;
    bool ok = g_rt.dispatch_time_us(G->util_sig, &a1, &b1);
    if (one) a0 = a1;
    else ok = ok && g_rt.dispatch_time_us(first, &a0, &b0);
    hsa_signal_store_relaxed(G->util_sig, 1);
    hsa_signal_store_relaxed(first, 1);
    if (!ok) result = fail(DARIS_EHIP, "profiling layer %d: no time stamps", l);
    ms_per_layer[l] = (float)((b1 - a0) * 1e-3 / reps);
  }
  g_rt.free_signal(first);
  free_variants(&var);
  (void)hipFree(scratch_out);
  (void)hipFree(scratch_in);
  return result;
}

const char* daris_kernel_name(int32_t kernel_id) { return kernel_name(kernel_id); }

daris_status daris_kernel_timing_start(int every, int max_samples) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (G->nodev) return fail(DARIS_ESTATE, "no device in DARIS_NO_DEVICE mode");
  if (every < 0 || max_samples < 0 || max_samples > 1000000) return fail(DARIS_EINVAL, "bad arguments");
  daris_status st = make_streams();
  if (st != DARIS_OK) return st;
  std::lock_guard<std::mutex> lk(G->mu);
  if (!G->core.idle()) return fail(DARIS_ESTATE, "jobs are active");
  for (int i = 0; i < K_COUNT; ++i) {
    G->tm_launches[i] = 0;
    G->tm_ms[i] = 0;
    G->tm_flops[i] = 0;
  }
  G->tm_left = max_samples;
  G->tm_every = every;
  return DARIS_OK;
}

int32_t daris_kernel_timing_read(int32_t cap, int64_t* launches, double* total_ms, double* total_flops, double* empty_pair_ms) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (cap < K_COUNT || !launches || !total_ms || !total_flops) return fail(DARIS_EINVAL, "arrays must hold %d entries", (int)K_COUNT);
  daris_status st = daris_run_until_idle();
  if (st != DARIS_OK) return st;
  std::lock_guard<std::mutex> lk(G->mu);
  G->tm_every = 0;
  for (int i = 0; i < K_COUNT; ++i) {
    launches[i] = G->tm_launches[i];
    total_ms[i] = G->tm_ms[i];
    total_flops[i] = G->tm_flops[i];
    G->tm_launches[i] = 0;
    G->tm_ms[i] = 0;
    G->tm_flops[i] = 0;
  }
  // the durations are the command processor's own start and end stamps of each dispatch: nothing to subtract
  if (empty_pair_ms) *empty_pair_ms = 0.0;
  return K_COUNT;
}

daris_status daris_driver_profile(int enable, int64_t* out) {
  if (!G || !G->inited) return fail(DARIS_ESTATE, "library not initialised");
  if (G->vt) return fail(DARIS_ESTATE, "the driver profile belongs to real-time mode");
  daris_status st = daris_run_until_idle();
  if (st != DARIS_OK) return st;
  std::lock_guard<std::mutex> lk(G->mu);
  if (out)
    for (int i = 0; i < 8; ++i) out[i] = G->prof_acc[i];
  for (int i = 0; i < 8; ++i) G->prof_acc[i] = 0;
  G->prof = enable != 0;
  return DARIS_OK;
}

daris_status daris_probe_cus(daris_part p, int n_groups, int spin, uint32_t* out) {
  daris_status st = check_part(p);
  if (st != DARIS_OK) return st;
  if (G->nodev) return fail(DARIS_ESTATE, "no device in DARIS_NO_DEVICE mode");
  if (n_groups < 1 || n_groups > 65536 || spin < 0 || spin > 100000 || !out) return fail(DARIS_EINVAL, "bad arguments");
  st = make_streams();
  if (st != DARIS_OK) return st;
  uint32_t* d = nullptr;
  const size_t bytes = (size_t)n_groups * 2 * sizeof(uint32_t);
  HIP_TRY(hipMalloc((void**)&d, bytes));
  std::vector<KernelLaunch> ks;
  {
    std::lock_guard<std::mutex> lk(G->mu);
    st = encode_cu_probe(g_kt, d, n_groups, spin, &ks) ? run_one(ks, *G->parts[p].streams[0]) : fail(DARIS_EHIP, "probe: launch encoding");
  }
  hipError_t e = st == DARIS_OK ? hipMemcpy(out, d, bytes, hipMemcpyDeviceToHost) : hipSuccess;
  (void)hipFree(d);
  if (e != hipSuccess) return fail(DARIS_EHIP, "probe: %s", hipGetErrorString(e));
  return st;
}

daris_status daris_calibrate_afet(daris_task t, daris_part p, int reps) {
  daris_status st = direct_checks(t, p);
  if (st != DARIS_OK) return st;
  if (reps < 1) return fail(DARIS_EINVAL, "reps must be >= 1");
  std::lock_guard<std::mutex> lk(G->mu);
  if (G->core.has_active(t) || G->core.stats(t).released > 0) return fail(DARIS_ESTATE, "calibrate before the first release of task %d", t);
  TaskRt& T = *G->tasks[t];
  StreamRt& S = *G->parts[p].streams[0];
  const int k = (int)T.net.stage_first.size();
  float* in = nullptr;
  float* out = nullptr;
  const size_t in_elems = (size_t)T.net.in_c * T.net.in_h * T.net.in_w;
  IoVariants var;
  hipError_t ea = hipMalloc((void**)&in, in_elems * sizeof(float));
  if (ea == hipSuccess) ea = hipMemset(in, 0, in_elems * sizeof(float));
  if (ea == hipSuccess) ea = hipMalloc((void**)&out, (size_t)std::max(T.net.n_out, 4) * sizeof(float));
  if (ea == hipSuccess) ea = build_variants(T, in, 1, 0, out, 1, 0, &var);
  if (ea != hipSuccess) {
    if (in) (void)hipFree(in);
    if (out) (void)hipFree(out);
    return fail(DARIS_ENOMEM, "calibration buffers: %s", hipGetErrorString(ea));
  }
  JobIo io;
  io.in = in;
  io.out = out;
  if (!var.in.empty()) io.in_args = var.in[0];
  if (!var.out.empty()) io.out_args = var.out[0];
  std::vector<int64_t> best(k, 0);
  daris_status result = DARIS_OK;
  for (int r = 0; r <= reps && result == DARIS_OK; ++r) {  // run 0 is a warm-up
    for (int j = 0; j < k; ++j) {
      int lo, hi;
      stage_range(T, j, &lo, &hi);
      auto t0 = std::chrono::steady_clock::now();
      result = run_direct(T, lo, hi, io, S);
      auto t1 = std::chrono::steady_clock::now();
      if (result != DARIS_OK) break;
      const int64_t ns = std::chrono::duration_cast<std::chrono::nanoseconds>(t1 - t0).count();
      if (r > 0) best[j] = std::max(best[j], ns);
    }
  }
  free_variants(&var);
  (void)hipFree(in);
  (void)hipFree(out);
  if (result != DARIS_OK) return result;
  for (int j = 0; j < k; ++j) G->core.set_afet(t, j, std::max<int64_t>(best[j], 1));
  return DARIS_OK;
}

// Sec. IV-A1: AFET = average execution time of the target while other tasks run in the remaining streams.
daris_status daris_calibrate_afet_loaded(daris_task t, daris_part p, int reps) {
  daris_status st = direct_checks(t, p);
  if (st != DARIS_OK) return st;
  if (reps < 1) return fail(DARIS_EINVAL, "reps must be >= 1");
  std::lock_guard<std::mutex> lk(G->mu);
  for (int i = 0; i < (int)G->tasks.size(); ++i)
    if (G->core.has_active(i)) return fail(DARIS_ESTATE, "calibrate while no job is active");
  if (G->core.stats(t).released > 0) return fail(DARIS_ESTATE, "calibrate before the first release of task %d", t);
  const int nt = (int)G->tasks.size();
  // one zero-filled input and one logits buffer per task
  std::vector<float*> in(nt, nullptr), out(nt, nullptr);
  IoVariants var;  // the target's two job-dependent argument blocks, in device memory as in production
  auto cleanup = [&]() {
    for (float* q : in) if (q) (void)hipFree(q);
    for (float* q : out) if (q) (void)hipFree(q);
    free_variants(&var);
  };
  for (int i = 0; i < nt; ++i) {
    const NetPlan& n = G->tasks[i]->net;
    const size_t ie = (size_t)n.in_c * n.in_h * n.in_w;
    hipError_t e = hipMalloc((void**)&in[i], ie * sizeof(float));
    if (e == hipSuccess) e = hipMemset(in[i], 0, ie * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&out[i], (size_t)std::max(n.n_out, 4) * sizeof(float));
    if (e != hipSuccess) {
      cleanup();
      return fail(DARIS_ENOMEM, "calibration buffers: %s", hipGetErrorString(e));
    }
  }
  TaskRt& T = *G->tasks[t];
  StreamRt& S = *G->parts[p].streams[0];
  {
    hipError_t e = build_variants(T, in[t], 1, 0, out[t], 1, 0, &var);
    if (e != hipSuccess) {
      cleanup();
      return fail(DARIS_ENOMEM, "calibration buffers: %s", hipGetErrorString(e));
    }
  }
  const int k = (int)T.net.stage_first.size();
  std::vector<int64_t> sum(k, 0);
  uint64_t rng = G->seed * 6364136223846793005ull + 1442695040888963407ull + (uint64_t)t;
  daris_status result = DARIS_OK;
  for (int r = 0; r <= reps && result == DARIS_OK; ++r) {  // run 0 is a warm-up
    // every other stream gets one whole forward pass of a distinct, randomly drawn other task
    std::vector<int> others;
    for (int i = 0; i < nt; ++i)
      if (i != t) others.push_back(i);
    std::vector<StreamRt*> loaded;
    for (size_t q = 0; q < G->parts.size() && result == DARIS_OK; ++q)
      for (size_t si = 0; si < G->parts[q].streams.size() && result == DARIS_OK; ++si) {
        if ((int)q == p && si == 0) continue;
        if (others.empty()) break;
        rng = rng * 6364136223846793005ull + 1442695040888963407ull;
        const size_t pick = (size_t)((rng >> 33) % others.size());
        const int o = others[pick];
        others.erase(others.begin() + pick);
        TaskRt& O = *G->tasks[o];
        StreamRt& Q = *G->parts[q].streams[si];
        JobIo io;
        io.in = in[o];
        io.out = out[o];
        EnqueueOpts eo;
        eo.done = Q.done;  // no job is active, so the stream's worker is not using its signal
        eo.acquire_system = eo.release_system = true;
        std::lock_guard<std::mutex> ql(Q.hw->mu);
        const char* err = enqueue_range(O, 0, (int)O.launches.size(), io, Q, eo);
        if (err) result = fail(DARIS_EHIP, "calibration load: %s", err);
        else loaded.push_back(&Q);
      }
    JobIo io;
    io.in = in[t];
    io.out = out[t];
    if (!var.in.empty()) io.in_args = var.in[0];
    if (!var.out.empty()) io.out_args = var.out[0];
    for (int j = 0; j < k && result == DARIS_OK; ++j) {
      int lo, hi;
      stage_range(T, j, &lo, &hi);
      auto t0 = std::chrono::steady_clock::now();
      result = run_direct(T, lo, hi, io, S);
      auto t1 = std::chrono::steady_clock::now();
      if (r > 0) sum[j] += std::chrono::duration_cast<std::chrono::nanoseconds>(t1 - t0).count();
    }
    for (StreamRt* Q : loaded)
      if (!aql_wait(Q->done, &Q->hw->q) && result == DARIS_OK) result = gpu_wait_failed(*Q, "calibration load");
  }
  cleanup();
  if (result != DARIS_OK) return result;
  for (int j = 0; j < k; ++j) G->core.set_afet(t, j, std::max<int64_t>(sum[j] / reps, 1));
  return DARIS_OK;
}

}  // extern "C"
