#include "aql.h"

#include <cxxabi.h>
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>

namespace daris {

namespace {

std::string hsa_err(const char* what, hsa_status_t st) {
  const char* msg = nullptr;
  hsa_status_string(st, &msg);
  return std::string(what) + ": " + (msg ? msg : "unknown HSA error");
}

struct AgentScan {
  std::vector<hsa_agent_t> gpus;
  hsa_agent_t cpu{};
  bool have_cpu = false;
};

hsa_status_t scan_agents(hsa_agent_t a, void* data) {
  AgentScan* s = (AgentScan*)data;
  hsa_device_type_t t;
  if (hsa_agent_get_info(a, HSA_AGENT_INFO_DEVICE, &t) != HSA_STATUS_SUCCESS) return HSA_STATUS_SUCCESS;
  if (t == HSA_DEVICE_TYPE_GPU) s->gpus.push_back(a);
  else if (t == HSA_DEVICE_TYPE_CPU && !s->have_cpu) {
    s->cpu = a;
    s->have_cpu = true;
  }
  return HSA_STATUS_SUCCESS;
}

struct PoolScan {
  hsa_amd_memory_pool_t pool{};
  bool found = false;
};

hsa_status_t scan_host_pools(hsa_amd_memory_pool_t p, void* data) {
  PoolScan* s = (PoolScan*)data;
  hsa_amd_segment_t seg;
  uint32_t flags = 0;
  bool alloc_ok = false;
  if (hsa_amd_memory_pool_get_info(p, HSA_AMD_MEMORY_POOL_INFO_SEGMENT, &seg) != HSA_STATUS_SUCCESS || seg != HSA_AMD_SEGMENT_GLOBAL)
    return HSA_STATUS_SUCCESS;
  hsa_amd_memory_pool_get_info(p, HSA_AMD_MEMORY_POOL_INFO_GLOBAL_FLAGS, &flags);
  hsa_amd_memory_pool_get_info(p, HSA_AMD_MEMORY_POOL_INFO_RUNTIME_ALLOC_ALLOWED, &alloc_ok);
  if ((flags & HSA_AMD_MEMORY_POOL_GLOBAL_FLAG_KERNARG_INIT) && alloc_ok && !s->found) {
    s->pool = p;
    s->found = true;
  }
  return HSA_STATUS_SUCCESS;
}

struct SymbolScan {
  std::unordered_map<std::string, AqlKernel>* out;
  std::string error;
};

hsa_status_t scan_symbols(hsa_executable_t, hsa_agent_t, hsa_executable_symbol_t sym, void* data) {
  SymbolScan* s = (SymbolScan*)data;
  hsa_symbol_kind_t kind;
  if (hsa_executable_symbol_get_info(sym, HSA_EXECUTABLE_SYMBOL_INFO_TYPE, &kind) != HSA_STATUS_SUCCESS || kind != HSA_SYMBOL_KIND_KERNEL)
    return HSA_STATUS_SUCCESS;
  uint32_t len = 0;
  hsa_executable_symbol_get_info(sym, HSA_EXECUTABLE_SYMBOL_INFO_NAME_LENGTH, &len);
  std::string name(len, '\0');
  hsa_executable_symbol_get_info(sym, HSA_EXECUTABLE_SYMBOL_INFO_NAME, &name[0]);
  if (name.size() > 3 && name.compare(name.size() - 3, 3, ".kd") == 0) name.resize(name.size() - 3);
  AqlKernel k;
  uint32_t priv = 0;
  hsa_executable_symbol_get_info(sym, HSA_EXECUTABLE_SYMBOL_INFO_KERNEL_OBJECT, &k.object);
  hsa_executable_symbol_get_info(sym, HSA_EXECUTABLE_SYMBOL_INFO_KERNEL_KERNARG_SEGMENT_SIZE, &k.kernarg_size);
  hsa_executable_symbol_get_info(sym, HSA_EXECUTABLE_SYMBOL_INFO_KERNEL_GROUP_SEGMENT_SIZE, &k.lds);
  hsa_executable_symbol_get_info(sym, HSA_EXECUTABLE_SYMBOL_INFO_KERNEL_PRIVATE_SEGMENT_SIZE, &priv);
  int status = 0;
  char* dem = abi::__cxa_demangle(name.c_str(), nullptr, nullptr, &status);
  std::string full = (status == 0 && dem) ? dem : name;
  std::free(dem);
  // "void daris::fc_kernel<false>(daris::FcArgs)" -> "daris::fc_kernel<false>"
  if (full.compare(0, 5, "void ") == 0) full.erase(0, 5);
  int depth = 0;
  size_t cut = full.size();
  for (size_t i = 0; i < full.size(); ++i) {
    if (full[i] == '<') ++depth;
    else if (full[i] == '>') --depth;
    else if (full[i] == '(' && depth == 0) {
      cut = i;
      break;
    }
  }
  full.resize(cut);
  if (priv != 0 && s->error.empty()) s->error = "kernel " + full + " needs scratch memory, which the dispatch path does not provide";
  (*s->out)[full] = k;
  return HSA_STATUS_SUCCESS;
}

}  // namespace

std::string AqlRuntime::init(int hip_device, const void* image, size_t bytes) {
  if (ready_) return "";
  hsa_status_t st = hsa_init();  // reference counted: HIP holds its own reference
  if (st != HSA_STATUS_SUCCESS) return hsa_err("hsa_init", st);
  AgentScan scan;
  st = hsa_iterate_agents(scan_agents, &scan);
  if (st != HSA_STATUS_SUCCESS || scan.gpus.empty() || !scan.have_cpu) {
    hsa_shut_down();
    return "no GPU / CPU agent found through HSA";
  }
  // the agent with the PCI address of HIP's device; enumeration order as the fallback
  int pick = hip_device < (int)scan.gpus.size() ? hip_device : -1;
  char bus[64] = {0};
  if (hipDeviceGetPCIBusId(bus, sizeof(bus), hip_device) == hipSuccess) {
    unsigned dom = 0, b = 0, d = 0, f = 0;
    if (std::sscanf(bus, "%x:%x:%x.%x", &dom, &b, &d, &f) == 4) {
      for (size_t i = 0; i < scan.gpus.size(); ++i) {
        uint32_t bdf = 0, domain = 0;
        hsa_agent_get_info(scan.gpus[i], (hsa_agent_info_t)HSA_AMD_AGENT_INFO_BDFID, &bdf);
        hsa_agent_get_info(scan.gpus[i], (hsa_agent_info_t)HSA_AMD_AGENT_INFO_DOMAIN, &domain);
        if (bdf == ((b << 8) | (d << 3) | f) && domain == dom) pick = (int)i;
      }
    }
  }
  if (pick < 0) {
    hsa_shut_down();
    return "HIP device " + std::to_string(hip_device) + " has no HSA agent";
  }
  gpu_ = scan.gpus[pick];
  cpu_ = scan.cpu;
  PoolScan ps;
  hsa_amd_agent_iterate_memory_pools(cpu_, scan_host_pools, &ps);
  if (!ps.found) {
    hsa_shut_down();
    return "no host memory pool for kernel arguments";
  }
  host_pool_ = ps.pool;
  uint64_t freq = 0;
  if (hsa_system_get_info(HSA_SYSTEM_INFO_TIMESTAMP_FREQUENCY, &freq) == HSA_STATUS_SUCCESS && freq > 0) ticks_per_us_ = (double)freq / 1e6;

  image_.assign((const char*)image, (const char*)image + bytes);
  if (image_.empty()) {
    hsa_shut_down();
    return "the library was built without its kernel code object";
  }
  st = hsa_code_object_reader_create_from_memory(image_.data(), image_.size(), &reader_);
  if (st == HSA_STATUS_SUCCESS) st = hsa_executable_create_alt(HSA_PROFILE_FULL, HSA_DEFAULT_FLOAT_ROUNDING_MODE_DEFAULT, nullptr, &exec_);
  if (st == HSA_STATUS_SUCCESS) st = hsa_executable_load_agent_code_object(exec_, gpu_, reader_, nullptr, nullptr);
  if (st == HSA_STATUS_SUCCESS) st = hsa_executable_freeze(exec_, nullptr);
  if (st != HSA_STATUS_SUCCESS) {
    hsa_shut_down();
    return hsa_err("loading the kernel code object", st);
  }
  SymbolScan ss{&kernels_, ""};
  hsa_executable_iterate_agent_symbols(exec_, gpu_, scan_symbols, &ss);
  if (!ss.error.empty() || kernels_.empty()) {
    std::string e = ss.error.empty() ? "the code object holds no kernels" : ss.error;
    hsa_executable_destroy(exec_);
    hsa_code_object_reader_destroy(reader_);
    kernels_.clear();
    hsa_shut_down();
    return e;
  }
  ready_ = true;
  return "";
}

void AqlRuntime::shutdown() {
  if (!ready_) return;
  hsa_executable_destroy(exec_);
  hsa_code_object_reader_destroy(reader_);
  kernels_.clear();
  image_.clear();
  ready_ = false;
  hsa_shut_down();
}

const AqlKernel* AqlRuntime::kernel(const std::string& name) const {
  auto it = kernels_.find(name);
  return it == kernels_.end() ? nullptr : &it->second;
}

void* AqlRuntime::alloc_host_coherent(size_t bytes) {
  void* p = nullptr;
  if (hsa_amd_memory_pool_allocate(host_pool_, bytes, 0, &p) != HSA_STATUS_SUCCESS) return nullptr;
  if (hsa_amd_agents_allow_access(1, &gpu_, nullptr, p) != HSA_STATUS_SUCCESS) {
    hsa_amd_memory_pool_free(p);
    return nullptr;
  }
  return p;
}

void AqlRuntime::free_mem(void* p) {
  if (p) hsa_amd_memory_pool_free(p);
}

hsa_signal_t AqlRuntime::new_signal(int64_t initial) {
  hsa_signal_t s{0};
  if (hsa_signal_create(initial, 0, nullptr, &s) != HSA_STATUS_SUCCESS) s.handle = 0;
  return s;
}

void AqlRuntime::free_signal(hsa_signal_t s) {
  if (s.handle) hsa_signal_destroy(s);
}

bool AqlRuntime::dispatch_time_us(hsa_signal_t s, double* start_us, double* end_us) const {
  hsa_amd_profiling_dispatch_time_t t{};
  if (hsa_amd_profiling_get_dispatch_time(gpu_, s, &t) != HSA_STATUS_SUCCESS) return false;
  *start_us = (double)t.start / ticks_per_us_;
  *end_us = (double)t.end / ticks_per_us_;
  return true;
}

void AqlQueue::on_error(hsa_status_t, hsa_queue_t*, void* data) {
  // called by the runtime's own thread when the queue goes inactive (a fault in a kernel, a malformed packet)
  static_cast<AqlQueue*>(data)->dead_.store(true, std::memory_order_release);
}

bool AqlQueue::drain(hsa_signal_t s, int64_t limit_ns) {
  if (!q_ || !s.handle) return false;
  bool ok = false;
  const int64_t saved = aql_wait_limit_ns();
  aql_set_wait_limit_ns(limit_ns);
  const uint64_t idx = dead() ? kNoSlot : claim_slot();
  if (idx != kNoSlot) {
    hsa_barrier_and_packet_t* p = (hsa_barrier_and_packet_t*)q_->base_address + (idx & (q_->size - 1));
    p->reserved0 = 0;
    p->reserved1 = 0;
    for (int i = 0; i < 5; ++i) p->dep_signal[i] = hsa_signal_t{0};
    p->reserved2 = 0;
    p->completion_signal = s;
    const uint16_t header = (uint16_t)((HSA_PACKET_TYPE_BARRIER_AND << HSA_PACKET_HEADER_TYPE) | (1u << HSA_PACKET_HEADER_BARRIER) |
                                       (HSA_FENCE_SCOPE_SYSTEM << HSA_PACKET_HEADER_SCACQUIRE_FENCE_SCOPE) |
                                       (HSA_FENCE_SCOPE_SYSTEM << HSA_PACKET_HEADER_SCRELEASE_FENCE_SCOPE));
    __atomic_store_n((uint16_t*)p, header, __ATOMIC_RELEASE);
    hsa_signal_store_screlease(q_->doorbell_signal, (hsa_signal_value_t)idx);
    ok = aql_spin(s, this);
  }
  aql_set_wait_limit_ns(saved);
  if (ok) hsa_signal_destroy(s);  // a signal the GPU may still write is left alone
  return ok;
}

std::string AqlQueue::create(AqlRuntime* rt, const uint32_t mask[8]) {
  rt_ = rt;
  dead_.store(false);
  hsa_status_t st = hsa_queue_create(rt->gpu(), kSlots, HSA_QUEUE_TYPE_SINGLE, &AqlQueue::on_error, this, UINT32_MAX, UINT32_MAX, &q_);
  if (st != HSA_STATUS_SUCCESS) {
    q_ = nullptr;
    return hsa_err("hsa_queue_create", st);
  }
  if (q_->size > kSlots) {  // the argument ring has one slot per packet slot
    destroy();
    return "the queue is larger than asked for";
  }
  st = hsa_amd_queue_cu_set_mask(q_, 256, mask);
  if (st != HSA_STATUS_SUCCESS && st != (hsa_status_t)HSA_STATUS_CU_MASK_REDUCED) {
    destroy();
    return hsa_err("hsa_amd_queue_cu_set_mask", st);
  }
  ring_ = (char*)rt->alloc_host_coherent((size_t)kSlots * kSlotBytes);
  if (!ring_) {
    destroy();
    return "argument ring allocation failed";
  }
  return "";
}

void AqlQueue::destroy() {
  if (q_) hsa_queue_destroy(q_);
  q_ = nullptr;
  if (ring_ && rt_) rt_->free_mem(ring_);
  ring_ = nullptr;
}

void AqlQueue::set_profiling(bool on) {
  if (q_) hsa_amd_profiling_set_profiler_enabled(q_, on ? 1 : 0);
}

void AqlQueue::write_packet(uint64_t idx, const AqlKernel& k, uint32_t groups, uint32_t threads, const void* kernarg, hsa_signal_t completion,
                            unsigned flags) {
  hsa_kernel_dispatch_packet_t* p = (hsa_kernel_dispatch_packet_t*)q_->base_address + (idx & (q_->size - 1));
  p->setup = 1;  // one grid dimension
  p->workgroup_size_x = (uint16_t)threads;
  p->workgroup_size_y = 1;
  p->workgroup_size_z = 1;
  p->reserved0 = 0;
  p->grid_size_x = groups * threads;
  p->grid_size_y = 1;
  p->grid_size_z = 1;
  p->private_segment_size = 0;
  p->group_segment_size = k.lds;
  p->kernel_object = k.object;
  p->kernarg_address = const_cast<void*>(kernarg);
  p->reserved2 = 0;
  p->completion_signal = completion;
  // in order (barrier bit); acquire: what earlier packets wrote is visible to this kernel; release: what it writes is
  // visible to the next packet of any queue of the device, or (system scope) to the host as well
  const unsigned acq = (flags & kAcquireSystem) ? HSA_FENCE_SCOPE_SYSTEM : HSA_FENCE_SCOPE_AGENT;
  const unsigned rel = (flags & kReleaseSystem) ? HSA_FENCE_SCOPE_SYSTEM : HSA_FENCE_SCOPE_AGENT;
  const uint16_t header = (uint16_t)((HSA_PACKET_TYPE_KERNEL_DISPATCH << HSA_PACKET_HEADER_TYPE) | (1u << HSA_PACKET_HEADER_BARRIER) |
                                     (acq << HSA_PACKET_HEADER_SCACQUIRE_FENCE_SCOPE) | (rel << HSA_PACKET_HEADER_SCRELEASE_FENCE_SCOPE));
  __atomic_store_n((uint16_t*)p, header, __ATOMIC_RELEASE);
  hsa_signal_store_screlease(q_->doorbell_signal, (hsa_signal_value_t)idx);
}

// Next packet index.  Waits while the ring is full but for one slot, so that the packet which used this slot (and its
// argument slot) before has not only been fetched but, the queue being in order, has completed.
uint64_t AqlQueue::claim_slot() {
  // one producer at a time, so the index can be read first and taken only once there is room
  const uint64_t idx = hsa_queue_load_write_index_relaxed(q_);
  if (idx - hsa_queue_load_read_index_scacquire(q_) >= q_->size - 1) {
    const auto t0 = std::chrono::steady_clock::now();
    const int64_t limit = aql_wait_limit_ns();
    for (uint32_t spins = 0; idx - hsa_queue_load_read_index_scacquire(q_) >= q_->size - 1; ++spins) {
      if (dead()) return kNoSlot;
      if ((spins & 1023u) == 1023u &&
          std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0).count() > limit)
        return kNoSlot;
      __builtin_ia32_pause();
    }
  }
  hsa_queue_store_write_index_relaxed(q_, idx + 1);
  return idx;
}

bool AqlQueue::dispatch(const AqlKernel& k, uint32_t groups, uint32_t threads, const void* kernarg, hsa_signal_t completion, unsigned flags) {
  if (!q_ || dead() || !kernarg || groups == 0 || threads == 0 || threads > 1024 || (uint64_t)groups * threads > 0xffffffffull) return false;
  const uint64_t idx = claim_slot();
  if (idx == kNoSlot) return false;
  write_packet(idx, k, groups, threads, kernarg, completion, flags);
  return true;
}

bool AqlQueue::dispatch_copy(const AqlKernel& k, uint32_t groups, uint32_t threads, const void* args, uint32_t bytes, hsa_signal_t completion,
                             unsigned flags) {
  if (!q_ || dead() || bytes != k.kernarg_size || bytes > kSlotBytes || groups == 0 || threads == 0 || threads > 1024 ||
      (uint64_t)groups * threads > 0xffffffffull)
    return false;
  const uint64_t idx = claim_slot();
  if (idx == kNoSlot) return false;
  char* slot = ring_ + (size_t)(idx & (kSlots - 1)) * kSlotBytes;
  std::memcpy(slot, args, bytes);
  write_packet(idx, k, groups, threads, slot, completion, flags);
  return true;
}

namespace {
std::atomic<int64_t> g_wait_limit_ns{20ll * 1000 * 1000 * 1000};  // 20 s: far above any stage of the configured networks
}

void aql_set_wait_limit_ns(int64_t ns) { g_wait_limit_ns.store(ns < 1 ? 1 : ns, std::memory_order_relaxed); }
int64_t aql_wait_limit_ns() { return g_wait_limit_ns.load(std::memory_order_relaxed); }

bool aql_spin(hsa_signal_t s, const AqlQueue* q, const std::atomic<bool>* stop) {
  if (aql_done(s)) return true;
  const auto t0 = std::chrono::steady_clock::now();
  const int64_t limit = aql_wait_limit_ns();
  for (uint32_t spins = 0;; ++spins) {
    for (int i = 0; i < 8; ++i) __builtin_ia32_pause();
    if (aql_done(s)) return true;
    if ((spins & 255u) == 255u) {  // the clock and the flags every ~10 us only: the common case is a wait of microseconds
      if (q && q->dead()) return false;
      if (stop && stop->load(std::memory_order_relaxed)) return false;
      if (std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0).count() > limit) return aql_done(s);
    }
  }
}

bool aql_wait(hsa_signal_t s, const AqlQueue* q) {
  if (!aql_spin(s, q)) return false;
  hsa_signal_store_relaxed(s, 1);
  return true;
}

}  // namespace daris
