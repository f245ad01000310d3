// Direct AQL dispatch: the library's kernels are launched by writing dispatch packets into its own HSA queues
// instead of going through the HIP launch path.
//
// Why: a DNN stage at batch 1 is a chain of kernels of a few microseconds each.  Measured on MI355X with 15 trivial
// kernels of 160-byte arguments on a CU-masked queue: HIP launches cost 4.2 us of host time each and the chain is done
// after 85 us; packets written directly (arguments in device memory) cost 0.3 us each and the chain is done after
// 28 us, with agent-scope acquire and release on every packet.  The stage boundary (the synchronisation point of
// Sec. III-B1) becomes a poll of the completion signal's memory word.
//
// One AqlQueue = one user-mode hardware queue restricted to a compute-unit mask (a stream of a partition,
// Sec. III-C), in order (every packet carries the barrier bit).  Argument blocks live in device memory and are
// written once, at registration, by an ordinary device copy: a launch writes 64 bytes of packet and rings the doorbell.
#pragma once
#include <hsa/hsa.h>
#include <hsa/hsa_ext_amd.h>

#include <atomic>
#include <cstdint>
#include <string>
#include <unordered_map>
#include <vector>

namespace daris {

struct AqlKernel {
  uint64_t object = 0;        // kernel descriptor address
  uint32_t kernarg_size = 0;  // bytes of explicit arguments (the kernels use no hidden arguments)
  uint32_t lds = 0;           // static LDS bytes per workgroup
};

// Process-wide state: HSA agents and memory pools, the loaded code object and its kernels.
class AqlRuntime {
 public:
  // Attaches to the GPU that HIP calls `hip_device` and loads the code object image.  Returns "" or an error text.
  std::string init(int hip_device, const void* image, size_t bytes);
  void shutdown();
  bool ready() const { return ready_; }

  // Kernel by demangled name without return type and parameter list, e.g. "daris::fc_kernel<false>".
  const AqlKernel* kernel(const std::string& name) const;

  hsa_agent_t gpu() const { return gpu_; }
  // Host memory the GPU reads coherently (argument rings of dispatch_copy).
  void* alloc_host_coherent(size_t bytes);
  void free_mem(void* p);
  hsa_signal_t new_signal(int64_t initial);
  void free_signal(hsa_signal_t s);
  // Start and end of the dispatch that decremented `s` (queue profiling must have been on), in microseconds of one clock.
  bool dispatch_time_us(hsa_signal_t s, double* start_us, double* end_us) const;

 private:
  bool ready_ = false;
  hsa_agent_t gpu_{}, cpu_{};
  hsa_amd_memory_pool_t host_pool_{};
  hsa_executable_t exec_{};
  hsa_code_object_reader_t reader_{};
  std::vector<char> image_;
  std::unordered_map<std::string, AqlKernel> kernels_;
  double ticks_per_us_ = 100.0;
};

class AqlQueue {
 public:
  // Queue on rt's GPU limited to the compute units whose bits are set in mask (256 bits).  Returns "" or an error text.
  std::string create(AqlRuntime* rt, const uint32_t mask[8]);
  void destroy();
  bool valid() const { return q_ != nullptr; }
  // The runtime reported an error on this queue (its packet processor stopped): nothing queued on it will complete.
  bool dead() const { return dead_.load(std::memory_order_acquire); }
  // Appends a barrier packet that completes `s` (a fresh signal of value 1, destroyed here) once every earlier packet
  // has completed, and waits for it for at most limit_ns.  True when the queue ran dry in time.
  bool drain(hsa_signal_t s, int64_t limit_ns);

  enum : unsigned {
    kReleaseSystem = 1,  // when the kernel completes its writes are visible to the host too (default: to this device)
    kAcquireSystem = 2,  // the kernel sees what the host, copy engines and other devices wrote before (default: this device)
  };
  // Appends one kernel: `groups` workgroups of `threads` threads whose argument block already lies in device memory at
  // `kernarg` (written once at registration by a device copy; the host never writes it again).  The kernel starts
  // after every earlier packet of this queue has completed.  When it has completed, `completion` (if its handle is
  // not 0) is decremented.  One producer at a time.
  bool dispatch(const AqlKernel& k, uint32_t groups, uint32_t threads, const void* kernarg, hsa_signal_t completion = hsa_signal_t{0},
                unsigned flags = 0);
  // The same for arguments that exist only now (a caller's buffer address): they are copied into a ring of
  // host-coherent memory, which the kernel reads over the bus (slower for the kernel than device memory).  Returns
  // false if `bytes` is not what the kernel expects.
  bool dispatch_copy(const AqlKernel& k, uint32_t groups, uint32_t threads, const void* args, uint32_t bytes,
                     hsa_signal_t completion = hsa_signal_t{0}, unsigned flags = 0);
  // Time stamps for dispatches that carry a completion signal.
  void set_profiling(bool on);

 private:
  static constexpr uint32_t kSlots = 1024;     // packets in the ring = argument slots of dispatch_copy
  static constexpr uint32_t kSlotBytes = 384;  // >= the largest argument block (two convolution problems: 324)
  static void on_error(hsa_status_t status, hsa_queue_t* source, void* data);
  // Next packet index, or kNoSlot when the ring stayed full for the whole wait limit (or the queue is dead).
  static constexpr uint64_t kNoSlot = ~0ull;
  uint64_t claim_slot();
  void write_packet(uint64_t idx, const AqlKernel& k, uint32_t groups, uint32_t threads, const void* kernarg, hsa_signal_t completion,
                    unsigned flags);
  AqlRuntime* rt_ = nullptr;
  hsa_queue_t* q_ = nullptr;
  char* ring_ = nullptr;  // host-coherent argument slots
  std::atomic<bool> dead_{false};
};

// Every host wait for the GPU is bounded: a kernel that never completes (or a queue whose packet processor has stopped)
// must surface as an error code, not as a hung thread.  The limit is process-wide, in nanoseconds.
void aql_set_wait_limit_ns(int64_t ns);
int64_t aql_wait_limit_ns();
inline bool aql_done(hsa_signal_t s) { return hsa_signal_load_scacquire(s) == 0; }
// Spins until the signal reads 0 (its dispatch has completed).  False when the wait limit expired first, when `q` (may be
// null) reported an error, or when *stop (may be null) became true.
bool aql_spin(hsa_signal_t s, const AqlQueue* q = nullptr, const std::atomic<bool>* stop = nullptr);
// aql_spin, then re-arms the signal to 1 on success.
bool aql_wait(hsa_signal_t s, const AqlQueue* q = nullptr);

}  // namespace daris
