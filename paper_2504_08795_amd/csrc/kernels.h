// Launch interface between the host runtime and the HIP kernels (gfx950 only).
//
// Device tensor format: NHWC, element type float (fp32 tasks) or bfloat16 stored as uint16 (bf16 tasks),
// channel stride Cs = channel count rounded up to one 16-byte vector (4 floats / 8 bf16); pad channels hold 0.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace daris {

enum KernelId : int32_t {
  K_NONE = 0,
  // wave-tile implicit GEMM: TN 32-channel blocks per wave, NW waves splitting K inside the workgroup
  K_CONVW_F32_T1W2, K_CONVW_F32_T1W4, K_CONVW_F32_T1W8, K_CONVW_F32_T2W2, K_CONVW_F32_T2W4, K_CONVW_F32_T2W8,
  K_CONVW_BF16_T1W2, K_CONVW_BF16_T1W4, K_CONVW_BF16_T1W8, K_CONVW_BF16_T2W2, K_CONVW_BF16_T2W4, K_CONVW_BF16_T2W8,
  K_SPLITK_REDUCE, K_DWCONV, K_MAXPOOL, K_GAVGPOOL, K_FC, K_INGEST, K_EGRESS,
  K_COUNT
};
const char* kernel_name(int32_t id);

struct ConvArgs {
  const void* x;      // [H][W][Cin]; with c_real > 0: the network input as the caller gives it, float [c_real][H][W]
  const void* w;      // packed weights in MFMA fragment order (see pack_conv)
  const float* bias;  // [Cout]
  const void* res;    // [Ho*Wo][Cout] or nullptr
  void* y;            // [Ho*Wo][Cout]
  float* ws;          // split-K partial sums (splitk > 1)
  int H, W, Cin, Ho, Wo, Cout;
  int kh, kw, stride, pad;
  int K, Kpad, M;
  int act;
  int splitk;  // grid.z
  int S, sz, sw;  // K steps in total, per K slice of a workgroup, per wave
  uint32_t mg_wo, mg_cin, mg_kw;  // multipliers for division by Wo, Cin, kw (see div_magic)
  int MT, NTn, G, xmode;  // pixel tiles, channel tiles, weight groups (= NTn * splitk), XCD mapping mode
  int c_real;             // > 0: layer 0 reads the fp32 [C][H][W] network input directly (Cin == one 16-byte vector, c_real <= 4)
  int wave_prio;          // 1: the waves raise their issue priority (stages of high-priority tasks on shared CUs)
};

struct DwArgs {
  const void* x;      // [H][W][C]
  const void* w;      // [k*k][C]
  const float* bias;  // [C]
  void* y;            // [Ho][Wo][C]
  int H, W, C, Ho, Wo, k, stride, pad, act;
};

struct PoolArgs {
  const void* x;
  void* y;
  int H, W, C, Ho, Wo, k, stride, pad;
};

struct FcArgs {
  const void* x;      // [K]
  const void* w;      // [N][K]
  const float* bias;  // [N]
  void* y;            // [Ns], element type of the task, or float when out_f32; outputs N..Ns-1 are written as 0
  int K, N, Ns, act, out_f32;
};

// Kernel and tile configuration chosen on the host for one dense convolution.
struct ConvPlan {
  int32_t kernel;  // KernelId
  int splitk;      // K slices across workgroups (1 = none); > 1 needs the workspace and the reduction launch
  int tn, nw, S, sz, sw, MT, NTn, G, xmode;
  int tiles;                       // output tiles per grid.z slice
  size_t ws_bytes;                 // split-K workspace this launch needs
  dim3 grid;
  int threads;
};
// bf16 = 0/1.  Chooses tile shape, waves per workgroup and split-K from (M, N, Kpad) only, so results do not depend on the
// partition a stage runs in.
ConvPlan plan_conv(int M, int N, int Kpad, int bf16);

// If t0/t1 are given they are recorded on `s` immediately before and after the main kernel (not the split-K reduce).
hipError_t launch_conv(const ConvPlan& pl, const ConvArgs& a, int bf16, hipStream_t s, hipEvent_t t0 = nullptr, hipEvent_t t1 = nullptr);
// Plan for a second convolution that is to share a launch with `first` (launch_conv_pair): the same wave-tile kernel
// variant, K not split across workgroups.  Returns a plan with kernel == K_NONE when that is not possible.
ConvPlan plan_conv_like(const ConvPlan& first, int M, int N, int Kpad, int bf16);
// One launch for two independent convolutions: pl0/a0 as planned by plan_conv, pl1/a1 by
// plan_conv_like(pl0, ...).  The event pair brackets the joint kernel.
hipError_t launch_conv_pair(const ConvPlan& pl0, const ConvArgs& a0, const ConvPlan& pl1, const ConvArgs& a1, int bf16, hipStream_t s,
                            hipEvent_t t0 = nullptr, hipEvent_t t1 = nullptr);
// Multiplier for fast_div: floor(2^32 / d) + 1, or 0 for d == 1.  Exact for every n >= 0 with n * d < 2^32.
inline uint32_t div_magic(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((1ull << 32) / d) + 1u; }

hipError_t launch_dwconv(const DwArgs& a, int bf16, hipStream_t s);
hipError_t launch_maxpool(const PoolArgs& a, int bf16, hipStream_t s);
hipError_t launch_gavgpool(const PoolArgs& a, int bf16, hipStream_t s);
hipError_t launch_fc(const FcArgs& a, int bf16, hipStream_t s);
// x: float [C][H][W] -> y: [H][W][Cs]
hipError_t launch_ingest(const float* x, void* y, int C, int Cs, int H, int W, int bf16, hipStream_t s);
// x: [H][W][Cs] -> y: float [C][H][W]
hipError_t launch_egress(const void* x, float* y, int C, int Cs, int H, int W, int bf16, hipStream_t s);
// Records, per workgroup, the XCC id and the hardware id register of the CU it ran on (mask probing).
hipError_t launch_cu_probe(uint32_t* out, int n_groups, int spin, hipStream_t s);

}  // namespace daris
