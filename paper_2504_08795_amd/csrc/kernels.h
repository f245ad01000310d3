// Interface between the host runtime and the HIP kernels (gfx950 only): argument structures shared by both sides,
// the host-side launch plans, and the encoders that turn a layer into ready-to-dispatch AQL launches.
//
// Device tensor format: NHWC, element type float (fp32 tasks) or bfloat16 stored as uint16 (bf16 tasks),
// channel stride Cs = channel count rounded up to one 16-byte vector (4 floats / 8 bf16); pad channels hold 0.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

namespace daris {

enum KernelId : int32_t {
  K_NONE = 0,
  // wave-tile implicit GEMM: TN 32-channel blocks per wave, NW waves splitting K inside the workgroup
  K_CONVW_F32_T1W2, K_CONVW_F32_T1W4, K_CONVW_F32_T1W8, K_CONVW_F32_T2W2, K_CONVW_F32_T2W4, K_CONVW_F32_T2W8,
  K_CONVW_BF16_T1W2, K_CONVW_BF16_T1W4, K_CONVW_BF16_T1W8, K_CONVW_BF16_T2W2, K_CONVW_BF16_T2W4, K_CONVW_BF16_T2W8,
  // the same with 16-pixel tiles of TN 16-channel blocks (deep, skinny layers)
  K_CONV16_F32_T1W2, K_CONV16_F32_T1W4, K_CONV16_F32_T1W8, K_CONV16_F32_T2W2, K_CONV16_F32_T2W4, K_CONV16_F32_T2W8,
  K_CONV16_BF16_T1W2, K_CONV16_BF16_T1W4, K_CONV16_BF16_T1W8, K_CONV16_BF16_T2W2, K_CONV16_BF16_T2W4, K_CONV16_BF16_T2W8,
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

// The 3x3 depthwise convolution (pad 1) that conv_wave_dw_kernel computes on the fly in front of a 1x1 convolution; the
// ConvArgs beside it describe that 1x1 convolution, except that ConvArgs::x is the DEPTHWISE layer's input tensor
// [H][W][Cin] (ConvArgs::H, W stay the 1x1 convolution's own input size = the depthwise layer's output size).
struct DwFusedArgs {
  const void* w = nullptr;      // [9][C]
  const float* bias = nullptr;  // [C]
  int H = 0, W = 0;             // the depthwise layer's input size
  int stride = 1, act = 0;
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
  int rows;                        // pixels per wave tile: 32 (conv_wave_*: channel blocks of 32) or 16 (conv_wave16_*: blocks of 16)
  int tn, nw, S, sz, sw, MT, NTn, G, xmode;
  int step_align;                  // K slices are multiples of this many steps (2: staged pixel operand possible)
  int tiles;                       // output tiles per grid.z slice
  size_t ws_bytes;                 // split-K workspace this launch needs
  uint32_t grid_x;                 // workgroups of the launch
  int threads;
};
// True when every pixel's channel vector is a whole number of 64-byte rows, the shape for which the convolution kernel
// fetches the pixel operand in coalesced rows through LDS (chunks of two K steps).
inline bool conv_rows_staged(int cin_stride, int bf16) { return cin_stride > 0 && (cin_stride * (bf16 ? 2 : 4)) % 64 == 0; }
// bf16 = 0/1.  Chooses tile shape, waves per workgroup and split-K from (M, N, Kpad) and the nominal partition size
// (nominal_cus: how many CUs the grid is balanced for) only, so results do not depend on the partition a stage runs in.  step_align = 2 cuts K in whole chunks of two steps (for conv_rows_staged shapes), else 1.
// cin_stride = the input tensor's channel stride: when it is a whole number of the 16-row kernel's K steps and the 32-row
// plan would split K across workgroups, a 16-row plan that does not need to is chosen instead (cin_stride 0: never).
ConvPlan plan_conv(int M, int N, int Kpad, int bf16, int step_align, int cin_stride = 0, int nominal_cus = 128);
// Plan for a second convolution that is to share a launch with `first`: the same wave-tile kernel variant, K not split
// across workgroups.  Returns a plan with kernel == K_NONE when that is not possible.
ConvPlan plan_conv_like(const ConvPlan& first, int M, int N, int Kpad, int bf16, int step_align, int nominal_cus = 128);
// Multiplier for fast_div: floor(2^32 / d) + 1, or 0 for d == 1.  Exact for every n >= 0 with n * d < 2^32.
inline uint32_t div_magic(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((1ull << 32) / d) + 1u; }

// ---- launches ------------------------------------------------------------------------------------------------------------
//
// The kernels are dispatched by AQL packets written by the library itself (aql.h).  An encoder turns the arguments of
// a layer into one or two Launch records: kernel, geometry and the exact argument bytes the kernel expects.

struct AqlKernel;
class AqlRuntime;

struct KernelLaunch {
  const AqlKernel* k = nullptr;
  uint32_t groups = 0, threads = 0;  // workgroups, threads per workgroup
  uint32_t nbytes = 0;               // bytes of args in use
  int32_t kernel_id = K_NONE;
  alignas(8) unsigned char args[336];
};

// Every kernel of the code object, looked up once.
struct KernelTable {
  const AqlKernel* conv[2][6][4] = {};  // [bf16][(tn - 1) * 3 + log2(nw) - 1][gather mode 0..3]
  const AqlKernel* pair[2][6][3] = {};  // gather modes 0, 1, 3
  const AqlKernel* conv16[2][6] = {};   // 16-row tiles: [bf16][(tn - 1) * 3 + log2(nw) - 1]
  const AqlKernel* pair16[2][6] = {};
  const AqlKernel* convdw[2][6] = {};   // 1x1 convolution with a fused depthwise producer (fp32: tn = 1 only)
  const AqlKernel *reduce[2] = {}, *dwconv[2] = {}, *maxpool[2] = {}, *gavgpool[2] = {}, *fc[2] = {}, *ingest[2] = {}, *egress[2] = {};
  const AqlKernel* cu_probe = nullptr;
  // "" or the name of the first kernel that is missing or whose argument size is not what this header declares
  std::string resolve(const AqlRuntime& rt);
};

// Dense convolution: the main kernel, then the split-K reduction if the plan has one.  False on an inconsistent plan.
bool encode_conv(const KernelTable& kt, const ConvPlan& pl, const ConvArgs& a, int bf16, std::vector<KernelLaunch>* out);
// Two independent convolutions in one launch: pl0/a0 as planned by plan_conv, pl1/a1 by plan_conv_like(pl0, ...).
bool encode_conv_pair(const KernelTable& kt, const ConvPlan& pl0, const ConvArgs& a0, const ConvPlan& pl1, const ConvArgs& a1, int bf16,
                      std::vector<KernelLaunch>* out);
// A depthwise 3x3 convolution (pad 1, stride d.stride) followed by the 1x1 convolution pl/a in one launch.  a.x must be the
// depthwise layer's input; the plan must be a staged 32-row one (conv_rows_staged shape, step_align 2).
bool encode_conv_dw(const KernelTable& kt, const ConvPlan& pl, const ConvArgs& a, const DwFusedArgs& d, int bf16, std::vector<KernelLaunch>* out);
// Whether a depthwise 3x3 layer in front of the 1x1 convolution planned as pl should be computed inside that convolution's
// launch.  Measured on MobileNetV2's blocks: the producer re-reads the depthwise input up to nine times through one CU's
// vector cache and pays a memory latency per chunk of 64 bytes of channels, so it wins only where the convolution has enough
// workgroups to fill a partition and a single channel block (no repetition per block, few chunks per wave); elsewhere the
// separate, fully parallel depthwise launch is faster (by 1.3 to 5 us per block).
bool conv_dw_fusable(const ConvPlan& pl, int bf16);
bool encode_dwconv(const KernelTable& kt, const DwArgs& a, int bf16, std::vector<KernelLaunch>* out);
bool encode_maxpool(const KernelTable& kt, const PoolArgs& a, int bf16, std::vector<KernelLaunch>* out);
bool encode_gavgpool(const KernelTable& kt, const PoolArgs& a, int bf16, std::vector<KernelLaunch>* out);
bool encode_fc(const KernelTable& kt, const FcArgs& a, int bf16, std::vector<KernelLaunch>* out);
// x: float [C][H][W] -> y: [H][W][Cs]
bool encode_ingest(const KernelTable& kt, const float* x, void* y, int C, int Cs, int H, int W, int bf16, std::vector<KernelLaunch>* out);
// x: [H][W][Cs] -> y: float [C][H][W]
bool encode_egress(const KernelTable& kt, const void* x, float* y, int C, int Cs, int H, int W, int bf16, std::vector<KernelLaunch>* out);
// Records, per workgroup, the XCC id and the hardware id register of the CU it ran on (mask probing).
bool encode_cu_probe(const KernelTable& kt, uint32_t* out_dev, int n_groups, int spin, std::vector<KernelLaunch>* out);

// Byte offsets inside a launch's argument block of the pointers that change from job to job.
constexpr uint32_t kConvInputOffset = 0;     // ConvArgs::x (layer 0 gathering from the job's input)
constexpr uint32_t kIngestInputOffset = 0;   // ingest: x
constexpr uint32_t kFcOutputOffset = 24;     // FcArgs::y
constexpr uint32_t kEgressOutputOffset = 8;  // egress: y

}  // namespace daris
