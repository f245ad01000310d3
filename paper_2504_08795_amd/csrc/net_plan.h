// Host-side plan of one task's DNN: tensor shapes, buffer slots, legal stage cuts, the MAC-balanced stage split
// (Sec. III-B1), weight packing for the HIP kernels, and the per-stage launch sequence.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/daris.h"
#include "kernels.h"

namespace daris {

struct TensorInfo {
  int C = 0, Cs = 0, H = 0, W = 0;  // logical channels, channel stride (padded), spatial size
  int slot = -1;                    // activation buffer slot, -1 = none (written straight to the caller's logits)
  size_t bytes = 0;
};

struct LayerPlan {
  daris_layer d;  // descriptor with the host pointers cleared
  TensorInfo out;
  int in_t = 0, res_t = -1;  // tensor indices: 0 = ingested network input, l + 1 = output of layer l
  int64_t macs = 0;
  bool depthwise = false;
  int K = 0, Kpad = 0;       // GEMM K (conv: kh*kw*Cs_in, fc: H*W*Cs_in) and its zero-padded length
  ConvPlan cp;
  // Two dense convolutions that read the same tensor and do not depend on each other share one launch: it is issued
  // at the later layer (pair_lead), the earlier one issues nothing; the lighter of the two is planned like the heavier.
  int pair_with = -1;
  bool pair_lead = false;
  // A 3x3 depthwise convolution whose only reader is the 1x1 convolution right after it is computed inside that
  // convolution's launch and never stored: the two layers are linked like a launch pair (the depthwise layer issues
  // nothing, the 1x1 convolution leads) and both carry this mark.
  bool fused_dw = false;
  bool fusable_dw = false;  // the plan allows it; fused_dw is switched off while a stage cut separates the two layers
  int32_t kernel_id = K_NONE;
  void* w_dev = nullptr;
  float* b_dev = nullptr;
};

struct NetPlan {
  int bf16 = 0;
  int in_c = 0, in_h = 0, in_w = 0;
  TensorInfo ingest;              // tensor 0
  std::vector<LayerPlan> layers;
  std::vector<size_t> slot_bytes; // activation slots after liveness-based reuse
  size_t ws_bytes = 0;            // split-K workspace
  std::vector<int> legal_cuts;    // l such that a cut after layer l is legal
  std::vector<int> stage_first;   // first layer of each stage (size = number of stages)
  int n_out = 0;                  // elements of the final output (C*H*W)
  bool final_direct = false;      // last layer is an FC writing fp32 logits itself
  bool fuse_ingest = false;       // layer 0 reads the caller's fp32 [C][H][W] input itself: no layout conversion launch

  const TensorInfo& tensor(int t) const { return t == 0 ? ingest : layers[t - 1].out; }
};

// Builds shapes, MACs, legal cuts, buffer slots and kernel plans.  pair_launches: two independent convolutions on one
// tensor share a launch; fuse_ingest: the first convolution may read the caller's input layout itself; staged_rows:
// convolutions whose pixels are whole 64-byte rows fetch them coalesced through LDS; small_tiles: deep, skinny layers
// get 16-pixel tiles instead of a K split across workgroups; fuse_dw: a depthwise convolution is computed inside the 1x1
// convolution that alone reads it.  Returns "" or an error text.
// plan_cus: the partition size the convolution grids are balanced for.
std::string build_plan(const daris_dnn& dnn, bool keep_activations, bool pair_launches, bool fuse_ingest, bool staged_rows, bool small_tiles, bool fuse_dw,
                       int plan_cus, NetPlan* out);
// Chooses k - 1 cuts minimising the largest per-stage MAC count, ties to the lexicographically smallest cut
// list.  Returns false when k exceeds the number of legal cuts + 1.
bool split_stages(NetPlan* net, int k);

// Weight packing (host): results are byte buffers in the device layouts of kernels.h.
void pack_conv(const NetPlan& net, const LayerPlan& L, const float* w, const float* b, std::vector<unsigned char>* wp,
               std::vector<float>* bp);
void pack_fc(const NetPlan& net, const LayerPlan& L, const float* w, const float* b, std::vector<unsigned char>* wp,
             std::vector<float>* bp);
uint16_t host_f32_to_bf16(float f);

}  // namespace daris
