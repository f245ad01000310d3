#include "net_plan.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <limits>

namespace daris {

static inline int round_up(int a, int b) { return (a + b - 1) / b * b; }

uint16_t host_f32_to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                           // nearest, ties to even
  return (uint16_t)(u >> 16);
}

std::string build_plan(const daris_dnn& dnn, bool keep_activations, bool pair_launches, bool fuse_ingest, bool staged_rows, bool small_tiles, bool fuse_dw,
                       int plan_cus, NetPlan* out) {
  NetPlan& net = *out;
  net = NetPlan();
  if (dnn.n_layers < 1 || !dnn.layers) return "DNN has no layers";
  if (dnn.in_c < 1 || dnn.in_h < 1 || dnn.in_w < 1) return "bad input shape";
  if (dnn.dtype != DARIS_FP32 && dnn.dtype != DARIS_BF16) return "bad dtype";
  net.bf16 = dnn.dtype == DARIS_BF16;
  const int vec = net.bf16 ? 8 : 4, es = net.bf16 ? 2 : 4;
  net.in_c = dnn.in_c;
  net.in_h = dnn.in_h;
  net.in_w = dnn.in_w;
  net.ingest.C = dnn.in_c;
  net.ingest.Cs = round_up(dnn.in_c, vec);
  net.ingest.H = dnn.in_h;
  net.ingest.W = dnn.in_w;
  net.ingest.bytes = (size_t)net.ingest.H * net.ingest.W * net.ingest.Cs * es;
  const int n = dnn.n_layers;
  net.layers.resize(n);

  for (int l = 0; l < n; ++l) {
    LayerPlan& L = net.layers[l];
    L.d = dnn.layers[l];
    L.d.w = nullptr;
    L.d.b = nullptr;
    const daris_layer& d = L.d;
    if (d.in_from < -1 || d.in_from >= l) return "layer " + std::to_string(l) + ": in_from must name an earlier layer or -1";
    if (d.res_from < -1 || d.res_from >= l) return "layer " + std::to_string(l) + ": res_from must name an earlier layer or -1";
    L.in_t = d.in_from + 1;
    L.res_t = d.res_from < 0 ? -1 : d.res_from + 1;
    const TensorInfo& in = net.tensor(L.in_t);
    TensorInfo& o = L.out;
    switch (d.op) {
      case DARIS_OP_CONV: {
        if (d.c_in != in.C) return "layer " + std::to_string(l) + ": c_in does not match its input";
        if (d.k < 1 || d.stride < 1 || d.pad < 0 || d.c_out < 1) return "layer " + std::to_string(l) + ": bad conv geometry";
        L.depthwise = d.groups != 1;
        if (L.depthwise && !(d.groups == d.c_in && d.c_in == d.c_out))
          return "layer " + std::to_string(l) + ": only dense (groups=1) and depthwise (groups=c_in=c_out) convolutions";
        o.C = d.c_out;
        o.Cs = round_up(d.c_out, vec);
        o.H = (in.H + 2 * d.pad - d.k) / d.stride + 1;
        o.W = (in.W + 2 * d.pad - d.k) / d.stride + 1;
        if (o.H < 1 || o.W < 1) return "layer " + std::to_string(l) + ": empty output";
        L.macs = (int64_t)o.H * o.W * d.c_out * (d.c_in / d.groups) * d.k * d.k;
        if (!L.depthwise) {
          L.K = d.k * d.k * in.Cs;
          L.Kpad = round_up(L.K, 2 * vec);  // whole K steps of the convolution kernel (two 16-byte vectors per pixel)
          // the kernels divide pixel and k indices by Wo, Cin and kw with 32-bit multipliers: operands must stay small
          if ((uint64_t)(o.H * (uint64_t)o.W + 64) * (uint64_t)o.W >= (1ull << 32) || (uint64_t)(L.Kpad + 64) * (uint64_t)in.Cs >= (1ull << 32))
            return "layer " + std::to_string(l) + ": tensor too large for the kernels' index arithmetic";
          L.cp = plan_conv(o.H * o.W, o.Cs, L.Kpad, net.bf16, staged_rows && conv_rows_staged(in.Cs, net.bf16) ? 2 : 1, small_tiles ? in.Cs : 0, plan_cus);
          L.kernel_id = L.cp.kernel;
          net.ws_bytes = std::max(net.ws_bytes, L.cp.ws_bytes);
        } else {
          L.kernel_id = K_DWCONV;
        }
        break;
      }
      case DARIS_OP_MAXPOOL:
        if (d.k < 1 || d.stride < 1 || d.pad < 0 || 2 * d.pad > d.k) return "layer " + std::to_string(l) + ": bad pool geometry";
        o.C = in.C;
        o.Cs = in.Cs;
        o.H = (in.H + 2 * d.pad - d.k) / d.stride + 1;
        o.W = (in.W + 2 * d.pad - d.k) / d.stride + 1;
        if (o.H < 1 || o.W < 1) return "layer " + std::to_string(l) + ": empty output";
        L.kernel_id = K_MAXPOOL;
        break;
      case DARIS_OP_GAVGPOOL:
        o.C = in.C;
        o.Cs = in.Cs;
        o.H = o.W = 1;
        L.kernel_id = K_GAVGPOOL;
        break;
      case DARIS_OP_FC:
        if (d.c_in != in.C * in.H * in.W) return "layer " + std::to_string(l) + ": FC c_in must equal C*H*W of its input";
        if (d.c_out < 1) return "layer " + std::to_string(l) + ": bad FC size";
        o.C = d.c_out;
        o.Cs = round_up(d.c_out, vec);
        o.H = o.W = 1;
        L.macs = (int64_t)d.c_in * d.c_out;
        L.K = in.H * in.W * in.Cs;
        L.Kpad = L.K;
        L.kernel_id = K_FC;
        break;
      default:
        return "layer " + std::to_string(l) + ": unknown op";
    }
    if (d.act < DARIS_ACT_NONE || d.act > DARIS_ACT_RELU6) return "layer " + std::to_string(l) + ": unknown activation";
    if (L.res_t >= 0) {
      const TensorInfo& r = net.tensor(L.res_t);
      if (d.op != DARIS_OP_CONV || L.depthwise) return "layer " + std::to_string(l) + ": residual only on dense convolutions";
      if (r.C != o.C || r.H != o.H || r.W != o.W) return "layer " + std::to_string(l) + ": residual shape mismatch";
    }
    o.bytes = (size_t)o.H * o.W * o.Cs * es;
  }
  // launch pairs (a residual block's first convolution and its shortcut convolution)
  for (int l = 0; l + 1 < n && pair_launches; ++l) {
    LayerPlan& A = net.layers[l];
    LayerPlan& B = net.layers[l + 1];
    if (A.d.op != DARIS_OP_CONV || B.d.op != DARIS_OP_CONV || A.depthwise || B.depthwise) continue;
    if (A.in_t != B.in_t || B.res_t == l + 1) continue;
    LayerPlan& heavy = A.macs > B.macs ? A : B;
    LayerPlan& light = A.macs > B.macs ? B : A;
    const ConvPlan like = plan_conv_like(heavy.cp, light.out.H * light.out.W, light.out.Cs, light.Kpad, net.bf16,
                                         staged_rows && conv_rows_staged(net.tensor(light.in_t).Cs, net.bf16) ? 2 : 1, plan_cus);
    if (like.kernel == K_NONE) continue;
    light.cp = like;
    light.kernel_id = like.kernel;
    A.pair_with = l + 1;
    B.pair_with = l;
    B.pair_lead = true;
    ++l;
  }
  // depthwise 3x3 + the 1x1 convolution that alone reads it: one launch, the depthwise output is never stored
  for (int l = 0; l + 1 < n && fuse_dw && staged_rows && !keep_activations; ++l) {
    LayerPlan& A = net.layers[l];
    LayerPlan& B = net.layers[l + 1];
    if (A.d.op != DARIS_OP_CONV || !A.depthwise || A.d.k != 3 || A.d.pad != 1 || (A.d.stride != 1 && A.d.stride != 2)) continue;
    if (B.d.op != DARIS_OP_CONV || B.depthwise || B.d.k != 1 || B.d.stride != 1 || B.d.pad != 0 || B.in_t != l + 1 || B.pair_with >= 0) continue;
    bool only_reader = true;
    for (int q = l + 2; q < n; ++q)
      if (net.layers[q].in_t == l + 1 || net.layers[q].res_t == l + 1) only_reader = false;
    if (!only_reader || !conv_rows_staged(A.out.Cs, net.bf16)) continue;
    ConvPlan cp = B.cp;
    if (cp.rows != 32) cp = plan_conv(B.out.H * B.out.W, B.out.Cs, B.Kpad, net.bf16, 2, 0, plan_cus);  // the fused producer exists for 32-pixel tiles
    if (!conv_dw_fusable(cp, net.bf16)) continue;  // the separate launch is faster (or no such kernel variant)
    B.cp = cp;
    B.kernel_id = cp.kernel;
    net.ws_bytes = std::max(net.ws_bytes, cp.ws_bytes);
    A.pair_with = l + 1;
    B.pair_with = l;
    B.pair_lead = true;
    A.fused_dw = B.fused_dw = true;
    A.fusable_dw = B.fusable_dw = true;
    ++l;
  }
  // Layer 0 can gather straight from the caller's input when that is its only reader and one filter tap is exactly
  // one 16-byte vector of the padded layout (1..4 real channels).
  {
    const LayerPlan& L0 = net.layers[0];
    bool only_reader = true;
    for (int l = 1; l < n; ++l)
      if (net.layers[l].in_t == 0 || net.layers[l].res_t == 0) only_reader = false;
    net.fuse_ingest = !keep_activations && fuse_ingest && L0.d.op == DARIS_OP_CONV && !L0.depthwise &&
                      L0.in_t == 0 && L0.res_t < 0 && L0.pair_with < 0 && only_reader && net.ingest.Cs == vec && dnn.in_c <= 4;
  }
  const TensorInfo& fin = net.layers[n - 1].out;
  net.n_out = fin.C * fin.H * fin.W;
  net.final_direct = net.layers[n - 1].d.op == DARIS_OP_FC;

  // legal cuts: after layer l, when every later layer reads only tensors produced at or after l
  for (int l = 0; l + 1 < n; ++l) {
    bool ok = true;
    for (int q = l + 1; q < n && ok; ++q) {
      const daris_layer& d = net.layers[q].d;
      if (d.in_from < l) ok = false;
      if (d.res_from >= 0 && d.res_from < l) ok = false;
    }
    if (ok) net.legal_cuts.push_back(l);
  }
  net.stage_first.assign(1, 0);

  // activation slots: a tensor's slot is free again once its last reader has been issued (same stream, in order)
  // The earlier member of a launch pair is issued with the later one (and its split-K reduction after that launch):
  // what it reads must stay in place until then, so its reads count as reads of the later layer.
  std::vector<int> last_use(n + 1, -1);
  for (int l = 0; l < n; ++l) {
    const LayerPlan& L = net.layers[l];
    const int at = std::max(l, L.pair_with);
    last_use[L.in_t] = std::max(last_use[L.in_t], at);
    if (L.res_t >= 0) last_use[L.res_t] = std::max(last_use[L.res_t], at);
  }
  std::vector<int> slot_owner;  // tensor currently held by each slot, -1 = free
  auto take_slot = [&](int tensor, size_t bytes) {
    int s = -1;
    if (!keep_activations)
      for (size_t i = 0; i < slot_owner.size(); ++i)
        if (slot_owner[i] < 0) { s = (int)i; break; }
    if (s < 0) {
      slot_owner.push_back(-1);
      net.slot_bytes.push_back(0);
      s = (int)slot_owner.size() - 1;
    }
    slot_owner[s] = tensor;
    net.slot_bytes[s] = std::max(net.slot_bytes[s], bytes);
    return s;
  };
  net.ingest.slot = take_slot(0, net.ingest.bytes);
  for (int l = 0; l < n; ++l) {
    for (size_t i = 0; i < slot_owner.size(); ++i)
      if (slot_owner[i] >= 0 && last_use[slot_owner[i]] < l) slot_owner[i] = -1;
    if (l == n - 1 && net.final_direct) break;  // logits go straight to the caller's buffer
    net.layers[l].out.slot = take_slot(l + 1, net.layers[l].out.bytes);
  }
  return "";
}

bool split_stages(NetPlan* net, int k) {
  const int n = (int)net->layers.size();
  if (k < 1 || k - 1 > (int)net->legal_cuts.size()) return false;
  std::vector<int64_t> pre(n + 1, 0);
  for (int l = 0; l < n; ++l) pre[l + 1] = pre[l] + net->layers[l].macs;
  auto sum = [&](int a, int b) { return pre[b + 1] - pre[a]; };  // layers a..b inclusive
  const int64_t INF = std::numeric_limits<int64_t>::max();
  std::vector<char> legal(n, 0);
  for (int c : net->legal_cuts) legal[c] = 1;
  // f[r][s]: least possible largest-stage MACs when layers s..n-1 form r stages
  std::vector<std::vector<int64_t>> f(k + 1, std::vector<int64_t>(n + 1, INF));
  for (int s = 0; s < n; ++s) f[1][s] = sum(s, n - 1);
  for (int r = 2; r <= k; ++r)
    for (int s = 0; s < n; ++s)
      for (int c = s; c + 1 < n; ++c) {
        if (!legal[c] || f[r - 1][c + 1] == INF) continue;
        f[r][s] = std::min(f[r][s], std::max(sum(s, c), f[r - 1][c + 1]));
      }
  const int64_t best = f[k][0];
  if (best == INF) return false;
  std::vector<int> first(1, 0);
  int pos = 0;
  for (int r = k; r >= 2; --r) {
    int chosen = -1;
    for (int c = pos; c + 1 < n; ++c) {
      if (!legal[c] || f[r - 1][c + 1] == INF) continue;
      if (std::max(sum(pos, c), f[r - 1][c + 1]) <= best) { chosen = c; break; }
    }
    if (chosen < 0) return false;
    pos = chosen + 1;
    first.push_back(pos);
  }
  net->stage_first = first;
  return true;
}

template <typename T>
static void put(std::vector<unsigned char>* buf, size_t idx, float v, bool bf16) {
  if (bf16) reinterpret_cast<uint16_t*>(buf->data())[idx] = host_f32_to_bf16(v);
  else reinterpret_cast<float*>(buf->data())[idx] = v;
}

void pack_conv(const NetPlan& net, const LayerPlan& L, const float* w, const float* b, std::vector<unsigned char>* wp,
               std::vector<float>* bp) {
  const daris_layer& d = L.d;
  const TensorInfo& in = net.tensor(L.in_t);
  const bool bf = net.bf16;
  const size_t es = bf ? 2 : 4;
  const int kk = d.k * d.k;
  bp->assign(L.out.Cs, 0.f);
  if (b)
    for (int o = 0; o < d.c_out; ++o) (*bp)[o] = b[o];
  if (L.depthwise) {
    // [tap][C]
    wp->assign((size_t)kk * in.Cs * es, 0);
    for (int c = 0; c < d.c_out; ++c)
      for (int t = 0; t < kk; ++t) put<float>(wp, (size_t)t * in.Cs + c, w[(size_t)c * kk + t], bf);
    return;
  }
  if (L.cp.rows == 16) {
    // 16-row kernel: [channel block of 16][step][lane = j + 16 q][VEC], element e of lane (j, q) at step s is
    // W[n = 16 nb + j][k = s * 4 VEC + q * VEC + e], k = tap * Cs_in + ci; blocks padded to a multiple of TN
    const int vec = bf ? 8 : 4, ks = 4 * vec, S = L.cp.S;
    const int nblocks = (L.out.Cs + 15) / 16;
    const int nb_alloc = (nblocks + L.cp.tn - 1) / L.cp.tn * L.cp.tn;
    wp->assign((size_t)nb_alloc * S * 64 * 16 + 8 * 1024, 0);  // + slack for the pipeline's refills past the last step
    for (int o = 0; o < d.c_out; ++o)
      for (int ci = 0; ci < d.c_in; ++ci)
        for (int t = 0; t < kk; ++t) {
          const int k = t * in.Cs + ci;
          const int st = k / ks, q = (k % ks) / vec, e = k % vec;
          const size_t lane = (size_t)(o % 16) + 16 * q;
          put<float>(wp, (((size_t)(o / 16) * S + st) * 64 + lane) * vec + e, w[((size_t)o * d.c_in + ci) * kk + t], bf);
        }
    return;
  }
  // [channel block of 32][step][lane = i + 32 h][VEC], element e of lane (i, h) at step s is
  // W[n = 32 nb + i][k = s*KS + h*VEC + e], k = tap * Cs_in + ci; blocks padded to a multiple of TN, zeros elsewhere
  const int vec = bf ? 8 : 4, ks = 2 * vec, S = L.cp.S;
  const int nblocks = (L.out.Cs + 31) / 32;
  const int nb_alloc = (nblocks + L.cp.tn - 1) / L.cp.tn * L.cp.tn;
  wp->assign((size_t)nb_alloc * S * 64 * 16 + 8 * 1024, 0);  // + slack for the kernel's pipeline refills past the last step
  for (int o = 0; o < d.c_out; ++o)
    for (int ci = 0; ci < d.c_in; ++ci)
      for (int t = 0; t < kk; ++t) {
        const int k = t * in.Cs + ci;
        const int st = k / ks, h = (k % ks) / vec, e = k % vec;
        const size_t lane = (size_t)(o % 32) + 32 * h;
        put<float>(wp, (((size_t)(o / 32) * S + st) * 64 + lane) * vec + e, w[((size_t)o * d.c_in + ci) * kk + t], bf);
      }
}

void pack_fc(const NetPlan& net, const LayerPlan& L, const float* w, const float* b, std::vector<unsigned char>* wp,
             std::vector<float>* bp) {
  const daris_layer& d = L.d;
  const TensorInfo& in = net.tensor(L.in_t);
  const bool bf = net.bf16;
  const size_t es = bf ? 2 : 4;
  const int hw = in.H * in.W;
  bp->assign(d.c_out, 0.f);
  if (b)
    for (int o = 0; o < d.c_out; ++o) (*bp)[o] = b[o];
  // [N][H*W*Cs]: caller order is (c, y, x); device tensors are (y, x, c) with channel stride Cs
  wp->assign((size_t)d.c_out * L.K * es, 0);
  for (int o = 0; o < d.c_out; ++o)
    for (int c = 0; c < in.C; ++c)
      for (int px = 0; px < hw; ++px)
        put<float>(wp, (size_t)o * L.K + (size_t)px * in.Cs + c, w[(size_t)o * d.c_in + (size_t)c * hw + px], bf);
}

}  // namespace daris
