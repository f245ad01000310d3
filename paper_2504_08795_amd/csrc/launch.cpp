// Host side of the kernels: names, launch plans of the convolutions, and the encoders that turn a layer's arguments
// into ready-to-dispatch launches (kernel, geometry, argument bytes).
#include "kernels.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "aql.h"

namespace daris {

static const char* const kNames[K_COUNT] = {
    "none",
    "conv_wave_f32_t1w2", "conv_wave_f32_t1w4", "conv_wave_f32_t1w8", "conv_wave_f32_t2w2", "conv_wave_f32_t2w4", "conv_wave_f32_t2w8",
    "conv_wave_bf16_t1w2", "conv_wave_bf16_t1w4", "conv_wave_bf16_t1w8", "conv_wave_bf16_t2w2", "conv_wave_bf16_t2w4", "conv_wave_bf16_t2w8",
    "conv_wave16_f32_t1w2", "conv_wave16_f32_t1w4", "conv_wave16_f32_t1w8", "conv_wave16_f32_t2w2", "conv_wave16_f32_t2w4", "conv_wave16_f32_t2w8",
    "conv_wave16_bf16_t1w2", "conv_wave16_bf16_t1w4", "conv_wave16_bf16_t1w8", "conv_wave16_bf16_t2w2", "conv_wave16_bf16_t2w4", "conv_wave16_bf16_t2w8",
    "splitk_reduce", "dwconv", "maxpool", "gavgpool", "fc", "ingest", "egress"};

const char* kernel_name(int32_t id) { return (id >= 0 && id < K_COUNT) ? kNames[id] : "?"; }

static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Launches of equal workgroups run in ceil(workgroups / CUs) rounds: how many rounds' worth of time the grid needs per
// round's worth of work.  1 = perfectly even; 98 workgroups on 96 CUs: 1.96.
static double round_waste(int groups, int cus) { return (double)cdiv(groups, cus) * cus / groups; }

static ConvPlan plan_conv_wave(int M, int N, int Kpad, int bf16, int step_align, int nominal_cus, int force_tn = 0, int force_nw = 0) {
  const int kNominalWaveSlots = 4 * nominal_cus;  // SIMDs of the partition size the plan is balanced for
  // Measured on a 128-CU partition (fp32, ResNet-18 shapes): the K loop itself runs near the MFMA rate; what a
  // launch pays for is its fixed cost and idle CUs.  Best found: 8 waves per workgroup splitting K, and enough
  // grid.z slices that tiles * z is about the number of CUs, while a wave keeps at least ~6 steps.
  ConvPlan pl = ConvPlan();
  const int ks = bf16 ? 16 : 8;  // k per step: two 16-byte vectors
  const int S = Kpad / ks;
  const int nb = cdiv(N, 32);
  // A wave tile two channel blocks wide halves the reads of the pixel operand, but also halves the number of tiles:
  // below about 3/4 of the partition's CUs it is better to keep 32-channel tiles and split K less (or not at all,
  // which saves the reduction launch).
  int tn = (nb % 2 == 0 && cdiv(M, 32) * (nb / 2) >= nominal_cus * 3 / 4) ? 2 : 1;
  // ... unless the 64-channel tiles are a few more than the CUs (98 on 96): the launch then takes two rounds for hardly more
  // than one round's work, and twice as many tiles of half the work take three half rounds
  if (tn == 2) {
    const int t2 = cdiv(M, 32) * (nb / 2);
    // (only for grids of one to two rounds: with more, the loss is smaller and the next round's workgroups overlap the tail -- measured: no gain)
    if (t2 > nominal_cus && t2 <= 2 * nominal_cus && round_waste(t2, nominal_cus) > 1.3 && round_waste(2 * t2, nominal_cus) < round_waste(t2, nominal_cus)) tn = 1;
  }
  if (force_tn) tn = force_tn;
  // Fetching the pixel operand as coalesced rows through LDS pays where a launch is bound by its loads: every bf16 shape
  // (+11 % on the saturated ResNet-50 set) and 32-channel fp32 tiles.  fp32 tiles of 64 channels are bound by the matrix
  // pipe; there the extra LDS round trip and registers cost 10-25 % (measured on VGG-16's layers; still 10 % with the
  // register count held at 128), so they stay register-fed.
  if (step_align > 1 && !bf16 && tn == 2) step_align = 1;
  const int tiles = cdiv(M, 32) * (nb / tn);
  int nw = bf16 ? 4 : 8;  // bf16 steps are short: fewer waves to sum through LDS beat a finer K split (measured 0.4-0.8 us per layer)
  while (nw > 2 && (S / nw < 4 || tiles * nw > 8 * kNominalWaveSlots)) nw /= 2;  // >= 4 steps per wave, <= 8 waves per SIMD
  int z = nominal_cus / tiles;
  if (z < 1) z = 1;
  const int max_by_k = S / (nw * 6) > 0 ? S / (nw * 6) : 1;
  if (z > max_by_k) z = max_by_k;
  if (z > 16) z = 16;
  if (tiles > nominal_cus) {
    // More tiles than CUs: the launch runs in ceil(tiles * z / CUs) rounds of workgroups whose K loops take
    // (S / z) * tn * c cycles of MFMA time per SIMD, so a K split can even out the last round (200 tiles: z = 1 and 2
    // need the time of 2 whole tiles, z = 3 that of 5/3).  Model checked against measured VGG-16 layers (within 3 %):
    // loop time x 1.3 + a reduction pass of 3 us + its traffic at 1.5 TB/s.
    const double cyc = bf16 ? tn * 8.0 : tn * 64.0;
    double best = 1e30;
    for (int zz = 1; zz <= 6 && S / (nw * zz) >= 6; ++zz) {
      const double rounds = (double)cdiv(tiles * zz, nominal_cus);
      double us = 1.3 * rounds * cdiv(S, zz) * cyc / 2400.0;
      if (zz > 1) us += 3.0 + (double)zz * M * N * 4.0 / 1.5e6;
      if (us < best) {
        best = us;
        z = zz;
      }
    }
  }
  if (force_nw) {  // second problem of a two-problem launch: the first one's kernel variant, no split across workgroups
    nw = force_nw;
    z = 1;
  }
  // K slices of workgroups and waves in whole multiples of step_align steps (2 when the kernel fetches the pixel
  // operand in chunks of two steps; S is then even as well)
  const int sz = cdiv(cdiv(S, z), step_align) * step_align;
  z = cdiv(S, sz);
  pl.rows = 32;
  pl.tn = tn;
  pl.nw = nw;
  pl.S = S;
  pl.sz = sz;
  pl.sw = cdiv(cdiv(sz, nw), step_align) * step_align;
  pl.step_align = step_align;
  pl.splitk = z;
  pl.tiles = tiles;
  pl.threads = nw * 64;
  pl.MT = cdiv(M, 32);  // (the division multipliers are filled in by the caller, which knows Wo, Cin and kw)
  pl.NTn = nb / tn;
  pl.G = pl.NTn * z;
  if (pl.G % 8 == 0) {
    pl.xmode = 1;
    pl.grid_x = (uint32_t)(pl.G * pl.MT);
  } else if (8 % pl.G == 0) {
    pl.xmode = 2;
    pl.grid_x = (uint32_t)(8 * cdiv(pl.MT, 8 / pl.G));
  } else {
    pl.xmode = 0;
    pl.grid_x = (uint32_t)(pl.G * pl.MT);
  }
  pl.ws_bytes = z > 1 ? (size_t)z * M * N * sizeof(float) : 0;
  const int wi = nw == 2 ? 0 : (nw == 4 ? 1 : 2);
  pl.kernel = (bf16 ? K_CONVW_BF16_T1W2 : K_CONVW_F32_T1W2) + (tn - 1) * 3 + wi;
  return pl;
}

// 16-pixel tiles of tn 16-channel blocks, K split among the waves of a workgroup only.  Chosen for layers whose 32-row
// plan needs a reduction launch; returns kernel == K_NONE when the shape does not fill three quarters of the nominal
// partition either, or is too shallow to split eight (four) ways.
static ConvPlan plan_conv_wave16(int M, int N, int Kpad, int bf16, int nominal_cus, int force_tn = 0, int force_nw = 0) {
  ConvPlan pl = ConvPlan();
  const int ks = bf16 ? 32 : 16;
  if (Kpad % ks) return pl;
  const int S = Kpad / ks;
  const int nb = cdiv(N, 16), mt = cdiv(M, 16);
  // two channel blocks per wave halve the reads of the pixel operand: taken when that still gives nearly one workgroup per CU
  // (and not a few more than one per CU, see plan_conv_wave)
  int tn = (nb % 2 == 0 && mt * (nb / 2) >= nominal_cus * 3 / 4) ? 2 : 1;
  if (tn == 2) {
    const int t2 = mt * (nb / 2);
    // (only for grids of one to two rounds: with more, the loss is smaller and the next round's workgroups overlap the tail -- measured: no gain)
    if (t2 > nominal_cus && t2 <= 2 * nominal_cus && round_waste(t2, nominal_cus) > 1.3 && round_waste(2 * t2, nominal_cus) < round_waste(t2, nominal_cus)) tn = 1;
  }
  if (force_tn) tn = force_tn;
  if (nb % tn) return pl;
  const int tiles = mt * (nb / tn);
  int nw = bf16 ? 4 : 8;
  while (nw > 2 && S / nw < 4) nw /= 2;
  if (force_nw) {  // second problem of a two-problem launch: the first one's kernel variant, whatever its own shape
    nw = force_nw;
  } else if (tiles < nominal_cus * 3 / 4 || tiles > 4 * nominal_cus || S / nw < 2) {
    return pl;
  }
  pl.rows = 16;
  pl.tn = tn;
  pl.nw = nw;
  pl.S = S;
  pl.sz = S;
  pl.sw = cdiv(S, nw);
  pl.step_align = 1;
  pl.splitk = 1;
  pl.tiles = tiles;
  pl.threads = nw * 64;
  pl.MT = mt;
  pl.NTn = nb / tn;
  pl.G = pl.NTn;
  if (pl.G % 8 == 0) {
    pl.xmode = 1;
    pl.grid_x = (uint32_t)(pl.G * pl.MT);
  } else if (8 % pl.G == 0) {
    pl.xmode = 2;
    pl.grid_x = (uint32_t)(8 * cdiv(pl.MT, 8 / pl.G));
  } else {
    pl.xmode = 0;
    pl.grid_x = (uint32_t)(pl.G * pl.MT);
  }
  pl.ws_bytes = 0;
  const int wi = nw == 2 ? 0 : (nw == 4 ? 1 : 2);
  pl.kernel = (bf16 ? K_CONV16_BF16_T1W2 : K_CONV16_F32_T1W2) + (tn - 1) * 3 + wi;
  return pl;
}

ConvPlan plan_conv(int M, int N, int Kpad, int bf16, int step_align, int cin_stride, int nominal_cus) {
  if (nominal_cus < 8) nominal_cus = 8;
  if (nominal_cus > 256) nominal_cus = 256;
  const ConvPlan pl = plan_conv_wave(M, N, Kpad, bf16, step_align, nominal_cus);
  if (pl.splitk > 1 && cin_stride > 0 && cin_stride % (bf16 ? 32 : 16) == 0) {
    const ConvPlan p16 = plan_conv_wave16(M, N, Kpad, bf16, nominal_cus);
    if (p16.kernel != K_NONE) return p16;
  }
  return pl;
}

ConvPlan plan_conv_like(const ConvPlan& first, int M, int N, int Kpad, int bf16, int step_align, int nominal_cus) {
  ConvPlan none = ConvPlan();
  if (nominal_cus < 8) nominal_cus = 8;
  if (nominal_cus > 256) nominal_cus = 256;
  if (first.rows == 16) return plan_conv_wave16(M, N, Kpad, bf16, nominal_cus, first.tn, first.nw);
  if (cdiv(N, 32) % first.tn != 0) return none;
  return plan_conv_wave(M, N, Kpad, bf16, step_align, nominal_cus, first.tn, first.nw);
}


// ---- kernel table ------------------------------------------------------------------------------------------------------------

namespace {

struct ReduceArgs {  // splitk_reduce_kernel(ws, bias, res, y, M, N, splitk, act)
  const float* ws;
  const float* bias;
  const void* res;
  void* y;
  int M, N, splitk, act;
};
struct IngestArgs {  // ingest_kernel / egress_kernel (x, y, C, Cs, HW)
  const void* x;
  void* y;
  int C, Cs, HW;
};
struct ProbeArgs {  // cu_probe_kernel(out, spin)
  uint32_t* out;
  int spin;
};
struct PairArgs {  // conv_wave_pair_kernel(p0, p1, n0)
  ConvArgs p0, p1;
  int n0;
};
struct ConvDwArgs {  // conv_wave_dw_kernel(p, d)
  ConvArgs p;
  DwFusedArgs d;
};
constexpr uint32_t kIngestBytes = 28, kProbeBytes = 12, kPairBytes = 2 * sizeof(ConvArgs) + 4;
static_assert(sizeof(DwFusedArgs) == 32 && sizeof(ConvDwArgs) == 192 && offsetof(ConvDwArgs, d) == sizeof(ConvArgs), "fused depthwise arguments");
static_assert(sizeof(ConvArgs) == 160 && sizeof(DwArgs) == 72 && sizeof(PoolArgs) == 48 && sizeof(FcArgs) == 56 && sizeof(ReduceArgs) == 48,
              "argument structures must match what the kernels were compiled for");
static_assert(offsetof(ConvArgs, x) == kConvInputOffset && offsetof(FcArgs, y) == kFcOutputOffset && offsetof(IngestArgs, x) == kIngestInputOffset &&
                  offsetof(IngestArgs, y) == kEgressOutputOffset && offsetof(PairArgs, p1) == sizeof(ConvArgs) &&
                  offsetof(PairArgs, n0) == 2 * sizeof(ConvArgs),
              "argument offsets");

bool push(std::vector<KernelLaunch>* out, const AqlKernel* k, int32_t id, uint32_t groups, uint32_t threads, const void* args, uint32_t nbytes) {
  if (!k || k->kernarg_size != nbytes || nbytes > sizeof(KernelLaunch::args) || groups == 0) return false;
  KernelLaunch l;
  l.k = k;
  l.kernel_id = id;
  l.groups = groups;
  l.threads = threads;
  l.nbytes = nbytes;
  std::memcpy(l.args, args, nbytes);
  out->push_back(l);
  return true;
}

}  // namespace

std::string KernelTable::resolve(const AqlRuntime& rt) {
  std::string missing;
  auto get = [&](const std::string& name, uint32_t want_bytes) -> const AqlKernel* {
    const AqlKernel* k = rt.kernel(name);
    if ((!k || k->kernarg_size != want_bytes) && missing.empty())
      missing = name + (k ? " (argument block of " + std::to_string(k->kernarg_size) + " bytes, expected " + std::to_string(want_bytes) + ")" : " (not in the code object)");
    return k;
  };
  static const int tn_[6] = {1, 1, 1, 2, 2, 2}, nw_[6] = {2, 4, 8, 2, 4, 8};
  for (int b = 0; b < 2; ++b) {
    const std::string B = b ? "true" : "false";
    for (int v = 0; v < 6; ++v) {
      const std::string tp = B + ", " + std::to_string(tn_[v]) + ", " + std::to_string(nw_[v]) + ", ";
      for (int m = 0; m < 4; ++m) conv[b][v][m] = get("daris::conv_wave_kernel<" + tp + std::to_string(m) + ">", sizeof(ConvArgs));
      static const int pair_modes[3] = {0, 1, 3};
      for (int m = 0; m < 3; ++m) pair[b][v][m] = get("daris::conv_wave_pair_kernel<" + tp + std::to_string(pair_modes[m]) + ">", kPairBytes);
    }
    for (int v = 0; v < 6; ++v) {
      conv16[b][v] = get("daris::conv_wave16_kernel<" + B + ", " + std::to_string(tn_[v]) + ", " + std::to_string(nw_[v]) + ">", sizeof(ConvArgs));
      pair16[b][v] = get("daris::conv_wave16_pair_kernel<" + B + ", " + std::to_string(tn_[v]) + ", " + std::to_string(nw_[v]) + ">", kPairBytes);
      if (b ? nw_[v] != 8 : tn_[v] == 1)
        convdw[b][v] = get("daris::conv_wave_dw_kernel<" + B + ", " + std::to_string(tn_[v]) + ", " + std::to_string(nw_[v]) + ">", sizeof(ConvDwArgs));
    }
    reduce[b] = get("daris::splitk_reduce_kernel<" + B + ">", sizeof(ReduceArgs));
    dwconv[b] = get("daris::dwconv_kernel<" + B + ">", sizeof(DwArgs));
    maxpool[b] = get("daris::maxpool_kernel<" + B + ">", sizeof(PoolArgs));
    gavgpool[b] = get("daris::gavgpool_kernel<" + B + ">", sizeof(PoolArgs));
    fc[b] = get("daris::fc_kernel<" + B + ">", sizeof(FcArgs));
    ingest[b] = get("daris::ingest_kernel<" + B + ">", kIngestBytes);
    egress[b] = get("daris::egress_kernel<" + B + ">", kIngestBytes);
  }
  cu_probe = get("daris::cu_probe_kernel", kProbeBytes);
  return missing;
}

// ---- encoders ----------------------------------------------------------------------------------------------------------------

static bool push_reduce(const KernelTable& kt, const ConvPlan& pl, const ConvArgs& a, int bf16, std::vector<KernelLaunch>* out) {
  if (pl.splitk <= 1) return true;
  const size_t total4 = (size_t)a.M * a.Cout / 4;
  ReduceArgs r{a.ws, a.bias, a.res, a.y, a.M, a.Cout, pl.splitk, a.act};
  return push(out, kt.reduce[bf16], K_SPLITK_REDUCE, (uint32_t)((total4 + 255) / 256), 256, &r, sizeof(r));
}

bool encode_conv(const KernelTable& kt, const ConvPlan& pl, const ConvArgs& a, int bf16, std::vector<KernelLaunch>* out) {
  if (pl.rows == 16) {
    const int v16 = pl.kernel - (bf16 ? K_CONV16_BF16_T1W2 : K_CONV16_F32_T1W2);
    const int ks16 = bf16 ? 32 : 16;
    if (v16 < 0 || v16 >= 6 || pl.threads != 64 * pl.nw || a.c_real > 0 || a.Cin % ks16 || a.Kpad % ks16 || pl.S * ks16 != a.Kpad) return false;
    if (pl.splitk > 1 && !a.ws) return false;
    if (!push(out, kt.conv16[bf16][v16], pl.kernel, pl.grid_x, (uint32_t)pl.threads, &a, sizeof(a))) return false;
    return push_reduce(kt, pl, a, bf16, out);
  }
  const int variant = pl.kernel - (bf16 ? K_CONVW_BF16_T1W2 : K_CONVW_F32_T1W2);
  if (variant < 0 || variant >= 6 || pl.threads != 64 * pl.nw) return false;
  // 0: a K step never straddles a filter tap; 1: general walk; 2: layer 0 reading the caller's fp32 [C][H][W] input;
  // 3: a pixel's channels are whole 64-byte rows and the plan cuts K in chunks of two steps: pixel operand through LDS
  const int mode = a.c_real > 0 ? 2 : (conv_rows_staged(a.Cin, bf16) && pl.step_align == 2 ? 3 : (a.Cin % (bf16 ? 16 : 8) == 0 ? 0 : 1));
  if (mode == 3 && (pl.S % 2 || pl.sz % 2 || pl.sw % 2)) return false;
  if (mode == 2 && (a.Cin != (bf16 ? 8 : 4) || a.c_real > 4)) return false;
  if (pl.splitk > 1 && !a.ws) return false;
  if (!push(out, kt.conv[bf16][variant][mode], pl.kernel, pl.grid_x, (uint32_t)pl.threads, &a, sizeof(a))) return false;
  return push_reduce(kt, pl, a, bf16, out);
}

bool conv_dw_fusable(const ConvPlan& pl, int bf16) {
  if (pl.rows != 32 || pl.step_align != 2 || (!bf16 && pl.tn != 1) || (bf16 && pl.nw == 8)) return false;  // no such kernel variant
  return pl.MT >= 96 && pl.NTn == 1;
}

bool encode_conv_dw(const KernelTable& kt, const ConvPlan& pl, const ConvArgs& a, const DwFusedArgs& d, int bf16, std::vector<KernelLaunch>* out) {
  const int variant = pl.kernel - (bf16 ? K_CONVW_BF16_T1W2 : K_CONVW_F32_T1W2);
  if (pl.rows != 32 || variant < 0 || variant >= 6 || pl.threads != 64 * pl.nw || !conv_dw_fusable(pl, bf16)) return false;
  const AqlKernel* kernel = kt.convdw[bf16][variant];
  if (!kernel) return false;
  // what the kernel's producer assumes: a 1x1 / stride 1 / unpadded convolution over whole 64-byte rows, K cut in chunks of two steps,
  // a depthwise input that maps onto the convolution's pixels, and offsets that fit 32 bits
  if (a.kh != 1 || a.kw != 1 || a.stride != 1 || a.pad != 0 || a.c_real > 0 || a.Kpad != a.Cin || a.H != a.Ho || a.W != a.Wo) return false;
  if (!conv_rows_staged(a.Cin, bf16) || pl.step_align != 2 || pl.S % 2 || pl.sz % 2 || pl.sw % 2 || a.Cin < (bf16 ? 32 : 16)) return false;
  if (!d.w || !d.bias || (d.stride != 1 && d.stride != 2) || (d.H + 2 - 3) / d.stride + 1 != a.H || (d.W + 2 - 3) / d.stride + 1 != a.W) return false;
  if ((uint64_t)d.H * (uint64_t)d.W * (uint64_t)a.Cin >= (1ull << 31)) return false;
  if (pl.splitk > 1 && !a.ws) return false;
  ConvDwArgs args;
  std::memset(&args, 0, sizeof(args));
  args.p = a;
  args.d = d;
  if (!push(out, kernel, pl.kernel, pl.grid_x, (uint32_t)pl.threads, &args, sizeof(args))) return false;
  return push_reduce(kt, pl, a, bf16, out);
}

bool encode_conv_pair(const KernelTable& kt, const ConvPlan& pl0, const ConvArgs& a0, const ConvPlan& pl1, const ConvArgs& a1, int bf16,
                      std::vector<KernelLaunch>* out) {
  if (pl0.rows == 16) {
    const int ks16 = bf16 ? 32 : 16;
    const int v16 = pl0.kernel - (bf16 ? K_CONV16_BF16_T1W2 : K_CONV16_F32_T1W2);
    if (pl1.rows != 16 || pl0.kernel != pl1.kernel || v16 < 0 || v16 >= 6 || pl0.splitk != 1 || pl1.splitk != 1 || a0.c_real > 0 || a1.c_real > 0 ||
        a0.Cin % ks16 || a1.Cin % ks16 || pl0.S * ks16 != a0.Kpad || pl1.S * ks16 != a1.Kpad)
      return false;
    PairArgs pa;
    std::memset(&pa, 0, sizeof(pa));
    pa.p0 = a0;
    pa.p1 = a1;
    pa.n0 = (int)((pl0.grid_x + 7) / 8 * 8);
    return push(out, kt.pair16[bf16][v16], pl0.kernel, (uint32_t)pa.n0 + pl1.grid_x, (uint32_t)pl0.threads, &pa, kPairBytes);
  }
  const int ks = bf16 ? 16 : 8;
  const bool aligned = a0.Cin % ks == 0;
  if (pl0.kernel != pl1.kernel || pl0.rows != 32 || aligned != (a1.Cin % ks == 0) || pl1.splitk != 1 || a0.c_real > 0 || a1.c_real > 0) return false;
  const bool staged = conv_rows_staged(a0.Cin, bf16) && conv_rows_staged(a1.Cin, bf16) && pl0.step_align == 2 && pl1.step_align == 2;
  if (staged && (pl0.S % 2 || pl0.sz % 2 || pl0.sw % 2 || pl1.S % 2 || pl1.sz % 2 || pl1.sw % 2)) return false;
  const int variant = pl0.kernel - (bf16 ? K_CONVW_BF16_T1W2 : K_CONVW_F32_T1W2);
  if (variant < 0 || variant >= 6 || (pl0.splitk > 1 && !a0.ws)) return false;
  PairArgs pa;
  std::memset(&pa, 0, sizeof(pa));
  pa.p0 = a0;
  pa.p1 = a1;
  pa.n0 = (int)((pl0.grid_x + 7) / 8 * 8);  // the second problem starts at a multiple of 8: its workgroup -> XCD relation is kept
  if (!push(out, kt.pair[bf16][variant][staged ? 2 : (aligned ? 0 : 1)], pl0.kernel, (uint32_t)pa.n0 + pl1.grid_x, (uint32_t)pl0.threads, &pa, kPairBytes)) return false;
  return push_reduce(kt, pl0, a0, bf16, out);
}

bool encode_dwconv(const KernelTable& kt, const DwArgs& a, int bf16, std::vector<KernelLaunch>* out) {
  const size_t total = (size_t)a.Ho * a.Wo * (a.C / (bf16 ? 8 : 4));
  return push(out, kt.dwconv[bf16], K_DWCONV, (uint32_t)((total + 255) / 256), 256, &a, sizeof(a));
}
bool encode_maxpool(const KernelTable& kt, const PoolArgs& a, int bf16, std::vector<KernelLaunch>* out) {
  const size_t total = (size_t)a.Ho * a.Wo * (a.C / (bf16 ? 8 : 4));
  return push(out, kt.maxpool[bf16], K_MAXPOOL, (uint32_t)((total + 255) / 256), 256, &a, sizeof(a));
}
bool encode_gavgpool(const KernelTable& kt, const PoolArgs& a, int bf16, std::vector<KernelLaunch>* out) {
  return push(out, kt.gavgpool[bf16], K_GAVGPOOL, (uint32_t)cdiv(a.C, 64), 256, &a, sizeof(a));
}
bool encode_fc(const KernelTable& kt, const FcArgs& a, int bf16, std::vector<KernelLaunch>* out) {
  return push(out, kt.fc[bf16], K_FC, (uint32_t)cdiv(a.Ns, 4), 256, &a, sizeof(a));
}
bool encode_ingest(const KernelTable& kt, const float* x, void* y, int C, int Cs, int H, int W, int bf16, std::vector<KernelLaunch>* out) {
  IngestArgs a{x, y, C, Cs, H * W};
  const size_t total = (size_t)H * W * Cs;
  return push(out, kt.ingest[bf16], K_INGEST, (uint32_t)((total + 255) / 256), 256, &a, kIngestBytes);
}
bool encode_egress(const KernelTable& kt, const void* x, float* y, int C, int Cs, int H, int W, int bf16, std::vector<KernelLaunch>* out) {
  IngestArgs a{x, y, C, Cs, H * W};
  const size_t total = (size_t)H * W * C;
  return push(out, kt.egress[bf16], K_EGRESS, (uint32_t)((total + 255) / 256), 256, &a, kIngestBytes);
}
bool encode_cu_probe(const KernelTable& kt, uint32_t* out_dev, int n_groups, int spin, std::vector<KernelLaunch>* out) {
  ProbeArgs a{out_dev, spin};
  return push(out, kt.cu_probe, K_NONE, (uint32_t)n_groups, 64, &a, kProbeBytes);
}

}  // namespace daris
