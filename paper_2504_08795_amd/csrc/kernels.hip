// HIP kernels of the DNN stages for gfx950 (CDNA4): implicit-GEMM convolution on MFMA with register-fed wave tiles
// and a fused bias / residual / activation epilogue, split-K reduction, depthwise convolution, pooling, FC
// (batch-1 GEMV), and the NCHW<->NHWC boundary conversions.  A DNN is, for the scheduler of the paper
// (Sec. I, Sec. III-B1), a sequence of such kernels cut into stages.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kernels.h"

namespace daris {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ---- element helpers ------------------------------------------------------------------------------------------

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// float -> bfloat16 bits, round to nearest, ties to even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == 1) v = fmaxf(v, 0.f);
  else if (act == 2) v = fminf(fmaxf(v, 0.f), 6.f);
  return v;
}

template <bool BF16>
__device__ __forceinline__ float load_elem(const void* p, size_t i) {
  if (BF16) return bf16_bits_to_f32(((const uint16_t*)p)[i]);
  return ((const float*)p)[i];
}

template <bool BF16>
__device__ __forceinline__ void store_elem(void* p, size_t i, float v) {
  if (BF16) ((uint16_t*)p)[i] = (uint16_t)f32_to_bf16_bits(v);
  else ((float*)p)[i] = v;
}

// n / d for 0 <= n with n * d < 2^32, through the host-made multiplier magic = floor(2^32 / d) + 1 (0 stands for d = 1):
// the quotient is the high word of n * magic, a handful of cycles instead of the ~40-instruction division sequence.
__device__ __forceinline__ int fast_div(int n, uint32_t magic) { return magic ? (int)__umulhi((uint32_t)n, magic) : n; }

// v if ok, else all zero bits; component-wise so that it stays a register select (a select between two uint4
// objects would be done through their addresses and push the access to scratch / flat memory).
__device__ __forceinline__ uint4 keep_if(bool ok, uint4 v) {
  v.x = ok ? v.x : 0u;
  v.y = ok ? v.y : 0u;
  v.z = ok ? v.z : 0u;
  v.w = ok ? v.w : 0u;
  return v;
}

// Unpack one 16-byte vector into VEC floats (4 for fp32, 8 for bf16).
template <bool BF16>
__device__ __forceinline__ void unpack(const uint4& v, float* o) {
  if (BF16) {
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
  } else {
    o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y); o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
  }
}

template <bool BF16>
__device__ __forceinline__ uint4 pack(const float* o) {
  uint4 v;
  if (BF16) {
    v.x = f32_to_bf16_bits(o[0]) | (f32_to_bf16_bits(o[1]) << 16);
    v.y = f32_to_bf16_bits(o[2]) | (f32_to_bf16_bits(o[3]) << 16);
    v.z = f32_to_bf16_bits(o[4]) | (f32_to_bf16_bits(o[5]) << 16);
    v.w = f32_to_bf16_bits(o[6]) | (f32_to_bf16_bits(o[7]) << 16);
  } else {
    v.x = __float_as_uint(o[0]); v.y = __float_as_uint(o[1]); v.z = __float_as_uint(o[2]); v.w = __float_as_uint(o[3]);
  }
  return v;
}

// Sums the split-K partials in split order and applies the fused epilogue.  One thread per 4 output channels.
template <bool BF16>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ ws, const float* __restrict__ bias,
                                                            const void* res, void* y, int M, int N, int splitk, int act) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t total4 = (size_t)M * N / 4;
  if (idx >= total4) return;
  const size_t o = idx * 4;
  const int n = (int)(o % N);
  float4 s = *(const float4*)(ws + o);
  for (int z = 1; z < splitk; ++z) {
    const float4 t = *(const float4*)(ws + (size_t)z * M * N + o);
    s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
  }
  const float4 b = *(const float4*)(bias + n);
  float v[4] = {s.x + b.x, s.y + b.y, s.z + b.z, s.w + b.w};
  if (res) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] += load_elem<BF16>(res, o + i);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = apply_act(v[i], act);
  if (BF16) {
    uint2 out;
    out.x = f32_to_bf16_bits(v[0]) | (f32_to_bf16_bits(v[1]) << 16);
    out.y = f32_to_bf16_bits(v[2]) | (f32_to_bf16_bits(v[3]) << 16);
    *(uint2*)((uint16_t*)y + o) = out;
  } else {
    *(float4*)((float*)y + o) = make_float4(v[0], v[1], v[2], v[3]);
  }
}

// ---- wave-tile implicit GEMM ---------------------------------------------------------------------------------------
//
// For the small-M, deep-K convolutions of batch-1 inference an output tile shared through LDS buys nothing: there
// are too few tiles to fill a partition, so K has to be split anyway.  Here one wave owns a 32 x (32*TN) output
// tile over a slice of K and feeds the MFMA straight from registers: lane (i, h) loads the 16 bytes of pixel
// m0+i at k = step*KS + h*VEC.. from the NHWC input and, per channel block, 16 bytes of weights that were packed
// at registration in exactly this order ([channel block][step][lane][16 B]: one fully coalesced 1 KiB read per
// step, consecutive steps consecutive in memory).  No barrier and no LDS in the K loop; D steps are in flight.
// The NW waves of a workgroup split the K slice of the workgroup; their partial tiles are summed through LDS in
// wave order.  With splitk > 1 several workgroups share one tile, split K as well and write partial sums to the workspace,
// which splitk_reduce_kernel adds in z order (a device-wide fence per workgroup for an in-kernel reduction was
// measured to cost several times the extra launch).
template <bool BF16, int TN, int NW, int MODE>
__device__ __forceinline__ void conv_wave_body(const ConvArgs& p, const int L, const DwFusedArgs& dwf) {
  // MODE 0: Cin a multiple of KS; 1: any Cin; 2: the network input itself, fp32 [C][H][W]; 3: a pixel's channels are whole
  // 64-byte rows (Cin * ES a multiple of 64): the pixel operand is fetched in coalesced rows and transposed through LDS;
  // 4: like 3 for a 1x1 convolution whose input is the output of a 3x3 depthwise convolution that is never stored: the
  // rows are computed here from the depthwise layer's input (p.x) and weights (dwf)
  constexpr bool ALIGNED = MODE == 0;
  constexpr bool STAGED = MODE == 3 || MODE == 4;
  constexpr bool DWF = MODE == 4;
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int VEC = 16 / ES;
  constexpr int KS = 2 * VEC;
  constexpr int NT = NW * 64;
  constexpr int TILE = TN * 1024;
  constexpr int D = 4;
  constexpr int STAGE_V = 32 * 5;  // 16-byte vectors of one wave's staging buffer: 32 pixels x (4 pieces + 1 pad)
  constexpr int LDS_F = (STAGED && NW * STAGE_V * 4 > NW * TILE) ? NW * STAGE_V * 4 : NW * TILE;
  static_assert(TN == 1 || TN == 2, "the epilogue selects between at most two channel blocks");
  static_assert((TILE / 4) % NT == 0 || NT % (TILE / 4) == 0, "tile / thread mismatch");

  __shared__ __align__(16) float red[LDS_F];

  if (p.wave_prio) __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the K loop's control flow scalar
  const int li = lane & 31, lh = lane >> 5;
  // Workgroup -> (pixel tile mt, weight group g = channel tile + n_tiles * K slice).  Workgroups are handed to the
  // 8 XCDs round-robin by linear id, and each XCD has its own L2: the mapping keeps all pixel tiles that read the
  // same weights on one XCD (xmode 1: groups are a multiple of 8) or on 8/G of them (xmode 2), so that a weight
  // byte is fetched from memory once per XCD that needs it instead of once per pixel tile.
  int mt, g;
  {
    const int x = L & 7, q = L >> 3;
    if (p.xmode == 1) {
      g = (q / p.MT) * 8 + x;
      mt = q % p.MT;
      if (g >= p.G) return;  // padding workgroups of a two-problem launch
    } else if (p.xmode == 2) {
      const int r = 8 / p.G;
      g = x / r;
      mt = q * r + (x % r);
      if (mt >= p.MT) return;
    } else {
      g = L / p.MT;
      mt = L % p.MT;
      if (g >= p.G) return;
    }
  }
  const int zi = g / p.NTn;
  const int m0 = mt * 32, nb0 = (g - zi * p.NTn) * TN;

  const int s_wg0 = zi * p.sz;
  const int s_wg1 = min(s_wg0 + p.sz, p.S);
  const int sbeg = min(s_wg0 + wave * p.sw, s_wg1);
  const int nsteps = min(sbeg + p.sw, s_wg1) - sbeg;

  const unsigned char* xb = (const unsigned char*)p.x;
  const int m = m0 + li;
  const bool a_ok = m < p.M;
  const int oy = fast_div(m, p.mg_wo), ox = m - oy * p.Wo;
  const int iy0 = oy * p.stride - p.pad, ix0 = ox * p.stride - p.pad;
  // Walk over k = (tap, ci).  ALIGNED (Cin a multiple of KS): both lane halves are always in the same tap, so the
  // walk state (ky, kx, ci) is wave-uniform and lives in scalars; a lane adds its half's offset lh*VEC, a step
  // inside a tap only advances the pointer and a new tap recomputes pointer and validity.  Otherwise (the padded
  // network input, Cin < KS, or Cin not a multiple of KS) each lane derives tap and channel of its vector from the
  // step number in closed form: no lane-dependent branch, so the loads stay unconditional and pipelined.
  int kcur = sbeg * KS;  // k of the next step to load (scalar)
  int tap = fast_div(kcur, p.mg_cin);
  int ci = kcur - tap * p.Cin;
  int ky = fast_div(tap, p.mg_kw), kx = tap - ky * p.kw;
  bool a_valid;
  const unsigned char* ap;
  auto enter_tap = [&]() {
    const int iy = iy0 + ky, ix = ix0 + kx;
    a_valid = a_ok && ky < p.kh && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
    ap = xb + ((size_t)(a_valid ? iy * p.W + ix : 0) * p.Cin + ci + lh * VEC) * ES;  // always a valid address
  };
  // MODE 2 reads the caller's fp32 [C][H][W] input directly (no separate layout conversion launch): the padded channel
  // count equals VEC, so a lane's vector is one filter tap, gathered as four scalar loads from the channel planes.
  // Planes beyond the real channel count repeat the last real one; their weights are zero.
  const size_t plane = (size_t)p.H * p.W;
  const size_t po1 = (size_t)min(1, p.c_real - 1) * plane, po2 = (size_t)min(2, p.c_real - 1) * plane,
               po3 = (size_t)min(3, p.c_real - 1) * plane;
  auto locate = [&]() {  // !ALIGNED: this lane's vector of step kcur
    const int k = kcur + lh * VEC;
    const int t = MODE == 2 ? k / VEC : fast_div(k, p.mg_cin), c = k - t * p.Cin;
    const int y = fast_div(t, p.mg_kw), x = t - y * p.kw;
    const int iy = iy0 + y, ix = ix0 + x;
    a_valid = a_ok && y < p.kh && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
    if (MODE == 2) ap = xb + (size_t)(a_valid ? iy * p.W + ix : 0) * 4;
    else ap = xb + ((size_t)(a_valid ? iy * p.W + ix : 0) * p.Cin + c) * ES;
  };
  if (ALIGNED) enter_tap();
  const unsigned char* wptr[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j)
    wptr[j] = (const unsigned char*)p.w + (((size_t)(nb0 + j) * p.S + sbeg) * 64 + lane) * 16;

  uint4 ar[D], br[D][TN];
  bool av[D];  // validity of slot d's A vector; the blanking is applied when the slot is consumed, so that a load's
               // result is not touched (and not waited for) until D-1 later steps have been issued
  auto load = [&](int d) {
    if (!ALIGNED) locate();
    if (MODE == 2) {
      const float* q = (const float*)ap;
      ar[d].x = __float_as_uint(q[0]);
      ar[d].y = __float_as_uint(q[po1]);
      ar[d].z = __float_as_uint(q[po2]);
      ar[d].w = __float_as_uint(q[po3]);
    } else {
      ar[d] = *(const uint4*)ap;
    }
    av[d] = a_valid;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      br[d][j] = *(const uint4*)wptr[j];
      wptr[j] += 1024;
    }
    if (ALIGNED) {
      ci += KS;
      if (ci >= p.Cin) {  // wave-uniform
        ci -= p.Cin;
        if (++kx == p.kw) { kx = 0; ++ky; }
        enter_tap();
      } else {
        ap += KS * ES;
      }
    } else {
      kcur += KS;
    }
  };

  // The epilogue works on quads of consecutive channels: quad q of the tile = elements 4q..4q+3 = lanes l..l+3 of one
  // accumulator row (j, v), i.e. one pixel and channels 32*(nb0+j) + l%32 .. +3.  A thread's quads q = tid + r*NT all
  // have the same l, so it needs the bias of one channel quad per channel block; fetched here, before the K loop,
  // so that the latency is hidden.
  const int ql = (4 * tid) & 63;  // first lane of this thread's quads
  float4 bias_j[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = (nb0 + j) * 32 + (ql & 31);
    bias_j[j] = (n < p.Cout) ? *(const float4*)(p.bias + n) : make_float4(0.f, 0.f, 0.f, 0.f);
  }

  // The residual operand of this thread's quads is fetched here as well (when this launch applies the epilogue itself).
  constexpr int QUADS = TILE / 4;
  constexpr int RQ = (QUADS + NT - 1) / NT;  // quads per thread
  using ResVec = typename std::conditional<BF16, uint2, uint4>::type;
  ResVec res_pre[RQ];
  const bool own_epilogue = p.splitk == 1;
  const bool use_res = own_epilogue && p.res != nullptr;
#pragma unroll
  for (int r = 0; r < RQ; ++r) {
    res_pre[r] = ResVec();
    const int e = 4 * (tid + r * NT);
    const int j = e >> 10, v = (e >> 6) & 15, l = e & 63;
    const int mm = m0 + (v >> 2) * 8 + (l >> 5) * 4 + (v & 3);
    const int n = (nb0 + j) * 32 + (l & 31);
    if (use_res && (QUADS % NT == 0 || e < TILE) && mm < p.M && n < p.Cout)
      res_pre[r] = *(const ResVec*)((const unsigned char*)p.res + ((size_t)mm * p.Cout + n) * ES);
  }

  f32x16 acc[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

  auto mma = [&](uint4 a4, const uint4* b) {
    if (BF16) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a4), __builtin_bit_cast(bf16x8, b[j]), acc[j], 0, 0, 0);
    } else {
      // the TN accumulators alternate so that consecutive MFMAs are independent
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a4.x), __uint_as_float(b[j].x), acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a4.y), __uint_as_float(b[j].y), acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a4.z), __uint_as_float(b[j].z), acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a4.w), __uint_as_float(b[j].w), acc[j], 0, 0, 0);
    }
  };
  auto compute = [&](int d) {
    uint4 a4 = keep_if(av[d], ar[d]);
    if (MODE == 2 && BF16) {  // four fp32 channels -> the 8-channel bf16 vector of the tap (same rounding as the conversion kernel)
      a4.x = f32_to_bf16_bits(__uint_as_float(a4.x)) | (f32_to_bf16_bits(__uint_as_float(a4.y)) << 16);
      a4.y = f32_to_bf16_bits(__uint_as_float(a4.z)) | (f32_to_bf16_bits(__uint_as_float(a4.w)) << 16);
      a4.z = 0u;
      a4.w = 0u;
    }
    mma(a4, br[d]);
  };

  // Software pipeline, D steps deep.  Every load in the prologue and in the steady-state loop is unconditional and
  // the loop is straight-line (compute slot d, refill slot d), so the compiler can count the loads in flight and
  // wait only for the oldest slot.  Refills past the end of the wave's K slice fetch valid memory that is never used
  // (the weight buffer carries D KiB of slack; the A pointer always points into the input); only the computes of the
  // ragged tail are conditional.
  if constexpr (!STAGED) {
#pragma unroll
    for (int d = 0; d < D; ++d) load(d);
    int done = 0;
    for (; done + D <= nsteps; done += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        compute(d);
        load(d);
      }
    }
#pragma unroll
    for (int d = 0; d < D; ++d)
      if (done + d < nsteps) compute(d);
  } else {
    // Staged pixel operand.  A load instruction is served 64 bytes per cycle only when four neighbouring lanes read one
    // 64-byte segment; the register-fed path above has every lane in a different pixel (a different cache line), which
    // makes the pixel operand cost four times the cycles of the same bytes of weights and binds the small layers to
    // the load unit instead of the matrix pipe.  Here a wave fetches, per chunk of two K steps, 64 contiguous bytes
    // of each of its 32 pixels as whole rows (lane = (pixel, 16-byte piece): 4 lanes per row, 16 rows per
    // instruction), parks them in its own corner of LDS, and reads them back in MFMA order (lane = pixel row, half =
    // K half).  No workgroup barrier is involved: the buffer is private to the wave.  Two chunks of rows and four steps
    // of weights are in flight.  The plan makes every wave's K slice a whole number of chunks.
    uint4* const st = reinterpret_cast<uint4*>(red) + wave * STAGE_V;
    const int piece = lane & 3, prow = lane >> 2;
    auto load_w = [&](int d) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        br[d][j] = *(const uint4*)wptr[j];
        wptr[j] += 1024;
      }
    };
    // rows in the wave's buffer -> MFMA order -> two K steps against the weights of pipeline slots d0, d0 + 1
    auto exchange_and_mma = [&](int d0) {
      // lanes exchange data through the wave's buffer: order the accesses of the whole wave, not only of each lane
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      uint4 a4[2];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) a4[s2] = st[li * 5 + 2 * s2 + lh];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        mma(a4[s2], br[d0 + s2]);
        load_w(d0 + s2);
      }
    };
    const int nchunks = nsteps >> 1;
    if constexpr (DWF) {
      // The 1x1 convolution's input row of pixel (y, x), channels c..c+VEC-1, is the depthwise layer's output there:
      // act(bias[c] + sum over the 3x3 taps inside the image, in (ky, kx) order, of in[y*stride-1+ky][x*stride-1+kx][c] * w[tap][c]),
      // accumulated with fused multiply-adds in exactly the order of dwconv_kernel, then rounded to the element type as a
      // stored tensor would be.  A lane computes the 16-byte piece it would otherwise have loaded.
      const unsigned char* dww = (const unsigned char*)dwf.w;
      int poff[2][9];     // element offset of each tap's input pixel (0 where the tap is outside: the value is not used)
      unsigned vmask[2];  // bit t: tap t of this lane's pixel lies inside the image
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int mj = m0 + 16 * j + prow;
        const bool okj = mj < p.M;
        const int y = fast_div(mj, p.mg_wo), x = mj - y * p.Wo;
        vmask[j] = 0u;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
          const int iy = y * dwf.stride - 1 + t / 3, ix = x * dwf.stride - 1 + t % 3;
          const bool v = okj && (unsigned)iy < (unsigned)dwf.H && (unsigned)ix < (unsigned)dwf.W;
          poff[j][t] = v ? (iy * dwf.W + ix) * p.Cin : 0;
          vmask[j] |= v ? (1u << t) : 0u;
        }
      }
      int cch = sbeg * KS;  // first channel of the wave's next chunk (wave-uniform)
      uint4 xv[2][9], wv[9];
      float4 bv[VEC / 4];
      auto dw_issue = [&]() {  // loads of the chunk at cch; past the end of the slice the last chunk of the tensor is read again (never used)
        const int c = min(cch, p.Cin - 2 * KS) + piece * VEC;
#pragma unroll
        for (int t = 0; t < 9; ++t) wv[t] = *(const uint4*)(dww + ((size_t)t * p.Cin + c) * ES);
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) bv[q] = *(const float4*)(dwf.bias + c + 4 * q);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int t = 0; t < 9; ++t) xv[j][t] = *(const uint4*)(xb + ((size_t)poff[j][t] + c) * ES);
        cch += 2 * KS;
      };
      auto dw_value = [&](int j) -> uint4 {
        float acc[VEC];
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
          acc[4 * q] = bv[q].x; acc[4 * q + 1] = bv[q].y; acc[4 * q + 2] = bv[q].z; acc[4 * q + 3] = bv[q].w;
        }
#pragma unroll
        for (int t = 0; t < 9; ++t) {
          float xf[VEC], wf[VEC];
          unpack<BF16>(xv[j][t], xf);
          unpack<BF16>(wv[t], wf);
          const bool v = (vmask[j] >> t) & 1u;
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[i] = v ? fmaf(xf[i], wf[i], acc[i]) : acc[i];
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = apply_act(acc[i], dwf.act);
        return pack<BF16>(acc);
      };
      auto chunk_dw = [&](int d0) {
#pragma unroll
        for (int j = 0; j < 2; ++j) st[(16 * j + prow) * 5 + piece] = dw_value(j);
        dw_issue();  // the next chunk's operands travel while this one goes through the matrix pipe
        exchange_and_mma(d0);
      };
      dw_issue();
#pragma unroll
      for (int d = 0; d < D; ++d) load_w(d);
      int c = 0;
      for (; c + 2 <= nchunks; c += 2) {
        chunk_dw(0);
        chunk_dw(2);
      }
      if (c < nchunks) chunk_dw(0);
    } else {
      int siy0[2], six0[2];
      bool sok[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int mj = m0 + 16 * j + prow;
        sok[j] = mj < p.M;
        const int y = fast_div(mj, p.mg_wo), x = mj - y * p.Wo;
        siy0[j] = y * p.stride - p.pad;
        six0[j] = x * p.stride - p.pad;
      }
      const unsigned char* gp[2];
      bool gv[2];
      auto enter_rows = [&]() {  // (ky, kx, ci) are wave-uniform
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int iy = siy0[j] + ky, ix = six0[j] + kx;
          gv[j] = sok[j] && ky < p.kh && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
          gp[j] = xb + ((size_t)(gv[j] ? iy * p.W + ix : 0) * p.Cin + ci) * ES + piece * 16;  // always a valid address
        }
      };
      enter_rows();
      uint4 gr[2][2];
      bool gok[2][2];
      auto load_rows = [&](int slot) {  // the chunk at (tap, ci) into register slot `slot`, then on to the next chunk
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          gr[slot][j] = *(const uint4*)gp[j];
          gok[slot][j] = gv[j];
        }
        ci += 2 * KS;
        if (ci >= p.Cin) {  // wave-uniform
          ci -= p.Cin;
          if (++kx == p.kw) { kx = 0; ++ky; }
          enter_rows();
        } else {
#pragma unroll
          for (int j = 0; j < 2; ++j) gp[j] += 64;
        }
      };
      // one chunk: rows of register slot `slot` -> LDS -> MFMA order; weights of pipeline slots d0, d0 + 1
      auto chunk = [&](int slot, int d0) {
#pragma unroll
        for (int j = 0; j < 2; ++j) st[(16 * j + prow) * 5 + piece] = keep_if(gok[slot][j], gr[slot][j]);
        load_rows(slot);  // two chunks ahead (past the end of the slice: valid memory, never used)
        exchange_and_mma(d0);
      };
      load_rows(0);
      load_rows(1);
#pragma unroll
      for (int d = 0; d < D; ++d) load_w(d);
      int c = 0;
      for (; c + 2 <= nchunks; c += 2) {
        chunk(0, 0);
        chunk(1, 2);
      }
      if (c < nchunks) chunk(0, 0);
    }
    __syncthreads();  // the partial tiles below reuse the LDS of every wave's staging buffer
  }

  // --- sum the NW partial tiles in wave order; tile element e = (j*16 + v)*64 + lane --------------------------------
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave * TILE + (j * 16 + v) * 64 + lane] = acc[j][v];
  __syncthreads();
  // --- epilogue per channel quad: pixel m0 + 8*(v/4) + 4*(lane/32) + v%4, channels 32*(nb0+j) + lane%32 .. +3 ---------
#pragma unroll
  for (int r = 0; r < RQ; ++r) {
    const int q = tid + r * NT;
    if (QUADS % NT != 0 && q >= QUADS) break;
    const int e = 4 * q;
    float4 sum = *(const float4*)&red[e];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
      const float4 t = *(const float4*)&red[w * TILE + e];
      sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
    }
    const int j = e >> 10, v = (e >> 6) & 15, l = e & 63;
    const int mm = m0 + (v >> 2) * 8 + (l >> 5) * 4 + (v & 3);
    const int n = (nb0 + j) * 32 + (l & 31);
    if (mm < p.M && n < p.Cout) {
      const size_t o = (size_t)mm * p.Cout + n;
      if (!own_epilogue) {  // partial sums of this K slice; splitk_reduce_kernel finishes the layer
        *(float4*)(p.ws + (size_t)zi * p.M * p.Cout + o) = sum;
      } else {
        float4 b = bias_j[0];  // component-wise select: indexing the array with a run-time j would move it out of registers
        if (TN == 2) {
          const bool hi = j != 0;
          b.x = hi ? bias_j[TN - 1].x : b.x; b.y = hi ? bias_j[TN - 1].y : b.y;
          b.z = hi ? bias_j[TN - 1].z : b.z; b.w = hi ? bias_j[TN - 1].w : b.w;
        }
        float val[4] = {sum.x + b.x, sum.y + b.y, sum.z + b.z, sum.w + b.w};
        if (use_res) {
          const ResVec rv = res_pre[r];
          if constexpr (BF16) {
            val[0] += __uint_as_float(rv.x << 16); val[1] += __uint_as_float(rv.x & 0xffff0000u);
            val[2] += __uint_as_float(rv.y << 16); val[3] += __uint_as_float(rv.y & 0xffff0000u);
          } else {
            val[0] += __uint_as_float(rv.x); val[1] += __uint_as_float(rv.y);
            val[2] += __uint_as_float(rv.z); val[3] += __uint_as_float(rv.w);
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) val[i] = apply_act(val[i], p.act);
        if (BF16) {
          uint2 out;
          out.x = f32_to_bf16_bits(val[0]) | (f32_to_bf16_bits(val[1]) << 16);
          out.y = f32_to_bf16_bits(val[2]) | (f32_to_bf16_bits(val[3]) << 16);
          *(uint2*)((uint16_t*)p.y + o) = out;
        } else {
          *(float4*)((float*)p.y + o) = make_float4(val[0], val[1], val[2], val[3]);
        }
      }
    }
  }
}

template <bool BF16, int TN, int NW, int MODE>
__global__ __launch_bounds__(NW * 64) void conv_wave_kernel(const ConvArgs p) {
  conv_wave_body<BF16, TN, NW, MODE>(p, (int)blockIdx.x, DwFusedArgs());
}

// A 1x1 convolution with the 3x3 depthwise convolution in front of it computed on the fly (gather mode 4): one launch for
// the second and third layer of an inverted residual block, and the depthwise output never touches memory.
template <bool BF16, int TN, int NW>
__global__ __launch_bounds__(NW * 64) void conv_wave_dw_kernel(const ConvArgs p, const DwFusedArgs d) {
  conv_wave_body<BF16, TN, NW, 4>(p, (int)blockIdx.x, d);
}
// Two independent convolutions of the same kernel variant in one launch (a residual block's first convolution and
// the 1x1 convolution of its shortcut read the same tensor): workgroups [0, n0) work on p0, the rest on p1.  n0 is
// a multiple of 8, so the workgroup -> XCD relation of each problem is the one its plan assumed.
template <bool BF16, int TN, int NW, int MODE>
__global__ __launch_bounds__(NW * 64) void conv_wave_pair_kernel(const ConvArgs p0, const ConvArgs p1, const int n0) {
  const int L = (int)blockIdx.x;
  if (L < n0) conv_wave_body<BF16, TN, NW, MODE>(p0, L, DwFusedArgs());
  else conv_wave_body<BF16, TN, NW, MODE>(p1, L - n0, DwFusedArgs());
}

// ---- 16-row wave tiles for deep, skinny layers -----------------------------------------------------------------------
//
// A layer with few output pixels and many channels (the 14x14 and 7x7 stages of a ResNet) has too few 32 x 32 tiles to
// fill a partition; the kernel above then splits K across workgroups and a second launch sums the partial tiles.  Here a
// wave owns 16 pixels x (16 * TB) channels (v_mfma_f32_16x16x4_f32 / 16x16x32_bf16): at the same matrix rate there are
// two to four times as many tiles, so the partition fills with K split only among the NW waves of a workgroup, the sum
// goes through LDS as before, and the reduction launch disappears.  One K step is 64 bytes of a pixel: lane (i, q) =
// (pixel row i = lane % 16, quarter q = lane / 16) loads the 16 bytes at k = step * KS + q * VEC, and the weights were
// packed at registration as [channel block of 16][step][lane (j, q)][16 B] with the same k order.  Cin is a multiple of
// KS, so a step never straddles a filter tap and the K walk is wave-uniform.
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool BF16, int TB, int NW>
__device__ __forceinline__ void conv_wave16_body(const ConvArgs& p, const int L) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int VEC = 16 / ES;
  constexpr int KS = 4 * VEC;  // k per step: 16 (fp32) / 32 (bf16)
  constexpr int TILE = TB * 256;
  constexpr int D = 4;
  constexpr int STAGE_V = 16 * 5;  // 16-byte vectors of one wave's staging buffer: 16 pixels x (4 pieces + 1 pad)
  constexpr int LDS_F = NW * STAGE_V * 4 > NW * TILE ? NW * STAGE_V * 4 : NW * TILE;
  static_assert(TB == 1 || TB == 2, "the epilogue selects between at most two channel blocks");

  __shared__ __align__(16) float red[LDS_F];

  if (p.wave_prio) __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lq = lane >> 4;
  int mt, g;  // workgroup -> (pixel tile, weight group), tiles that read the same weights on one XCD (see conv_wave_body)
  {
    const int x = L & 7, q = L >> 3;
    if (p.xmode == 1) {
      g = (q / p.MT) * 8 + x;
      mt = q % p.MT;
      if (g >= p.G) return;
    } else if (p.xmode == 2) {
      const int r = 8 / p.G;
      g = x / r;
      mt = q * r + (x % r);
      if (mt >= p.MT) return;
    } else {
      g = L / p.MT;
      mt = L % p.MT;
      if (g >= p.G) return;
    }
  }
  const int zi = g / p.NTn;
  const int m0 = mt * 16, nb0 = (g - zi * p.NTn) * TB;
  const int s_wg0 = zi * p.sz;
  const int s_wg1 = min(s_wg0 + p.sz, p.S);
  const int sbeg = min(s_wg0 + wave * p.sw, s_wg1);
  const int nsteps = min(sbeg + p.sw, s_wg1) - sbeg;

  // The pixel operand is fetched as whole 64-byte rows (lane = (pixel lane / 4, 16-byte piece lane % 4): four
  // neighbouring lanes read one contiguous row, the access shape the load unit serves at full rate) and turned into MFMA
  // order (lane = (pixel row, quarter)) through the wave's own corner of LDS, as in the staged mode of the 32-row kernel.
  const unsigned char* xb = (const unsigned char*)p.x;
  const int prow = lane >> 2, piece = lane & 3;
  const int m = m0 + prow;
  const bool a_ok = m < p.M;
  const int oy = fast_div(m, p.mg_wo), ox = m - oy * p.Wo;
  const int iy0 = oy * p.stride - p.pad, ix0 = ox * p.stride - p.pad;
  const int kcur = sbeg * KS;
  const int tap = fast_div(kcur, p.mg_cin);
  int ci = kcur - tap * p.Cin;
  int ky = fast_div(tap, p.mg_kw), kx = tap - ky * p.kw;
  bool a_valid;
  const unsigned char* ap;
  auto enter_tap = [&]() {
    const int iy = iy0 + ky, ix = ix0 + kx;
    a_valid = a_ok && ky < p.kh && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
    ap = xb + ((size_t)(a_valid ? iy * p.W + ix : 0) * p.Cin + ci) * ES + piece * 16;  // always a valid address
  };
  uint4* const st = reinterpret_cast<uint4*>(red) + wave * STAGE_V;
  enter_tap();
  const unsigned char* wptr[TB];
#pragma unroll
  for (int j = 0; j < TB; ++j) wptr[j] = (const unsigned char*)p.w + (((size_t)(nb0 + j) * p.S + sbeg) * 64 + lane) * 16;

  uint4 ar[D], br[D][TB];
  bool av[D];
  auto load = [&](int d) {
    ar[d] = *(const uint4*)ap;
    av[d] = a_valid;
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      br[d][j] = *(const uint4*)wptr[j];
      wptr[j] += 1024;
    }
    ci += KS;
    if (ci >= p.Cin) {  // wave-uniform
      ci -= p.Cin;
      if (++kx == p.kw) { kx = 0; ++ky; }
      enter_tap();
    } else {
      ap += KS * ES;
    }
  };

  // epilogue operands fetched ahead of the K loop: this thread's quad of consecutive channels (see below)
  constexpr int QUADS = TILE / 4;
  const bool has_quad = tid < QUADS;
  const int qe = 4 * tid;                                     // first tile element of the quad: (b * 4 + v) * 64 + lane
  const int qb = qe >> 8, qv = (qe >> 6) & 3, ql = qe & 63;
  const int qm = m0 + 4 * (ql >> 4) + qv;                      // pixel
  const int qn = (nb0 + qb) * 16 + (ql & 15);                  // first channel
  const bool q_ok = has_quad && qm < p.M && qn < p.Cout;
  const bool own_epilogue = p.splitk == 1;
  float4 bias = make_float4(0.f, 0.f, 0.f, 0.f);
  if (q_ok) bias = *(const float4*)(p.bias + qn);
  using ResVec = typename std::conditional<BF16, uint2, uint4>::type;
  ResVec res_pre = ResVec();
  const bool use_res = own_epilogue && p.res != nullptr;
  if (use_res && q_ok) res_pre = *(const ResVec*)((const unsigned char*)p.res + ((size_t)qm * p.Cout + qn) * ES);

  f32x4 acc[TB];
#pragma unroll
  for (int j = 0; j < TB; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[j][v] = 0.f;

  auto compute = [&](int d) {
    st[prow * 5 + piece] = keep_if(av[d], ar[d]);
    // lanes exchange data through the wave's buffer: order the accesses of the whole wave, not only of each lane
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint4 a4 = st[li * 5 + lq];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (BF16) {
#pragma unroll
      for (int j = 0; j < TB; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a4), __builtin_bit_cast(bf16x8, br[d][j]), acc[j], 0, 0, 0);
    } else {
#pragma unroll
      for (int j = 0; j < TB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a4.x), __uint_as_float(br[d][j].x), acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a4.y), __uint_as_float(br[d][j].y), acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a4.z), __uint_as_float(br[d][j].z), acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a4.w), __uint_as_float(br[d][j].w), acc[j], 0, 0, 0);
    }
  };

  // the same D-deep software pipeline as the 32-row kernel: unconditional loads, conditional computes only in the tail
#pragma unroll
  for (int d = 0; d < D; ++d) load(d);
  int done = 0;
  for (; done + D <= nsteps; done += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      compute(d);
      load(d);
    }
  }
#pragma unroll
  for (int d = 0; d < D; ++d)
    if (done + d < nsteps) compute(d);

  // partial tiles of the NW waves summed in wave order; accumulator v of lane l is pixel 4 * (l / 16) + v, channel l % 16
  __syncthreads();  // the partial tiles reuse the LDS of every wave's staging buffer
#pragma unroll
  for (int j = 0; j < TB; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave * TILE + (j * 4 + v) * 64 + lane] = acc[j][v];
  __syncthreads();
  if (!q_ok) return;
  float4 sum = *(const float4*)&red[qe];
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    const float4 t = *(const float4*)&red[w * TILE + qe];
    sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
  }
  const size_t o = (size_t)qm * p.Cout + qn;
  if (!own_epilogue) {
    *(float4*)(p.ws + (size_t)zi * p.M * p.Cout + o) = sum;
    return;
  }
  float val[4] = {sum.x + bias.x, sum.y + bias.y, sum.z + bias.z, sum.w + bias.w};
  if (use_res) {
    if constexpr (BF16) {
      val[0] += __uint_as_float(res_pre.x << 16); val[1] += __uint_as_float(res_pre.x & 0xffff0000u);
      val[2] += __uint_as_float(res_pre.y << 16); val[3] += __uint_as_float(res_pre.y & 0xffff0000u);
    } else {
      val[0] += __uint_as_float(res_pre.x); val[1] += __uint_as_float(res_pre.y);
      val[2] += __uint_as_float(res_pre.z); val[3] += __uint_as_float(res_pre.w);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) val[i] = apply_act(val[i], p.act);
  if (BF16) {
    uint2 out;
    out.x = f32_to_bf16_bits(val[0]) | (f32_to_bf16_bits(val[1]) << 16);
    out.y = f32_to_bf16_bits(val[2]) | (f32_to_bf16_bits(val[3]) << 16);
    *(uint2*)((uint16_t*)p.y + o) = out;
  } else {
    *(float4*)((float*)p.y + o) = make_float4(val[0], val[1], val[2], val[3]);
  }
}

template <bool BF16, int TB, int NW>
__global__ __launch_bounds__(NW * 64) void conv_wave16_kernel(const ConvArgs p) {
  conv_wave16_body<BF16, TB, NW>(p, (int)blockIdx.x);
}

// Two independent convolutions on one tensor in one launch, as conv_wave_pair_kernel: workgroups [0, n0) work on p0.
template <bool BF16, int TB, int NW>
__global__ __launch_bounds__(NW * 64) void conv_wave16_pair_kernel(const ConvArgs p0, const ConvArgs p1, const int n0) {
  const int L = (int)blockIdx.x;
  if (L < n0) conv_wave16_body<BF16, TB, NW>(p0, L);
  else conv_wave16_body<BF16, TB, NW>(p1, L - n0);
}

// ---- depthwise convolution: memory bound, one thread per (output pixel, 16-byte channel vector) -----------------------
template <bool BF16>
__global__ __launch_bounds__(256) void dwconv_kernel(const DwArgs a) {
  constexpr int VEC = BF16 ? 8 : 4;
  constexpr int ES = BF16 ? 2 : 4;
  const int cvn = a.C / VEC;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)a.Ho * a.Wo * cvn) return;
  const int cv = (int)(idx % cvn);
  const int m = (int)(idx / cvn);
  const int oy = m / a.Wo, ox = m - oy * a.Wo;
  const int c0 = cv * VEC;
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = a.bias[c0 + i];
  const unsigned char* xb = (const unsigned char*)a.x;
  const unsigned char* wb = (const unsigned char*)a.w;
  for (int ky = 0; ky < a.k; ++ky) {
    const int iy = oy * a.stride + ky - a.pad;
    if ((unsigned)iy >= (unsigned)a.H) continue;
    for (int kx = 0; kx < a.k; ++kx) {
      const int ix = ox * a.stride + kx - a.pad;
      if ((unsigned)ix >= (unsigned)a.W) continue;
      float xv[VEC], wv[VEC];
      unpack<BF16>(*(const uint4*)(xb + ((size_t)(iy * a.W + ix) * a.C + c0) * ES), xv);
      unpack<BF16>(*(const uint4*)(wb + ((size_t)(ky * a.k + kx) * a.C + c0) * ES), wv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] = fmaf(xv[i], wv[i], acc[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = apply_act(acc[i], a.act);
  *(uint4*)((unsigned char*)a.y + ((size_t)m * a.C + c0) * ES) = pack<BF16>(acc);
}

// ---- max pooling: padding acts as -inf --------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void maxpool_kernel(const PoolArgs a) {
  constexpr int VEC = BF16 ? 8 : 4;
  constexpr int ES = BF16 ? 2 : 4;
  const int cvn = a.C / VEC;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)a.Ho * a.Wo * cvn) return;
  const int cv = (int)(idx % cvn);
  const int m = (int)(idx / cvn);
  const int oy = m / a.Wo, ox = m - oy * a.Wo;
  const int c0 = cv * VEC;
  float best[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) best[i] = -INFINITY;
  const unsigned char* xb = (const unsigned char*)a.x;
  for (int ky = 0; ky < a.k; ++ky) {
    const int iy = oy * a.stride + ky - a.pad;
    if ((unsigned)iy >= (unsigned)a.H) continue;
    for (int kx = 0; kx < a.k; ++kx) {
      const int ix = ox * a.stride + kx - a.pad;
      if ((unsigned)ix >= (unsigned)a.W) continue;
      float xv[VEC];
      unpack<BF16>(*(const uint4*)(xb + ((size_t)(iy * a.W + ix) * a.C + c0) * ES), xv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) best[i] = fmaxf(best[i], xv[i]);
    }
  }
  *(uint4*)((unsigned char*)a.y + ((size_t)m * a.C + c0) * ES) = pack<BF16>(best);
}

// ---- global average pooling: 64 channels per workgroup, 4 threads per channel over the pixels, LDS sum --------------
template <bool BF16>
__global__ __launch_bounds__(256) void gavgpool_kernel(const PoolArgs a) {
  __shared__ float part[4][64];
  const int cl = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const int hw = a.H * a.W;
  float s = 0.f;
  if (c < a.C)
    for (int i = q; i < hw; i += 4) s += load_elem<BF16>(a.x, (size_t)i * a.C + c);
  part[q][cl] = s;
  __syncthreads();
  if (q == 0 && c < a.C) store_elem<BF16>(a.y, c, (part[0][cl] + part[1][cl] + part[2][cl] + part[3][cl]) / (float)hw);
}

// ---- FC, batch 1: one wave per output, 16-byte loads along K, butterfly reduction ------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void fc_kernel(const FcArgs a) {
  constexpr int VEC = BF16 ? 8 : 4;
  constexpr int ES = BF16 ? 2 : 4;
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= a.Ns) return;
  if (n >= a.N) {  // pad element of the output vector
    if (lane == 0) store_elem<BF16>(a.y, n, 0.f);
    return;
  }
  const unsigned char* wrow = (const unsigned char*)a.w + (size_t)n * a.K * ES;
  const unsigned char* xb = (const unsigned char*)a.x;
  const int nvec = a.K / VEC;
  // Short rows are latency-bound: four independent 16-byte weight loads in flight per lane, each with its own partial sum.
  // Long rows (VGG-16's first FC: 100 KB per wave, 411 MB in all) are pure streaming and run at the memory system's
  // rate with one load per lane; more loads in flight slowed them down (measured: 84 -> 110 us), so they keep the plain loop.
  float acc4[4] = {0.f, 0.f, 0.f, 0.f};
  int v = lane;
  if (nvec <= 2048) {
    for (; v + 192 < nvec; v += 256) {
      uint4 wq[4], xq[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) wq[u] = *(const uint4*)(wrow + (size_t)(v + 64 * u) * 16);
#pragma unroll
      for (int u = 0; u < 4; ++u) xq[u] = *(const uint4*)(xb + (size_t)(v + 64 * u) * 16);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float wv[VEC], xv[VEC];
        unpack<BF16>(wq[u], wv);
        unpack<BF16>(xq[u], xv);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc4[u] = fmaf(wv[i], xv[i], acc4[u]);
      }
    }
  }
  for (; v < nvec; v += 64) {
    float wv[VEC], xv[VEC];
    unpack<BF16>(*(const uint4*)(wrow + (size_t)v * 16), wv);
    unpack<BF16>(*(const uint4*)(xb + (size_t)v * 16), xv);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc4[0] = fmaf(wv[i], xv[i], acc4[0]);
  }
  float acc = (acc4[0] + acc4[1]) + (acc4[2] + acc4[3]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (lane == 0) {
    const float v = apply_act(acc + a.bias[n], a.act);
    if (a.out_f32) ((float*)a.y)[n] = v;
    else store_elem<BF16>(a.y, n, v);
  }
}

// ---- boundary conversions ------------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void ingest_kernel(const float* __restrict__ x, void* y, int C, int Cs, int HW) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)HW * Cs) return;
  const int c = (int)(idx % Cs);
  const size_t px = idx / Cs;
  store_elem<BF16>(y, idx, c < C ? x[(size_t)c * HW + px] : 0.f);
}

template <bool BF16>
__global__ __launch_bounds__(256) void egress_kernel(const void* x, float* __restrict__ y, int C, int Cs, int HW) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)HW * C) return;
  const int c = (int)(idx / HW);
  const size_t px = idx % HW;
  y[idx] = load_elem<BF16>(x, px * Cs + c);
}

// ---- CU mask probe: which XCC / CU did each workgroup run on ----------------------------------------------------------------
__global__ __launch_bounds__(64) void cu_probe_kernel(uint32_t* out, int spin) {
  uint32_t xcc, hwid;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid));
  // bounded busy wait so that the workgroups of one launch spread over every CU the mask allows
  for (int i = 0; i < spin; ++i) __builtin_amdgcn_s_sleep(8);
  if (threadIdx.x == 0) {
    out[2 * blockIdx.x] = xcc;
    out[2 * blockIdx.x + 1] = hwid;
  }
}

// ---- explicit instantiations: the host never references the kernels (they are dispatched by name from the code object) --------
#define DARIS_INST_CONV(B, TN_, NW_)                                                              \
  template __global__ void conv_wave_kernel<B, TN_, NW_, 0>(const ConvArgs);                      \
  template __global__ void conv_wave_kernel<B, TN_, NW_, 1>(const ConvArgs);                      \
  template __global__ void conv_wave_kernel<B, TN_, NW_, 2>(const ConvArgs);                      \
  template __global__ void conv_wave_kernel<B, TN_, NW_, 3>(const ConvArgs);                      \
  template __global__ void conv_wave_pair_kernel<B, TN_, NW_, 0>(const ConvArgs, const ConvArgs, const int); \
  template __global__ void conv_wave_pair_kernel<B, TN_, NW_, 1>(const ConvArgs, const ConvArgs, const int); \
  template __global__ void conv_wave_pair_kernel<B, TN_, NW_, 3>(const ConvArgs, const ConvArgs, const int);
#define DARIS_INST_CONV16(B, TB_)                                                                  \
  template __global__ void conv_wave16_kernel<B, TB_, 2>(const ConvArgs);                          \
  template __global__ void conv_wave16_kernel<B, TB_, 4>(const ConvArgs);                          \
  template __global__ void conv_wave16_kernel<B, TB_, 8>(const ConvArgs);                          \
  template __global__ void conv_wave16_pair_kernel<B, TB_, 2>(const ConvArgs, const ConvArgs, const int); \
  template __global__ void conv_wave16_pair_kernel<B, TB_, 4>(const ConvArgs, const ConvArgs, const int); \
  template __global__ void conv_wave16_pair_kernel<B, TB_, 8>(const ConvArgs, const ConvArgs, const int);
#define DARIS_INST_CONVDW(B, TN_, NW_)                                                             \
  template __global__ void conv_wave_dw_kernel<B, TN_, NW_>(const ConvArgs, const DwFusedArgs);
#define DARIS_INST_ALL(B)                                                                          \
  DARIS_INST_CONV(B, 1, 2) DARIS_INST_CONV(B, 1, 4) DARIS_INST_CONV(B, 1, 8)                        \
  DARIS_INST_CONV(B, 2, 2) DARIS_INST_CONV(B, 2, 4) DARIS_INST_CONV(B, 2, 8)                        \
  DARIS_INST_CONV16(B, 1) DARIS_INST_CONV16(B, 2)                                                   \
  template __global__ void splitk_reduce_kernel<B>(const float*, const float*, const void*, void*, int, int, int, int); \
  template __global__ void dwconv_kernel<B>(const DwArgs);                                         \
  template __global__ void maxpool_kernel<B>(const PoolArgs);                                      \
  template __global__ void gavgpool_kernel<B>(const PoolArgs);                                     \
  template __global__ void fc_kernel<B>(const FcArgs);                                             \
  template __global__ void ingest_kernel<B>(const float*, void*, int, int, int);                   \
  template __global__ void egress_kernel<B>(const void*, float*, int, int, int);
DARIS_INST_ALL(false)
DARIS_INST_ALL(true)
// Fused depthwise variants.  fp32 tiles of 64 channels are never staged, so they have none; bf16 plans never use 8 waves per
// workgroup, and those variants would need scratch memory, which the dispatch path does not provide.
DARIS_INST_CONVDW(false, 1, 2) DARIS_INST_CONVDW(false, 1, 4) DARIS_INST_CONVDW(false, 1, 8)
DARIS_INST_CONVDW(true, 1, 2) DARIS_INST_CONVDW(true, 1, 4) DARIS_INST_CONVDW(true, 2, 2) DARIS_INST_CONVDW(true, 2, 4)
#undef DARIS_INST_CONVDW
#undef DARIS_INST_ALL
#undef DARIS_INST_CONV
#undef DARIS_INST_CONV16

}  // namespace daris
