// Host side of the C ABI declared in include/bolt.h: descriptor validation, instance tables,
// the built-in pick rule, the light-weight profiler (Section 3.2.2), and the small helper kernels
// (channel padding, split-K reduction, roofline probes).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/bolt.h"
#include "instances.hpp"

namespace bolt {

static constexpr int kNumCU = 256;            // MI355X compute units
static constexpr int kLdsPerCU = 160 * 1024;  // bytes of LDS per compute unit / per workgroup
static constexpr int kMaxSplitK = 8;

// ------------------------------------------------------------------------------------------
// helper kernels
// ------------------------------------------------------------------------------------------

// Sums split-K partials and applies the epilogue once.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* partial, const half_t* bias, half_t* Y,
                                                            int M, int N, int ldy, int split_k, float alpha,
                                                            float beta, int act, const half_t* res, int ldr,
                                                            float gamma) {
  const int64_t quads = (int64_t)M * (N / 4);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < quads; i += (int64_t)gridDim.x * blockDim.x) {
    const int m = (int)(i / (N / 4)), n = (int)(i % (N / 4)) * 4;
    floatx4 s = {0.f, 0.f, 0.f, 0.f};
    for (int zz = 0; zz < split_k; ++zz) s += *(const floatx4*)(partial + ((int64_t)zz * M + m) * N + n);
    half4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float v = alpha * s[e];
      if (bias) v += beta * (float)bias[n + e];
      if (res) v += gamma * (float)res[(int64_t)m * ldr + n + e];
      o[e] = (half_t)apply_act(v, act);
    }
    *(half4*)(Y + (int64_t)m * ldy + n) = o;
  }
}

// Kernel padding (Section 3.2.3): one thread writes one 16-byte chunk of the padded tensor.  An even
// channel count is read as 32-bit pairs (a pair never straddles the end of a pixel), an odd one half
// by half.  The host guarantees pixels * C8 / 8 < 2^31.
template <bool EVEN>
__global__ __launch_bounds__(256) void pad_channels_kernel(const half_t* src, half_t* dst, int pixels, int C, int C8) {
  const int chunks = C8 / 8;
  const int total = pixels * chunks;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    const int pix = i / chunks;
    const int c0 = (i - pix * chunks) * 8;
    const half_t* s = src + (int64_t)pix * C + c0;
    half8 v;
    if constexpr (EVEN) {
      uintx4 u;
#pragma unroll
      for (int e = 0; e < 4; ++e) u[e] = (c0 + 2 * e < C) ? *(const unsigned*)(s + 2 * e) : 0u;
      v = __builtin_bit_cast(half8, u);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (c0 + e < C) ? s[e] : (half_t)0.f;
    }
    *(half8*)(dst + (int64_t)pix * C8 + c0) = v;
  }
}

// Layout transformation (Section 3.2.3): NCHW <-> NHWC through a 64-channel x 64-pixel LDS tile, so that both
// sides are coalesced: 128-byte runs of consecutive pixels of one channel plane on the NCHW side, 16-byte
// chunks of 8 consecutive channels (128 bytes per pixel) on the NHWC side.  Channels C .. C8-1 of the NHWC
// tensor are written as zeros (kernel padding in the same pass).  grid = (pixel tiles, channel tiles, N).
static constexpr int kLayoutTile = 64, kLayoutPitch = 66;  // LDS row pitch in halves: 33 words, conflict-free columns
__global__ __launch_bounds__(256) void nchw_to_nhwc_kernel(const half_t* src, half_t* dst, int C, int HW, int C8) {
  __shared__ half_t tile[kLayoutTile * kLayoutPitch];  // [channel][pixel]
  const int t = threadIdx.x, p0 = blockIdx.x * kLayoutTile, c0 = blockIdx.y * kLayoutTile;
  const int64_t n = blockIdx.z;
  {
    const int p = t & 63;
#pragma unroll 4
    for (int c = t >> 6; c < kLayoutTile; c += 4) {
      const bool ok = c0 + c < C && p0 + p < HW;
      tile[c * kLayoutPitch + p] = ok ? src[(n * C + c0 + c) * HW + p0 + p] : (half_t)0.f;
    }
  }
  __syncthreads();
  const int ch = t & 7;
#pragma unroll
  for (int p = t >> 3; p < kLayoutTile; p += 32) {
    if (p0 + p < HW && c0 + ch * 8 < C8) {
      half8 v;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = tile[(ch * 8 + e) * kLayoutPitch + p];
      *(half8*)(dst + (n * HW + p0 + p) * C8 + c0 + ch * 8) = v;
    }
  }
}

// The same for thin tensors (C <= 8, a network's input image): one thread per pixel reads its C channel planes
// (consecutive threads read consecutive pixels: coalesced) and writes one 16-byte chunk.
__global__ __launch_bounds__(256) void nchw_to_nhwc8_kernel(const half_t* src, half_t* dst, int C, int HW, int64_t pixels) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < pixels; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t n = i / HW, p = i - n * HW;
    half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < 8; ++c)
      if (c < C) v[c] = src[(n * C + c) * HW + p];
    *(half8*)(dst + i * 8) = v;
  }
}

// src holds Cs >= C channels per pixel (Cs % 8 == 0); the first C are kept.
__global__ __launch_bounds__(256) void nhwc_to_nchw_kernel(const half_t* src, half_t* dst, int C, int HW, int Cs) {
  __shared__ half_t tile[kLayoutTile * kLayoutPitch];  // [channel][pixel]
  const int t = threadIdx.x, p0 = blockIdx.x * kLayoutTile, c0 = blockIdx.y * kLayoutTile;
  const int64_t n = blockIdx.z;
  {
    const int ch = t & 7;
#pragma unroll
    for (int p = t >> 3; p < kLayoutTile; p += 32) {
      half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (p0 + p < HW && c0 + ch * 8 < Cs) v = *(const half8*)(src + (n * HW + p0 + p) * Cs + c0 + ch * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) tile[(ch * 8 + e) * kLayoutPitch + p] = v[e];
    }
  }
  __syncthreads();
  const int p = t & 63;
#pragma unroll 4
  for (int c = t >> 6; c < kLayoutTile; c += 4)
    if (c0 + c < C && p0 + p < HW) dst[(n * C + c0 + c) * HW + p0 + p] = tile[c * kLayoutPitch + p];
}

// Stand-alone epilogue (the un-fused baseline of Section 4.1.1): one thread rewrites one 16-byte
// chunk of D in place, D = act(alpha * D + beta * bias[n]).  ldd and N are multiples of 8.
__global__ __launch_bounds__(256) void bias_act_kernel(half_t* D, const half_t* bias, int64_t M, int N, int ldd,
                                                       float alpha, float beta, int act) {
  const int chunks = N / 8;
  const int64_t total = M * chunks;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t m = i / chunks;
    const int n0 = (int)(i - m * chunks) * 8;
    half8* p = (half8*)(D + m * ldd + n0);
    const half8 v = *p;
    half8 b = {0, 0, 0, 0, 0, 0, 0, 0};
    if (bias) b = *(const half8*)(bias + n0);
    half8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (half_t)apply_act(alpha * (float)v[e] + beta * (float)b[e], act);
    *p = o;
  }
}

// MFMA-only loop, no memory traffic: the measured ceiling of the matrix pipes under the chip's power limit.
// v_mfma_f32_16x16x32_f16 (the instruction of the ping-pong kernel) on operands that look like data: the
// sustained rate depends on how many operand bits toggle (all-zero operands run at the nominal 2.5 PFLOP/s, random
// halves at about 1.9-2.0 with this instruction and 1.7 with the 32 x 32 x 16 form).  Six operand registers and
// 16 independent accumulators per wave, cycled as a 128 x 64 wave tile would use them.
__global__ __launch_bounds__(256) void mfma_peak_kernel(float* sink, int iters) {
  half8 x[4], w[4];
  unsigned z = 0x9E3779B9u * (threadIdx.x + 1) + blockIdx.x;
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 8; ++e) {
      z = z * 1664525u + 1013904223u;
      x[i][e] = (half_t)((float)(z >> 8) * (2.f / 16777216.f) - 1.f);
      z = z * 1664525u + 1013904223u;
      w[i][e] = (half_t)((float)(z >> 8) * (2.f / 16777216.f) - 1.f);
    }
  floatx4 c[4][4];
  for (int a = 0; a < 4; ++a)
    for (int b = 0; b < 4; ++b) c[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) c[a][b] = mfma_16x16x32(w[a], x[b], c[a][b]);
  }
  float s = 0.f;
  for (int a = 0; a < 4; ++a)
    for (int b = 0; b < 4; ++b)
      for (int e = 0; e < 4; ++e) s += c[a][b][e];
  if (s == 123.456f) sink[0] = s;  // keeps the loop alive; practically never true
}

__global__ __launch_bounds__(256) void copy_kernel(const floatx4* src, floatx4* dst, int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// Eight zero halves: what a kernel's bias pointer addresses when the caller gave no bias.
__device__ __attribute__((aligned(16))) half_t g_zero_bias[8];

static const half_t* zero_bias() {
  static const half_t* ptr = [] {
    void* q = nullptr;
    return hipGetSymbolAddress(&q, HIP_SYMBOL(g_zero_bias)) == hipSuccess ? (const half_t*)q : nullptr;
  }();
  return ptr;
}

// Split-K partial sums of bolt_gemm_epilogue_noalloc: a file-scope device array, so that entry point never
// allocates.  Every GPU the library runs on holds its own copy (at its own address) until the process ends.
static __device__ __align__(256) unsigned char scratch[BOLT_NOALLOC_SCRATCH_BYTES];

// The array's name is a host-side stand-in, not a device address: host code only ever uses the pointer that
// hipGetSymbolAddress returns for the current device, looked up once per device.
static constexpr int kMaxDevices = 64;
static void* scratch_of_current_device() {
  static std::once_flag once[kMaxDevices];
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::call_once(once[dev], [dev] {
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) == hipSuccess) ptr[dev] = q;
  });
  return ptr[dev];
}

// ------------------------------------------------------------------------------------------
// instance tables
// ------------------------------------------------------------------------------------------
struct Tables {
  std::vector<FpropInstance> gemm, conv;
  std::vector<B2bInstance> b2b_gemm, b2b_conv;
  std::vector<ChainInstance> gemm_chain, conv_chain;
  Tables() {
    register_gemm_chain_instances(gemm_chain);
    register_conv_chain_instances(conv_chain);
    register_gemm_kn_instances(gemm);
    register_gemm_nk_instances(gemm);
    register_gemm_kn_dma_instances(gemm);  // (after the older families: their kernel ids stay what they were)
    register_conv_instances(conv);
    register_conv_halo_instances(conv);
    register_gemm_nk_instances(conv);  // for 1x1 / stride 1 / pad 0 filters
    register_conv_align2_instances(conv);  // even channel counts that are not multiples of 8
    register_conv_smallc_instances(conv);  // first layers: at most 4 channels, unpadded NHWC or NCHW
    register_conv_nchw_out_instances(conv);  // last layers: the output written as NCHW
    register_b2b_gemm_instances(b2b_gemm);
    register_b2b_gemm_dma_instances(b2b_gemm);
    register_b2b_gemm_dma_kn_instances(b2b_gemm);
    register_b2b_conv_instances(b2b_conv);
    register_b2b_conv_dma_instances(b2b_conv);
    register_b2b_conv_halo_instances(b2b_conv);
  }
};
static const Tables& tables() {
  static Tables t;
  return t;
}

static inline bool is_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline bool valid_act(int a) { return a >= BOLT_ACT_NONE && a <= BOLT_ACT_SOFTPLUS; }

// ------------------------------------------------------------------------------------------
// validation (no GPU needed)
// ------------------------------------------------------------------------------------------
static bolt_status check_gemm_desc(const bolt_gemm_desc* d) {
  if (!d) return BOLT_ERR_INVALID_ARG;
  if (d->M <= 0 || d->N <= 0 || d->K <= 0) return BOLT_ERR_INVALID_ARG;
  if (!valid_act(d->act)) return BOLT_ERR_INVALID_ARG;
  if (d->b_layout != BOLT_LAYOUT_KN && d->b_layout != BOLT_LAYOUT_NK) return BOLT_ERR_INVALID_ARG;
  if (d->lda < d->K || d->ldd < d->N) return BOLT_ERR_INVALID_ARG;
  if (d->b_layout == BOLT_LAYOUT_KN ? d->ldb < d->N : d->ldb < d->K) return BOLT_ERR_INVALID_ARG;
  if ((d->N | d->K | d->lda | d->ldb | d->ldd) & 7) return BOLT_ERR_ALIGNMENT;
  if (d->lda > (1 << 21) || d->ldb > (1 << 21) || d->ldd > (1 << 21)) return BOLT_ERR_UNSUPPORTED;
  return BOLT_OK;
}

struct ConvDims {
  int P, Q, M, Kg;
};

static bolt_status check_conv_desc(const bolt_conv_desc* d, ConvDims* out) {
  if (!d) return BOLT_ERR_INVALID_ARG;
  if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0)
    return BOLT_ERR_INVALID_ARG;
  if (d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0) return BOLT_ERR_INVALID_ARG;
  if (!valid_act(d->act)) return BOLT_ERR_INVALID_ARG;
  if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return BOLT_ERR_INVALID_ARG;
  if (d->x_layout != BOLT_TENSOR_NHWC && d->x_layout != BOLT_TENSOR_NCHW) return BOLT_ERR_INVALID_ARG;
  if (d->y_layout != BOLT_TENSOR_NHWC && d->y_layout != BOLT_TENSOR_NCHW) return BOLT_ERR_INVALID_ARG;
  // C % 8 == 0 is the fast path (128-bit accesses); an even C runs on the alignment-2 instances; C <= 4 (any
  // parity, either input layout) on the first-layer instances
  if ((d->K & 7) || ((d->C & 1) && d->C > 4)) return BOLT_ERR_ALIGNMENT;
  if (d->x_layout == BOLT_TENSOR_NCHW && d->C > 4) return BOLT_ERR_UNSUPPORTED;
  const int64_t P = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1;
  const int64_t Q = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
  const int64_t M = (int64_t)d->N * P * Q;
  const int64_t Kg = (int64_t)d->R * d->S * d->C;
  const int64_t in_elems = (int64_t)d->N * d->H * d->W * d->C;
  // the kernels address the input through one buffer descriptor (< 2 GiB), index outputs with
  // 32-bit element offsets and pack window origins in 16 bits
  if (d->H > 16384 || d->W > 16384 || d->pad_h > 8192 || d->pad_w > 8192) return BOLT_ERR_UNSUPPORTED;
  if (in_elems >= (1ll << 30) || M * d->K >= (1ll << 31) || M >= (1ll << 30) || Kg >= (1 << 24))
    return BOLT_ERR_UNSUPPORTED;
  if (out) *out = {(int)P, (int)Q, (int)M, (int)Kg};
  return BOLT_OK;
}

static ConvGeom make_geom(const bolt_conv_desc* d, const ConvDims& cd) {
  ConvGeom g;
  g.H = d->H; g.Wi = d->W; g.C = d->C; g.R = d->R; g.S = d->S; g.P = cd.P; g.Q = cd.Q;
  g.stride_h = d->stride_h; g.stride_w = d->stride_w; g.pad_h = d->pad_h; g.pad_w = d->pad_w;
  return g;
}

static bolt_status check_b2b_gemm(const bolt_gemm_desc* g0, const bolt_gemm_desc* g1) {
  if (!g0 || !g1) return BOLT_ERR_INVALID_ARG;
  bolt_gemm_desc a = *g0, b = *g1;
  a.ldd = a.N;  // D0 is never stored: its leading dimension is irrelevant
  b.lda = b.K;
  bolt_status s = check_gemm_desc(&a);
  if (s != BOLT_OK) return s;
  s = check_gemm_desc(&b);
  if (s != BOLT_OK) return s;
  if (g1->M != g0->M || g1->K != g0->N) return BOLT_ERR_ILLEGAL_FUSION;
  if (g0->b_layout != g1->b_layout) return BOLT_ERR_UNSUPPORTED;
  return BOLT_OK;
}

static bolt_status check_b2b_conv(const bolt_conv_desc* c0, const bolt_conv_desc* c1, ConvDims* cd0) {
  ConvDims d0, d1;
  bolt_status s = check_conv_desc(c0, &d0);
  if (s != BOLT_OK) return s;
  s = check_conv_desc(c1, &d1);
  if (s != BOLT_OK) return s;
  if (c0->C & 7) return BOLT_ERR_ALIGNMENT;  // the fused kernels have no alignment-2 form
  if (c0->x_layout != BOLT_TENSOR_NHWC || c0->y_layout != BOLT_TENSOR_NHWC || c1->x_layout != BOLT_TENSOR_NHWC ||
      c1->y_layout != BOLT_TENSOR_NHWC)
    return BOLT_ERR_UNSUPPORTED;  // fused pairs and chains compute and store NHWC only
  if (c1->R != 1 || c1->S != 1 || c1->stride_h != 1 || c1->stride_w != 1 || c1->pad_h != 0 || c1->pad_w != 0)
    return BOLT_ERR_ILLEGAL_FUSION;
  if (c1->C != c0->K || c1->N != c0->N || c1->H != d0.P || c1->W != d0.Q) return BOLT_ERR_ILLEGAL_FUSION;
  if (cd0) *cd0 = d0;
  return BOLT_OK;
}

// ------------------------------------------------------------------------------------------
// single-op problems
// ------------------------------------------------------------------------------------------
struct FpropProblem {
  FpropParams p;  // pointers filled in at launch
  int xmode, wmode;
  bool residual;  // the call carries a residual matrix (Eq. 1's C): kernels without that epilogue are excluded
};

static bool fprop_supports(const FpropInstance& in, const FpropProblem& pr) {
  if (in.xmode == 4) {
    // first-layer kernels: at most 4 channels of any parity, NHWC or NCHW input, weights [K][R][S][C] as they are; no
    // residual epilogue.  The geometry test is the instance's own.
    const bool small_nhwc = pr.xmode == 2 && pr.p.cg.C <= 4;
    return (pr.xmode == 4 || small_nhwc) && !pr.residual && in.dyn_supports(pr.p);  // either output layout
  }
  // an NCHW output: only the instances with that store, and they have no other; no residual form
  if ((pr.p.y_nchw != 0) != in.nchw_out) return false;
  if (in.nchw_out && pr.residual) return false;
  if (in.wmode != pr.wmode) return false;
  if (in.xmode != pr.xmode) return false;
  if (in.kn_dma && (int64_t)pr.p.K * pr.p.ldw * 2 >= (1ll << 31)) return false;
  if (in.dyn_supports && (!in.dyn_supports(pr.p) || in.dyn_lds_bytes(pr.p) > kLdsPerCU)) return false;
  if (in.lds_bytes > kLdsPerCU) return false;
  // single-stage instances hold exactly one k-tile per k-group
  if (in.stages == 1 && ceil_div(pr.p.K, in.bk) > std::max(1, in.kgroups)) return false;
  // a tile more than half empty along N is never worth timing (64 is the narrowest tile family)
  if (in.bn > 64 && in.bn / 2 >= pr.p.N) return false;
  return true;
}

static void fprop_fill_config(const FpropInstance& in, int id, bolt_config* c) {
  c->kernel_id = id;
  c->tile_m = in.bm; c->tile_n = in.bn; c->tile_k = in.bk;
  c->waves_m = in.waves_m; c->waves_n = in.waves_n;
  c->mfma_shape = in.mi ? in.mi : 32; c->stages = in.stages; c->b2b_mode = 0;
}

// Built-in pick rule (a caller that passes no config and does not tune): the smallest estimated time, in
// microseconds, under a model of three overlapping parts plus a launch floor,
//   matrix work   tiles a compute unit runs one after the other x MACs of a tile (whole k-tiles) / (rate x eff), where
//                 eff = 1 / (1 + 71 (1 / wave_tile_m + 1 / wave_tile_n)) stands for the FLOP per LDS byte of the wave tile;
//   tile traffic  the same tiles' operands through the L2;
//   latency chain of one workgroup, prologue + k-tile steps (+ the k-groups' reduction), repeated once per round of
//                 co-resident workgroups;
//   memory        every tensor once at the bandwidth the kernels sustain.
// The constants are a fit to the per-instance timings of 53 problems - the ResNet-50 layers at batch 32 and a few
// other batches, the GEMM shapes of Section 4 in both weight layouts, 1671 measurements: least squares on log time,
// then perturbed for the smallest mean time of the pick over the fastest instance.  bolt_tune measures instead.
// The halo, single-stage and ping-pong kernels have no partial-sum output.
static bool fprop_can_split_k(const FpropInstance& in) {
  return !in.dyn_supports && in.stages != 1 && !in.no_split_k;
}

// BOLT_TUNE_LOG=1 in the environment prints every candidate's time (bolt_tune) or estimated cost (the built-in pick
// rule) to stderr.
static bool tune_log_enabled() {
  static const bool on = [] { const char* e = std::getenv("BOLT_TUNE_LOG"); return e && e[0] && e[0] != '0'; }();
  return on;
}

// need_split_k: only instances that can write partial sums qualify (the caller asked for split-K).
static int fprop_heuristic(const std::vector<FpropInstance>& tab, const FpropProblem& pr, bool need_split_k = false) {
  int best = -1;
  double best_cost = 0;
  for (int i = 0; i < (int)tab.size(); ++i) {
    const FpropInstance& in = tab[i];
    if (!fprop_supports(in, pr)) continue;
    if (need_split_k && !fprop_can_split_k(in)) continue;
    const FpropParams& p = pr.p;
    const double tiles = (double)ceil_div(p.M, in.bm) * ceil_div(p.N, in.bn);
    const int kg = std::max(1, in.kgroups);
    const int lds = in.dyn_lds_bytes ? in.dyn_lds_bytes(p) : in.lds_bytes;
    const int per_cu = std::max(1, std::min(kLdsPerCU / lds, 2048 / (64 * in.waves_m * in.waves_n * kg) / 2));
    const bool pingpong = in.mi == 16 && in.bn == 256, halo = !pingpong && in.dyn_supports && in.xmode == 1;
    const bool reg_staged = in.wmode == 1 && !in.kn_dma;  // the slow cover of the direct-to-LDS row-major kernels
    const double nk = ceil_div(p.K, in.bk), kpad = nk * in.bk;
    const double wtm = (double)in.bm / in.waves_m, wtn = (double)in.bn / in.waves_n;
    const double eff = 1.0 / (1.0 + 71.0 * (1.0 / wtm + 1.0 / wtn));
    const double family = reg_staged ? 1.95 : pingpong ? 0.88 : halo ? 0.84 : 1.0;
    const double seq = std::ceil(tiles / kNumCU);  // tiles a compute unit runs one after the other
    const double t_mfma = seq * in.bm * in.bn * kpad / eff / 7.99e6 * family;
    // one workgroup's chain: prologue, k-tile steps (a deeper pipeline hides more of each), the k-groups' reduction
    const double step = 0.526 * std::pow(2.0 / std::max(2, in.stages), 0.85);
    const double t_lat = std::ceil(tiles / (kNumCU * per_cu)) * (1.66 + nk / kg * step + (kg - 1) * 0.32);
    // operand tiles through the L2: (bm + bn) x bk halves per k-tile of every tile
    const double t_l2 = seq * nk * (in.bm + in.bn) * in.bk * 2.0 / 1.95e5;
    // activations: a 1x1 / stride 1 filter or a GEMM reads M x K, a filter window re-reads its pixels out of cache
    double in_halves = (double)p.M * p.K;
    if (pr.xmode != 0 && p.cg.C > 0) in_halves = (double)p.M * std::min<double>(p.K, (double)p.cg.C * p.cg.stride_h * p.cg.stride_w);
    const double t_mem = 2.0 * (in_halves + (double)p.N * p.K + (double)p.M * p.N) / 6.43e6;
    const double cost = 2.85 + (std::max(std::max(t_mfma, t_l2), std::max(t_lat, t_mem)) + 0.3 * std::min(t_mfma, t_lat)) *
                                   std::pow((double)in.bm / in.bn, 0.01);
    if (tune_log_enabled()) std::fprintf(stderr, "[bolt_pick] candidate %d %s cost %.4g\n", i, in.name, cost);
    if (best < 0 || cost < best_cost) { best = i; best_cost = cost; }
  }
  if (tune_log_enabled() && best >= 0) std::fprintf(stderr, "[bolt_pick] -> %d %s\n", best, tab[best].name);
  return best;
}

static size_t splitk_bytes(int M, int N, int split_k) {
  return split_k > 1 ? (size_t)split_k * (size_t)M * (size_t)N * sizeof(float) : 0;
}

// Launch one instance with run-time knobs.  Pointers in pr.p must be set.
static bolt_status fprop_launch(const FpropInstance& in, FpropProblem pr, int swizzle, int split_k, void* ws,
                                size_t ws_bytes, hipStream_t stream) {
  FpropParams& p = pr.p;
  p.bias_on = p.bias ? 1 : 0;
  if (!p.bias) p.bias = zero_bias();
  if (!p.bias) return BOLT_ERR_LAUNCH;
  p.tiles_m = ceil_div(p.M, in.bm);
  p.tiles_n = ceil_div(p.N, in.bn);
  p.swizzle = swizzle < 0 ? 0 : swizzle;
  if (split_k > 1 && !fprop_can_split_k(in)) return BOLT_ERR_UNSUPPORTED;
  const int nk = ceil_div(p.K, in.bk);
  split_k = std::max(1, std::min(std::min(split_k, kMaxSplitK), nk));
  p.ktiles_per_split = ceil_div(nk, split_k);
  split_k = ceil_div(nk, p.ktiles_per_split);  // no empty splits
  p.split_k = split_k;
  p.partial = nullptr;
  if (split_k > 1) {
    if (!ws || ws_bytes < splitk_bytes(p.M, p.N, split_k) || !is_aligned16(ws)) return BOLT_ERR_WORKSPACE;
    p.partial = (float*)ws;
  }
  if ((int64_t)p.tiles_m * p.tiles_n >= (1ll << 31)) return BOLT_ERR_UNSUPPORTED;
  if (in.launch(p, stream) != hipSuccess) return BOLT_ERR_LAUNCH;
  if (split_k > 1) {
    const int64_t quads = (int64_t)p.M * (p.N / 4);
    const int blocks = (int)std::min<int64_t>((quads + 255) / 256, kNumCU * 8);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, stream, p.partial,
                       p.bias_on ? p.bias : (const half_t*)nullptr, p.Y, p.M, p.N,
                       p.ldy, split_k, p.alpha, p.beta, p.act, p.res, p.ldr, p.gamma);
    if (hipGetLastError() != hipSuccess) return BOLT_ERR_LAUNCH;
  }
  return BOLT_OK;
}

static bolt_status make_gemm_problem(const bolt_gemm_desc* d, FpropProblem* pr) {
  bolt_status s = check_gemm_desc(d);
  if (s != BOLT_OK) return s;
  std::memset(pr, 0, sizeof(*pr));
  pr->xmode = 0;
  pr->wmode = d->b_layout == BOLT_LAYOUT_KN ? 1 : 0;
  FpropParams& p = pr->p;
  p.M = d->M; p.N = d->N; p.K = d->K;
  p.ldx = d->lda; p.ldw = d->ldb; p.ldy = d->ldd;
  p.alpha = d->alpha; p.beta = d->beta; p.act = d->act;
  return BOLT_OK;
}

static bolt_status make_conv_problem(const bolt_conv_desc* d, FpropProblem* pr) {
  ConvDims cd;
  bolt_status s = check_conv_desc(d, &cd);
  if (s != BOLT_OK) return s;
  std::memset(pr, 0, sizeof(*pr));
  pr->xmode = 1;
  pr->wmode = 0;
  FpropParams& p = pr->p;
  p.M = cd.M; p.N = d->K; p.K = cd.Kg;
  p.ldx = 0; p.ldw = cd.Kg; p.ldy = d->K;
  p.alpha = d->alpha; p.beta = d->beta; p.act = d->act;
  p.cg = make_geom(d, cd);
  // A 1x1 filter with unit stride and no padding is a plain GEMM over the [N*H*W][C] pixel matrix:
  // the GEMM instances (cheaper addressing than the implicit-GEMM gather) serve it.
  if (d->R == 1 && d->S == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 && d->pad_w == 0) {
    pr->xmode = 0;
    p.ldx = d->C;
  }
  if (d->C & 7) pr->xmode = pr->wmode = 2;  // alignment 2 (Section 3.2.3): the unpadded kernels
  // odd channel counts and NCHW inputs: only the first-layer instances (which also take C = 2 and 4 from NHWC)
  if ((d->C & 1) || d->x_layout == BOLT_TENSOR_NCHW) pr->xmode = 4;
  p.x_nchw = d->x_layout == BOLT_TENSOR_NCHW ? 1 : 0;
  p.y_nchw = d->y_layout == BOLT_TENSOR_NCHW ? 1 : 0;
  return BOLT_OK;
}

static bolt_status resolve_fprop(const std::vector<FpropInstance>& tab, const FpropProblem& pr,
                                 const bolt_config* cfg, int* id, int* swizzle, int* split_k) {
  *swizzle = cfg ? cfg->swizzle : 0;
  *split_k = cfg && cfg->split_k > 1 ? cfg->split_k : 1;
  if (*split_k > kMaxSplitK) return BOLT_ERR_INVALID_ARG;
  if (cfg && cfg->kernel_id >= 0) {
    if (cfg->kernel_id >= (int)tab.size()) return BOLT_ERR_INVALID_ARG;
    if (!fprop_supports(tab[cfg->kernel_id], pr)) return BOLT_ERR_UNSUPPORTED;
    if (*split_k > 1 && !fprop_can_split_k(tab[cfg->kernel_id])) return BOLT_ERR_UNSUPPORTED;
    *id = cfg->kernel_id;
    return BOLT_OK;
  }
  if (cfg && cfg->kernel_id < -1) return BOLT_ERR_INVALID_ARG;
  *id = fprop_heuristic(tab, pr, *split_k > 1);
  if (*id < 0) return BOLT_ERR_UNSUPPORTED;
  // No config at all: the XCD-aware tile order with bands of 4 where the tile grid has more than one column (measured
  // over 27 problems under the rule's own picks: 6 % less time in total; the halo kernels, whose neighbouring row
  // tiles share their halo through one L2, are 2-9 % better off in plain order).
  if (!cfg && !tab[*id].dyn_supports && ceil_div(pr.p.N, tab[*id].bn) > 1) *swizzle = 4;
  return BOLT_OK;
}

// ------------------------------------------------------------------------------------------
// back-to-back problems
// ------------------------------------------------------------------------------------------
struct B2bProblem {
  B2bParams p;
  int xmode, wmode;
  bool residual;  // the call carries a residual matrix for the last op: kernels without that epilogue are excluded
};

// Can this instance run the problem at all (threadblock residence within its compiled widths, LDS)?
static bool b2b_can_run(const B2bInstance& in, const B2bProblem& pr) {
  if (in.xmode != pr.xmode || in.wmode != pr.wmode) return false;
  if (pr.residual && !in.residual) return false;
  if (pr.p.N0 > in.n0t || pr.p.N1 > in.n1t) return false;
  // row-major weights are fetched through one buffer descriptor per matrix with 32-bit byte offsets
  if (in.wmode == 1 && ((int64_t)pr.p.K0 * pr.p.ldw0 * 2 >= (1ll << 31) || (int64_t)pr.p.N0 * pr.p.ldw1 * 2 >= (1ll << 31))) return false;
  if (in.dyn_supports) return in.dyn_supports(pr.p) && in.dyn_lds_bytes(pr.p) <= kLdsPerCU;
  if (in.lds_bytes(pr.p.K0) > kLdsPerCU) return false;
  return true;
}
// Threadblock residence with the tightest compiled bound: an instance that would carry more than 2x padding in a
// width is left out ...
static bool b2b_is_tight(const B2bInstance& in, const B2bProblem& pr) {
  return !((in.n0t > 32 && in.n0t / 2 >= pr.p.N0) || (in.n1t > 32 && in.n1t / 2 >= pr.p.N1));
}
// ... unless that leaves the problem without a kernel (e.g. N0 = 128 with N1 = 16: no compiled pair of widths is tight
// in both).
static bool b2b_supports(const std::vector<B2bInstance>& tab, int id, const B2bProblem& pr) {
  if (!b2b_can_run(tab[id], pr)) return false;
  if (b2b_is_tight(tab[id], pr)) return true;
  for (const B2bInstance& other : tab)
    if (b2b_can_run(other, pr) && b2b_is_tight(other, pr)) return false;
  return true;
}

static void b2b_fill_config(const B2bInstance& in, int id, bolt_config* c) {
  c->kernel_id = id;
  c->tile_m = in.bm; c->tile_n = in.n1t; c->tile_k = in.bk;
  c->waves_m = in.waves_m; c->waves_n = in.waves_n;
  c->mfma_shape = 32; c->stages = in.stages; c->swizzle = 0; c->split_k = 1; c->b2b_mode = in.mode;
}

static int b2b_heuristic(const std::vector<B2bInstance>& tab, const B2bProblem& pr) {
  int best = -1;
  double best_cost = 0;
  for (int i = 0; i < (int)tab.size(); ++i) {
    if (!b2b_supports(tab, i, pr)) continue;
    const B2bInstance& in = tab[i];
    const double tiles = ceil_div(pr.p.M, in.bm);
    const int lds = in.dyn_lds_bytes ? in.dyn_lds_bytes(pr.p) : in.lds_bytes(pr.p.K0);
    const int per_cu = std::max(1, std::min(kLdsPerCU / std::max(lds, 1), 2048 / in.nthreads));  // co-resident workgroups
    const double rounds = std::ceil(tiles / kNumCU);  // tiles a compute unit works through, co-resident or in turn
    const double kpad = (double)ceil_div(pr.p.K0, in.bk) * in.bk;  // a short reduction pays for the whole last k-tile
    double cost = rounds * in.bm * (in.mode == 0 ? 1.0 : 1.1) * (kpad * in.n0t + (double)in.n0t * in.n1t) *
                  (in.prior > 0.f ? in.prior : 1.0);
    // 64-row wave tiles read half the weight fragments per MFMA of 32-row ones, and a second co-resident workgroup
    // covers the load and store phases of the first (measured on the pairs of Table 2: 256-row tiles of 4 waves win
    // wherever two of them fit a compute unit)
    cost *= 1.0 + 32.0 / ((double)in.bm / in.waves_m);
    cost *= 1.0 + 0.5 / std::min<double>(per_cu, std::max(1.0, std::ceil(tiles / kNumCU)));
    if (tune_log_enabled()) std::fprintf(stderr, "[bolt_pick] candidate %d %s cost %.4g\n", i, in.name, cost);
    if (best < 0 || cost < best_cost) { best = i; best_cost = cost; }
  }
  if (tune_log_enabled() && best >= 0) std::fprintf(stderr, "[bolt_pick] -> %d %s\n", best, tab[best].name);
  return best;
}

static bolt_status b2b_launch(const B2bInstance& in, B2bProblem pr, hipStream_t stream) {
  B2bParams& p = pr.p;
  p.b0_on = p.b0 ? 1 : 0;
  p.b1_on = p.b1 ? 1 : 0;
  if (!p.b0) p.b0 = zero_bias();
  if (!p.b1) p.b1 = zero_bias();
  if (!p.b0 || !p.b1) return BOLT_ERR_LAUNCH;
  p.tiles_m = ceil_div(p.M, in.bm);
  const int lds = in.dyn_lds_bytes ? in.dyn_lds_bytes(p) : in.lds_bytes(p.K0);
  if (lds > kLdsPerCU) return BOLT_ERR_UNSUPPORTED;
  const int per_cu = std::max(1, std::min(kLdsPerCU / lds, 2048 / in.nthreads));
  const int grid = std::min(p.tiles_m, kNumCU * per_cu);
  if (in.launch(p, grid, lds, stream) != hipSuccess) return BOLT_ERR_LAUNCH;
  return BOLT_OK;
}

static bolt_status make_b2b_gemm_problem(const bolt_gemm_desc* g0, const bolt_gemm_desc* g1, B2bProblem* pr) {
  bolt_status s = check_b2b_gemm(g0, g1);
  if (s != BOLT_OK) return s;
  std::memset(pr, 0, sizeof(*pr));
  pr->xmode = 0;
  pr->wmode = g0->b_layout == BOLT_LAYOUT_KN ? 1 : 0;
  B2bParams& p = pr->p;
  p.M = g0->M; p.N0 = g0->N; p.K0 = g0->K; p.N1 = g1->N;
  p.ldx = g0->lda; p.ldw0 = g0->ldb; p.ldw1 = g1->ldb; p.ldy = g1->ldd;
  p.alpha0 = g0->alpha; p.beta0 = g0->beta; p.act0 = g0->act;
  p.alpha1 = g1->alpha; p.beta1 = g1->beta; p.act1 = g1->act;
  return BOLT_OK;
}

static bolt_status make_b2b_conv_problem(const bolt_conv_desc* c0, const bolt_conv_desc* c1, B2bProblem* pr) {
  ConvDims cd;
  bolt_status s = check_b2b_conv(c0, c1, &cd);
  if (s != BOLT_OK) return s;
  std::memset(pr, 0, sizeof(*pr));
  pr->xmode = 1;
  pr->wmode = 0;
  B2bParams& p = pr->p;
  p.M = cd.M; p.N0 = c0->K; p.K0 = cd.Kg; p.N1 = c1->K;
  p.ldx = 0; p.ldw0 = cd.Kg; p.ldw1 = c1->C; p.ldy = c1->K;
  p.alpha0 = c0->alpha; p.beta0 = c0->beta; p.act0 = c0->act;
  p.alpha1 = c1->alpha; p.beta1 = c1->beta; p.act1 = c1->act;
  p.cg = make_geom(c0, cd);
  return BOLT_OK;
}

static bolt_status resolve_b2b(const std::vector<B2bInstance>& tab, const B2bProblem& pr, const bolt_config* cfg,
                               int* id) {
  if (cfg && cfg->kernel_id >= 0) {
    if (cfg->kernel_id >= (int)tab.size()) return BOLT_ERR_INVALID_ARG;
    if (!b2b_supports(tab, cfg->kernel_id, pr)) return BOLT_ERR_UNSUPPORTED;
    *id = cfg->kernel_id;
    return BOLT_OK;
  }
  if (cfg && cfg->kernel_id < -1) return BOLT_ERR_INVALID_ARG;
  *id = b2b_heuristic(tab, pr);
  return *id < 0 ? BOLT_ERR_UNSUPPORTED : BOLT_OK;
}

// ------------------------------------------------------------------------------------------
// three-op chains
// ------------------------------------------------------------------------------------------
static bool chain_can_run(const ChainInstance& in, const B2bProblem& pr) {
  if (in.xmode != pr.xmode || in.wmode != pr.wmode) return false;
  const B2bParams& p = pr.p;
  if (p.N0 > in.n0t || p.N1 > in.n1t || p.N2 > in.n2t) return false;
  // row-major weights are fetched through one buffer descriptor per matrix with 32-bit byte offsets
  const int64_t lim = 1ll << 31;
  if (in.wmode == 1 && ((int64_t)p.K0 * p.ldw0 * 2 >= lim || (int64_t)p.N0 * p.ldw1 * 2 >= lim || (int64_t)p.N1 * p.ldw2 * 2 >= lim)) return false;
  if (in.dyn_supports) return in.dyn_supports(p) && in.dyn_lds_bytes(p) <= kLdsPerCU;
  return in.lds_bytes <= kLdsPerCU;
}
// threadblock residence with the tightest compiled bounds: no more than 2x padding per op ...
static bool chain_is_tight(const ChainInstance& in, const B2bProblem& pr) {
  const B2bParams& p = pr.p;
  return !((in.n0t > 64 && in.n0t / 2 >= p.N0) || (in.n1t > 64 && in.n1t / 2 >= p.N1) || (in.n2t > 64 && in.n2t / 2 >= p.N2));
}
// ... unless no instance that can run the problem is tight in all three widths
static bool chain_supports(const std::vector<ChainInstance>& tab, int id, const B2bProblem& pr) {
  if (!chain_can_run(tab[id], pr)) return false;
  if (chain_is_tight(tab[id], pr)) return true;
  for (const ChainInstance& other : tab)
    if (chain_can_run(other, pr) && chain_is_tight(other, pr)) return false;
  return true;
}

static void chain_fill_config(const ChainInstance& in, int id, bolt_config* c) {
  c->kernel_id = id;
  c->tile_m = in.bm; c->tile_n = in.n2t; c->tile_k = in.bk;
  c->waves_m = in.waves; c->waves_n = 1;
  c->mfma_shape = 32; c->stages = in.stages; c->swizzle = 0; c->split_k = 1; c->b2b_mode = BOLT_B2B_RF;
}

static bolt_status chain_launch(const ChainInstance& in, B2bProblem pr, hipStream_t stream) {
  B2bParams& p = pr.p;
  p.b0_on = p.b0 ? 1 : 0;
  p.b1_on = p.b1 ? 1 : 0;
  p.b2_on = p.b2 ? 1 : 0;
  if (!p.b0) p.b0 = zero_bias();
  if (!p.b1) p.b1 = zero_bias();
  if (!p.b2) p.b2 = zero_bias();
  if (!p.b0 || !p.b1 || !p.b2) return BOLT_ERR_LAUNCH;
  p.tiles_m = ceil_div(p.M, in.bm);
  return in.launch(p, stream) == hipSuccess ? BOLT_OK : BOLT_ERR_LAUNCH;
}

// Validates a chain of three descriptors and builds its problem (pointers left null).
static bolt_status make_chain_problem(bolt_op op, int32_t n_ops, const void* const* descs, B2bProblem* pr) {
  if (op != BOLT_OP_GEMM_CHAIN3 && op != BOLT_OP_CONV_CHAIN3) return BOLT_ERR_INVALID_ARG;
  if (!descs || n_ops <= 0) return BOLT_ERR_INVALID_ARG;
  if (n_ops != 3) return BOLT_ERR_UNSUPPORTED;
  if (!descs[0] || !descs[1] || !descs[2]) return BOLT_ERR_INVALID_ARG;
  bolt_status s;
  if (op == BOLT_OP_GEMM_CHAIN3) {
    const bolt_gemm_desc* g0 = (const bolt_gemm_desc*)descs[0];
    const bolt_gemm_desc* g1 = (const bolt_gemm_desc*)descs[1];
    const bolt_gemm_desc* g2 = (const bolt_gemm_desc*)descs[2];
    if ((s = make_b2b_gemm_problem(g0, g1, pr)) != BOLT_OK) return s;
    if ((s = check_b2b_gemm(g1, g2)) != BOLT_OK) return s;
    B2bParams& p = pr->p;
    p.N2 = g2->N; p.ldw2 = g2->ldb; p.ldy = g2->ldd;
    p.alpha2 = g2->alpha; p.beta2 = g2->beta; p.act2 = g2->act;
  } else {
    const bolt_conv_desc* c0 = (const bolt_conv_desc*)descs[0];
    const bolt_conv_desc* c1 = (const bolt_conv_desc*)descs[1];
    const bolt_conv_desc* c2 = (const bolt_conv_desc*)descs[2];
    if ((s = make_b2b_conv_problem(c0, c1, pr)) != BOLT_OK) return s;
    if ((s = check_b2b_conv(c1, c2, nullptr)) != BOLT_OK) return s;
    B2bParams& p = pr->p;
    p.N2 = c2->K; p.ldw2 = c2->C; p.ldy = c2->K;
    p.alpha2 = c2->alpha; p.beta2 = c2->beta; p.act2 = c2->act;
  }
  return BOLT_OK;
}

static int chain_heuristic(const std::vector<ChainInstance>& tab, const B2bProblem& pr) {
  int best = -1;
  double best_cost = 0;
  for (int i = 0; i < (int)tab.size(); ++i) {
    if (!chain_supports(tab, i, pr)) continue;
    // the tightest widths; the halo main loop where it applies; 64-row wave tiles (as for the fused pairs)
    double cost = (double)tab[i].n0t * tab[i].n1t + (double)tab[i].n1t * tab[i].n2t + 1e-3 * tab[i].lds_bytes;
    cost *= (tab[i].dyn_supports ? 0.75 : 1.0) * (1.0 + 32.0 / ((double)tab[i].bm / tab[i].waves));
    if (tune_log_enabled()) std::fprintf(stderr, "[bolt_pick] candidate %d %s cost %.4g\n", i, tab[i].name, cost);
    if (best < 0 || cost < best_cost) { best = i; best_cost = cost; }
  }
  if (tune_log_enabled() && best >= 0) std::fprintf(stderr, "[bolt_pick] -> %d %s\n", best, tab[best].name);
  return best;
}

static bolt_status resolve_chain(const std::vector<ChainInstance>& tab, const B2bProblem& pr, const bolt_config* cfg,
                                 int* id) {
  if (cfg && cfg->kernel_id >= 0) {
    if (cfg->kernel_id >= (int)tab.size()) return BOLT_ERR_INVALID_ARG;
    if (!chain_supports(tab, cfg->kernel_id, pr)) return BOLT_ERR_UNSUPPORTED;
    *id = cfg->kernel_id;
    return BOLT_OK;
  }
  if (cfg && cfg->kernel_id < -1) return BOLT_ERR_INVALID_ARG;
  *id = chain_heuristic(tab, pr);
  return *id < 0 ? BOLT_ERR_UNSUPPORTED : BOLT_OK;
}

// ------------------------------------------------------------------------------------------
// profiler
// ------------------------------------------------------------------------------------------
struct TuneKey {
  int op;
  std::string bytes;
  bool operator<(const TuneKey& o) const { return op != o.op ? op < o.op : bytes < o.bytes; }
};
struct TuneVal {
  bolt_config cfg;
  float ms;
  int tried;
};
static std::map<TuneKey, TuneVal>& tune_cache() {
  static std::map<TuneKey, TuneVal> c;
  return c;
}
static std::mutex& tune_mutex() {
  static std::mutex m;
  return m;
}

struct Candidate {
  int id, swizzle, split_k;
  float ms;
};

// Mean milliseconds per launch of `fn` over `reps` back-to-back launches (after `warm` untimed).
template <typename F>
static bolt_status time_launches(F&& fn, int warm, int reps, hipStream_t stream, hipEvent_t e0, hipEvent_t e1,
                                 float* ms) {
  for (int i = 0; i < warm; ++i) {
    bolt_status s = fn();
    if (s != BOLT_OK) return s;
  }
  if (hipEventRecord(e0, stream) != hipSuccess) return BOLT_ERR_LAUNCH;
  for (int i = 0; i < reps; ++i) {
    bolt_status s = fn();
    if (s != BOLT_OK) return s;
  }
  if (hipEventRecord(e1, stream) != hipSuccess) return BOLT_ERR_LAUNCH;
  if (hipEventSynchronize(e1) != hipSuccess) return BOLT_ERR_LAUNCH;
  float t = 0.f;
  if (hipEventElapsedTime(&t, e0, e1) != hipSuccess) return BOLT_ERR_LAUNCH;
  *ms = t / reps;
  return BOLT_OK;
}


template <typename RunF>
static bolt_status tune_candidates(std::vector<Candidate>& cands, RunF&& run, hipStream_t stream, Candidate* best,
                                   int* tried) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return BOLT_ERR_LAUNCH;
  bolt_status status = BOLT_OK;
  int n_ok = 0;
  // pass 1: a short timing of every candidate
  for (auto& c : cands) {
    bolt_status s = time_launches([&] { return run(c); }, 2, 8, stream, e0, e1, &c.ms);
    if (s == BOLT_ERR_LAUNCH) { status = s; break; }
    if (s != BOLT_OK) { c.ms = -1.f; continue; }
    if (tune_log_enabled())
      std::fprintf(stderr, "[bolt_tune] pass1 id %d swizzle %d split_k %d: %.4f ms\n", c.id, c.swizzle, c.split_k, c.ms);
    ++n_ok;
  }
  if (status == BOLT_OK && n_ok == 0) status = BOLT_ERR_UNSUPPORTED;
  if (status == BOLT_OK) {
    std::vector<Candidate*> order;
    for (auto& c : cands) if (c.ms >= 0.f) order.push_back(&c);
    // Near-ties go to the XCD-aware tile order: the same time with fewer operand bytes crossing the fabric.
    auto score = [](const Candidate* c) { return c->ms * (c->swizzle > 0 ? 0.985f : 1.f); };
    std::sort(order.begin(), order.end(), [&](Candidate* a, Candidate* b) { return score(a) < score(b); });
    // pass 2: the few fastest again, longer
    const int finalists = std::min<int>(6, (int)order.size());
    Candidate* win = nullptr;
    for (int i = 0; i < finalists && status == BOLT_OK; ++i) {
      Candidate* c = order[i];
      bolt_status s = time_launches([&] { return run(*c); }, 3, 60, stream, e0, e1, &c->ms);
      if (s != BOLT_OK) { status = s; break; }
      if (!win || score(c) < score(win)) win = c;
    }
    if (status == BOLT_OK) { *best = *win; *tried = n_ok; }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return status;
}

static std::vector<Candidate> fprop_candidates(const std::vector<FpropInstance>& tab, const FpropProblem& pr,
                                               size_t ws_bytes, bool have_ws) {
  std::vector<Candidate> out;
  for (int i = 0; i < (int)tab.size(); ++i) {
    const FpropInstance& in = tab[i];
    if (!fprop_supports(in, pr)) continue;
    const int tiles_m = ceil_div(pr.p.M, in.bm), tiles_n = ceil_div(pr.p.N, in.bn);
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int nk = ceil_div(pr.p.K, in.bk);
    if (in.dyn_supports) {  // no split-K / swizzle variants for these
      out.push_back({i, 0, 1, 0.f});
      continue;
    }
    const int swz[3] = {0, 1, 4};
    const int nswz = (tiles_n > 1 && tiles_m > 1 && tiles >= 64) ? 3 : 1;
    for (int s = 0; s < nswz; ++s) {
      out.push_back({i, swz[s], 1, 0.f});
    }
    // split-K only when the grid cannot fill the chip and K is deep enough to share
    for (int sk = 2; sk <= kMaxSplitK && fprop_can_split_k(in); sk *= 2) {
      if (tiles * (sk / 2) >= kNumCU || nk < 2 * sk) break;
      if (!have_ws || ws_bytes < splitk_bytes(pr.p.M, pr.p.N, sk)) break;
      out.push_back({i, 0, sk, 0.f});
    }
  }
  return out;
}

}  // namespace bolt

// ==========================================================================================
// C ABI
// ==========================================================================================
using namespace bolt;

extern "C" {

const char* bolt_status_string(bolt_status s) {
  switch (s) {
    case BOLT_OK: return "ok";
    case BOLT_ERR_INVALID_ARG: return "invalid argument";
    case BOLT_ERR_UNSUPPORTED: return "unsupported problem or configuration";
    case BOLT_ERR_ALIGNMENT: return "size, leading dimension or pointer not aligned to 8 halves / 16 bytes";
    case BOLT_ERR_WORKSPACE: return "workspace missing or too small";
    case BOLT_ERR_LAUNCH: return "HIP runtime error";
    case BOLT_ERR_ILLEGAL_FUSION: return "ops cannot be fused back to back";
    default: return "unknown status";
  }
}

int32_t bolt_num_instances(bolt_op op) {
  switch (op) {
    case BOLT_OP_GEMM: return (int32_t)tables().gemm.size();
    case BOLT_OP_CONV2D: return (int32_t)tables().conv.size();
    case BOLT_OP_B2B_GEMM: case BOLT_OP_B2B_GEMM_RES: return (int32_t)tables().b2b_gemm.size();
    case BOLT_OP_B2B_CONV: case BOLT_OP_B2B_CONV_RES: return (int32_t)tables().b2b_conv.size();
    case BOLT_OP_GEMM_CHAIN3: return (int32_t)tables().gemm_chain.size();
    case BOLT_OP_CONV_CHAIN3: return (int32_t)tables().conv_chain.size();
    default: return 0;
  }
}

bolt_status bolt_instance_config(bolt_op op, int32_t id, bolt_config* out) {
  if (!out || id < 0 || id >= bolt_num_instances(op)) return BOLT_ERR_INVALID_ARG;
  std::memset(out, 0, sizeof(*out));
  out->split_k = 1;
  switch (op) {
    case BOLT_OP_GEMM: fprop_fill_config(tables().gemm[id], id, out); break;
    case BOLT_OP_CONV2D: fprop_fill_config(tables().conv[id], id, out); break;
    case BOLT_OP_B2B_GEMM: case BOLT_OP_B2B_GEMM_RES: b2b_fill_config(tables().b2b_gemm[id], id, out); break;
    case BOLT_OP_B2B_CONV: case BOLT_OP_B2B_CONV_RES: b2b_fill_config(tables().b2b_conv[id], id, out); break;
    case BOLT_OP_GEMM_CHAIN3: chain_fill_config(tables().gemm_chain[id], id, out); break;
    case BOLT_OP_CONV_CHAIN3: chain_fill_config(tables().conv_chain[id], id, out); break;
    default: return BOLT_ERR_INVALID_ARG;
  }
  return BOLT_OK;
}

int32_t bolt_instance_supports(bolt_op op, int32_t id, const void* desc0, const void* desc1) {
  if (id < 0 || id >= bolt_num_instances(op)) return 0;
  FpropProblem fp;
  B2bProblem bp;
  switch (op) {
    case BOLT_OP_GEMM:
      return make_gemm_problem((const bolt_gemm_desc*)desc0, &fp) == BOLT_OK && fprop_supports(tables().gemm[id], fp);
    case BOLT_OP_CONV2D:
      return make_conv_problem((const bolt_conv_desc*)desc0, &fp) == BOLT_OK && fprop_supports(tables().conv[id], fp);
    case BOLT_OP_B2B_GEMM: case BOLT_OP_B2B_GEMM_RES:
      if (make_b2b_gemm_problem((const bolt_gemm_desc*)desc0, (const bolt_gemm_desc*)desc1, &bp) != BOLT_OK) return 0;
      bp.residual = op == BOLT_OP_B2B_GEMM_RES;
      return b2b_supports(tables().b2b_gemm, id, bp);
    case BOLT_OP_B2B_CONV: case BOLT_OP_B2B_CONV_RES:
      if (make_b2b_conv_problem((const bolt_conv_desc*)desc0, (const bolt_conv_desc*)desc1, &bp) != BOLT_OK) return 0;
      bp.residual = op == BOLT_OP_B2B_CONV_RES;
      return b2b_supports(tables().b2b_conv, id, bp);
    default: return 0;
  }
}

bolt_status bolt_check(bolt_op op, const void* desc0, const void* desc1, const bolt_config* config) {
  FpropProblem fp;
  B2bProblem bp;
  int id, swz, sk;
  bolt_status s;
  switch (op) {
    case BOLT_OP_GEMM:
      s = make_gemm_problem((const bolt_gemm_desc*)desc0, &fp);
      return s != BOLT_OK ? s : resolve_fprop(tables().gemm, fp, config, &id, &swz, &sk);
    case BOLT_OP_CONV2D:
      s = make_conv_problem((const bolt_conv_desc*)desc0, &fp);
      return s != BOLT_OK ? s : resolve_fprop(tables().conv, fp, config, &id, &swz, &sk);
    case BOLT_OP_B2B_GEMM: case BOLT_OP_B2B_GEMM_RES:
      s = make_b2b_gemm_problem((const bolt_gemm_desc*)desc0, (const bolt_gemm_desc*)desc1, &bp);
      if (s != BOLT_OK) return s;
      bp.residual = op == BOLT_OP_B2B_GEMM_RES;
      return resolve_b2b(tables().b2b_gemm, bp, config, &id);
    case BOLT_OP_B2B_CONV: case BOLT_OP_B2B_CONV_RES:
      s = make_b2b_conv_problem((const bolt_conv_desc*)desc0, (const bolt_conv_desc*)desc1, &bp);
      if (s != BOLT_OK) return s;
      bp.residual = op == BOLT_OP_B2B_CONV_RES;
      return resolve_b2b(tables().b2b_conv, bp, config, &id);
    default: return BOLT_ERR_INVALID_ARG;
  }
}

size_t bolt_workspace_bytes(bolt_op op, const void* desc0, const void* desc1, const bolt_config* config) {
  (void)desc1;
  FpropProblem fp;
  bolt_status s;
  if (op == BOLT_OP_GEMM) s = make_gemm_problem((const bolt_gemm_desc*)desc0, &fp);
  else if (op == BOLT_OP_CONV2D) s = make_conv_problem((const bolt_conv_desc*)desc0, &fp);
  else return 0;
  if (s != BOLT_OK) return 0;
  if (config) return splitk_bytes(fp.p.M, fp.p.N, std::min<int>(config->split_k, kMaxSplitK));
  // upper bound for tuning: split-K is only tried while the output is small
  size_t need = 0;
  for (int sk = 2; sk <= kMaxSplitK; sk *= 2) {
    const int64_t min_tiles = (int64_t)ceil_div(fp.p.M, 256) * ceil_div(fp.p.N, 256);
    if (min_tiles * (sk / 2) >= kNumCU) break;
    need = splitk_bytes(fp.p.M, fp.p.N, sk);
  }
  return need;
}

bolt_status bolt_gemm_epilogue(const bolt_gemm_desc* desc, const void* A, const void* B, const void* bias, void* D,
                               const bolt_config* config, void* workspace, size_t workspace_bytes, void* stream) {
  FpropProblem pr;
  bolt_status s = make_gemm_problem(desc, &pr);
  if (s != BOLT_OK) return s;
  if (!A || !B || !D) return BOLT_ERR_INVALID_ARG;
  if (!is_aligned16(A) || !is_aligned16(B) || !is_aligned16(D) || (bias && !is_aligned16(bias))) return BOLT_ERR_ALIGNMENT;
  int id, swz, sk;
  s = resolve_fprop(tables().gemm, pr, config, &id, &swz, &sk);
  if (s != BOLT_OK) return s;
  pr.p.X = (const half_t*)A; pr.p.W = (const half_t*)B; pr.p.bias = (const half_t*)bias; pr.p.Y = (half_t*)D;
  return fprop_launch(tables().gemm[id], pr, swz, sk, workspace, workspace_bytes, (hipStream_t)stream);
}

bolt_status bolt_gemm_epilogue_noalloc(const bolt_gemm_desc* desc, const void* A, const void* B, const void* bias,
                                       void* D, const bolt_config* config, void* stream) {
  FpropProblem pr;
  bolt_status s = make_gemm_problem(desc, &pr);
  if (s != BOLT_OK) return s;
  if (!A || !B || !D) return BOLT_ERR_INVALID_ARG;
  if (!is_aligned16(A) || !is_aligned16(B) || !is_aligned16(D) || (bias && !is_aligned16(bias))) return BOLT_ERR_ALIGNMENT;
  int id, swz, sk;
  s = resolve_fprop(tables().gemm, pr, config, &id, &swz, &sk);
  if (s != BOLT_OK) return s;
  // the partial sums of this call must fit the fixed array (the same clamp of split_k as the launch applies)
  const int nk = ceil_div(pr.p.K, tables().gemm[id].bk);
  const int sk_eff = std::max(1, std::min(std::min(sk, kMaxSplitK), nk));
  if (splitk_bytes(pr.p.M, pr.p.N, sk_eff) > (size_t)BOLT_NOALLOC_SCRATCH_BYTES) return BOLT_ERR_WORKSPACE;
  void* ws = scratch_of_current_device();
  if (!ws) return BOLT_ERR_LAUNCH;
  pr.p.X = (const half_t*)A; pr.p.W = (const half_t*)B; pr.p.bias = (const half_t*)bias; pr.p.Y = (half_t*)D;
  return fprop_launch(tables().gemm[id], pr, swz, sk, ws, (size_t)BOLT_NOALLOC_SCRATCH_BYTES, (hipStream_t)stream);
}

bolt_status bolt_conv2d_fprop_nhwc(const bolt_conv_desc* desc, const void* x, const void* w, const void* bias,
                                   void* y, const bolt_config* config, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  FpropProblem pr;
  bolt_status s = make_conv_problem(desc, &pr);
  if (s != BOLT_OK) return s;
  if (!x || !w || !y) return BOLT_ERR_INVALID_ARG;
  if (!is_aligned16(x) || !is_aligned16(w) || !is_aligned16(y) || (bias && !is_aligned16(bias))) return BOLT_ERR_ALIGNMENT;
  int id, swz, sk;
  s = resolve_fprop(tables().conv, pr, config, &id, &swz, &sk);
  if (s != BOLT_OK) return s;
  pr.p.X = (const half_t*)x; pr.p.W = (const half_t*)w; pr.p.bias = (const half_t*)bias; pr.p.Y = (half_t*)y;
  return fprop_launch(tables().conv[id], pr, swz, sk, workspace, workspace_bytes, (hipStream_t)stream);
}

bolt_status bolt_gemm_epilogue_residual(const bolt_gemm_desc* desc, const void* A, const void* B, const void* bias,
                                        const void* C, int32_t ldc, float gamma, void* D, const bolt_config* config,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  FpropProblem pr;
  bolt_status s = make_gemm_problem(desc, &pr);
  if (s != BOLT_OK) return s;
  if (!A || !B || !C || !D || ldc < desc->N) return BOLT_ERR_INVALID_ARG;
  if ((ldc & 7) || !is_aligned16(A) || !is_aligned16(B) || !is_aligned16(C) || !is_aligned16(D) ||
      (bias && !is_aligned16(bias)))
    return BOLT_ERR_ALIGNMENT;
  pr.residual = true;
  int id, swz, sk;
  s = resolve_fprop(tables().gemm, pr, config, &id, &swz, &sk);
  if (s != BOLT_OK) return s;
  pr.p.X = (const half_t*)A; pr.p.W = (const half_t*)B; pr.p.bias = (const half_t*)bias; pr.p.Y = (half_t*)D;
  pr.p.res = (const half_t*)C; pr.p.ldr = ldc; pr.p.gamma = gamma;
  return fprop_launch(tables().gemm[id], pr, swz, sk, workspace, workspace_bytes, (hipStream_t)stream);
}

bolt_status bolt_conv2d_fprop_nhwc_residual(const bolt_conv_desc* desc, const void* x, const void* w, const void* bias,
                                            const void* residual, float gamma, void* y, const bolt_config* config,
                                            void* workspace, size_t workspace_bytes, void* stream) {
  FpropProblem pr;
  bolt_status s = make_conv_problem(desc, &pr);
  if (s != BOLT_OK) return s;
  if (!x || !w || !residual || !y) return BOLT_ERR_INVALID_ARG;
  if (!is_aligned16(x) || !is_aligned16(w) || !is_aligned16(residual) || !is_aligned16(y) ||
      (bias && !is_aligned16(bias)))
    return BOLT_ERR_ALIGNMENT;
  pr.residual = true;
  int id, swz, sk;
  s = resolve_fprop(tables().conv, pr, config, &id, &swz, &sk);
  if (s != BOLT_OK) return s;
  pr.p.X = (const half_t*)x; pr.p.W = (const half_t*)w; pr.p.bias = (const half_t*)bias; pr.p.Y = (half_t*)y;
  pr.p.res = (const half_t*)residual; pr.p.ldr = desc->K; pr.p.gamma = gamma;
  return fprop_launch(tables().conv[id], pr, swz, sk, workspace, workspace_bytes, (hipStream_t)stream);
}

bolt_status bolt_b2b_gemm(const bolt_gemm_desc* g0, const bolt_gemm_desc* g1, const void* A0, const void* W0,
                          const void* b0, const void* W1, const void* b1, void* D1, const bolt_config* config,
                          void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  B2bProblem pr;
  bolt_status s = make_b2b_gemm_problem(g0, g1, &pr);
  if (s != BOLT_OK) return s;
  if (!A0 || !W0 || !W1 || !D1) return BOLT_ERR_INVALID_ARG;
  if (!is_aligned16(A0) || !is_aligned16(W0) || !is_aligned16(W1) || !is_aligned16(D1) ||
      (b0 && !is_aligned16(b0)) || (b1 && !is_aligned16(b1)))
    return BOLT_ERR_ALIGNMENT;
  int id;
  s = resolve_b2b(tables().b2b_gemm, pr, config, &id);
  if (s != BOLT_OK) return s;
  B2bParams& p = pr.p;
  p.X = (const half_t*)A0; p.W0 = (const half_t*)W0; p.b0 = (const half_t*)b0;
  p.W1 = (const half_t*)W1; p.b1 = (const half_t*)b1; p.Y = (half_t*)D1;
  return b2b_launch(tables().b2b_gemm[id], pr, (hipStream_t)stream);
}

bolt_status bolt_b2b_conv(const bolt_conv_desc* c0, const bolt_conv_desc* c1, const void* x, const void* w0,
                          const void* b0, const void* w1, const void* b1, void* y, const bolt_config* config,
                          void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  B2bProblem pr;
  bolt_status s = make_b2b_conv_problem(c0, c1, &pr);
  if (s != BOLT_OK) return s;
  if (!x || !w0 || !w1 || !y) return BOLT_ERR_INVALID_ARG;
  if (!is_aligned16(x) || !is_aligned16(w0) || !is_aligned16(w1) || !is_aligned16(y) ||
      (b0 && !is_aligned16(b0)) || (b1 && !is_aligned16(b1)))
    return BOLT_ERR_ALIGNMENT;
  int id;
  s = resolve_b2b(tables().b2b_conv, pr, config, &id);
  if (s != BOLT_OK) return s;
  B2bParams& p = pr.p;
  p.X = (const half_t*)x; p.W0 = (const half_t*)w0; p.b0 = (const half_t*)b0;
  p.W1 = (const half_t*)w1; p.b1 = (const half_t*)b1; p.Y = (half_t*)y;
  return b2b_launch(tables().b2b_conv[id], pr, (hipStream_t)stream);
}

bolt_status bolt_b2b_gemm_residual(const bolt_gemm_desc* g0, const bolt_gemm_desc* g1, const void* A0, const void* W0,
                                   const void* b0, const void* W1, const void* b1, const void* C, int32_t ldc,
                                   float gamma, void* D1, const bolt_config* config, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  B2bProblem pr;
  bolt_status s = make_b2b_gemm_problem(g0, g1, &pr);
  if (s != BOLT_OK) return s;
  if (!A0 || !W0 || !W1 || !C || !D1 || ldc < g1->N) return BOLT_ERR_INVALID_ARG;
  if ((ldc & 7) || !is_aligned16(A0) || !is_aligned16(W0) || !is_aligned16(W1) || !is_aligned16(C) || !is_aligned16(D1) ||
      (b0 && !is_aligned16(b0)) || (b1 && !is_aligned16(b1)))
    return BOLT_ERR_ALIGNMENT;
  pr.residual = true;
  int id;
  s = resolve_b2b(tables().b2b_gemm, pr, config, &id);
  if (s != BOLT_OK) return s;
  B2bParams& p = pr.p;
  p.X = (const half_t*)A0; p.W0 = (const half_t*)W0; p.b0 = (const half_t*)b0;
  p.W1 = (const half_t*)W1; p.b1 = (const half_t*)b1; p.Y = (half_t*)D1;
  p.res = (const half_t*)C; p.ldr = ldc; p.gamma = gamma;
  return b2b_launch(tables().b2b_gemm[id], pr, (hipStream_t)stream);
}

bolt_status bolt_b2b_conv_residual(const bolt_conv_desc* c0, const bolt_conv_desc* c1, const void* x, const void* w0,
                                   const void* b0, const void* w1, const void* b1, const void* residual, float gamma,
                                   void* y, const bolt_config* config, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  (void)workspace; (void)workspace_bytes;
  B2bProblem pr;
  bolt_status s = make_b2b_conv_problem(c0, c1, &pr);
  if (s != BOLT_OK) return s;
  if (!x || !w0 || !w1 || !residual || !y) return BOLT_ERR_INVALID_ARG;
  if (!is_aligned16(x) || !is_aligned16(w0) || !is_aligned16(w1) || !is_aligned16(residual) || !is_aligned16(y) ||
      (b0 && !is_aligned16(b0)) || (b1 && !is_aligned16(b1)))
    return BOLT_ERR_ALIGNMENT;
  pr.residual = true;
  int id;
  s = resolve_b2b(tables().b2b_conv, pr, config, &id);
  if (s != BOLT_OK) return s;
  B2bParams& p = pr.p;
  p.X = (const half_t*)x; p.W0 = (const half_t*)w0; p.b0 = (const half_t*)b0;
  p.W1 = (const half_t*)w1; p.b1 = (const half_t*)b1; p.Y = (half_t*)y;
  p.res = (const half_t*)residual; p.ldr = c1->K; p.gamma = gamma;
  return b2b_launch(tables().b2b_conv[id], pr, (hipStream_t)stream);
}

bolt_status bolt_tune(bolt_op op, const void* desc0, const void* desc1, const void* const* ptrs, void* workspace,
                      size_t workspace_bytes, void* stream_v, bolt_config* best, float* best_ms, int32_t* n_tried) {
  if (!desc0 || !ptrs || !best) return BOLT_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_v;
  const bool single = op == BOLT_OP_GEMM || op == BOLT_OP_CONV2D;
  const bool with_res = op == BOLT_OP_B2B_GEMM_RES || op == BOLT_OP_B2B_CONV_RES;
  const bool b2b_gemm = op == BOLT_OP_B2B_GEMM || op == BOLT_OP_B2B_GEMM_RES;
  const bool is_b2b = b2b_gemm || op == BOLT_OP_B2B_CONV || op == BOLT_OP_B2B_CONV_RES;
  if (!single && !is_b2b) return BOLT_ERR_INVALID_ARG;
  if (is_b2b && !desc1) return BOLT_ERR_INVALID_ARG;
  const size_t dsz = (op == BOLT_OP_GEMM || b2b_gemm) ? sizeof(bolt_gemm_desc) : sizeof(bolt_conv_desc);
  TuneKey key{(int)op, std::string((const char*)desc0, dsz)};
  if (is_b2b) key.bytes.append((const char*)desc1, dsz);

  bolt_status s;
  FpropProblem fp;
  B2bProblem bp;
  if (op == BOLT_OP_GEMM) s = make_gemm_problem((const bolt_gemm_desc*)desc0, &fp);
  else if (op == BOLT_OP_CONV2D) s = make_conv_problem((const bolt_conv_desc*)desc0, &fp);
  else if (b2b_gemm) s = make_b2b_gemm_problem((const bolt_gemm_desc*)desc0, (const bolt_gemm_desc*)desc1, &bp);
  else s = make_b2b_conv_problem((const bolt_conv_desc*)desc0, (const bolt_conv_desc*)desc1, &bp);
  if (s != BOLT_OK) return s;
  const int nptr = single ? 4 : with_res ? 7 : 6;  // the residual ops take the residual matrix as ptrs[6]
  for (int i = 0; i < nptr; ++i) {
    const bool optional = single ? (i == 2) : (i == 2 || i == 4);
    if (!ptrs[i] && !optional) return BOLT_ERR_INVALID_ARG;
    if (ptrs[i] && !is_aligned16(ptrs[i])) return BOLT_ERR_ALIGNMENT;
  }

  if (single) {
    // a winner found with a workspace may use split-K that a later call without one (or with a smaller one) cannot
    // run: the largest split the workspace admits is part of the key
    char ws_class = 1;
    const bool have_ws = workspace && is_aligned16(workspace);
    for (int sk = 2; sk <= kMaxSplitK; sk *= 2)
      if (have_ws && workspace_bytes >= splitk_bytes(fp.p.M, fp.p.N, sk)) ws_class = (char)sk;
    key.bytes.push_back(ws_class);
  }
  {
    std::lock_guard<std::mutex> lock(tune_mutex());
    auto it = tune_cache().find(key);
    if (it != tune_cache().end()) {
      *best = it->second.cfg;
      if (best_ms) *best_ms = it->second.ms;
      if (n_tried) *n_tried = it->second.tried;
      return BOLT_OK;
    }
  }

  Candidate win{};
  int tried = 0;
  bolt_config cfg;
  std::memset(&cfg, 0, sizeof(cfg));
  if (single) {
    const auto& tab = op == BOLT_OP_GEMM ? tables().gemm : tables().conv;
    fp.p.X = (const half_t*)ptrs[0]; fp.p.W = (const half_t*)ptrs[1];
    fp.p.bias = (const half_t*)ptrs[2]; fp.p.Y = (half_t*)ptrs[3];
    const bool have_ws = workspace && is_aligned16(workspace);
    std::vector<Candidate> cands = fprop_candidates(tab, fp, workspace_bytes, have_ws);
    if (cands.empty()) return BOLT_ERR_UNSUPPORTED;
    if (tune_log_enabled())
      std::fprintf(stderr, "[bolt_tune] problem op %d M %d N %d K %d: %zu candidates\n", (int)op, fp.p.M, fp.p.N, fp.p.K, cands.size());
    s = tune_candidates(cands, [&](const Candidate& c) {
      return fprop_launch(tab[c.id], fp, c.swizzle, c.split_k, workspace, workspace_bytes, stream);
    }, stream, &win, &tried);
    if (s != BOLT_OK) return s;
    fprop_fill_config(tab[win.id], win.id, &cfg);
    cfg.swizzle = win.swizzle;
    cfg.split_k = win.split_k;
  } else {
    const auto& tab = b2b_gemm ? tables().b2b_gemm : tables().b2b_conv;
    B2bParams& p = bp.p;
    p.X = (const half_t*)ptrs[0]; p.W0 = (const half_t*)ptrs[1]; p.b0 = (const half_t*)ptrs[2];
    p.W1 = (const half_t*)ptrs[3]; p.b1 = (const half_t*)ptrs[4]; p.Y = (half_t*)ptrs[5];
    if (with_res) {  // dense residual ([M][N1]), gamma 1: the timing does not depend on the values
      bp.residual = true;
      p.res = (const half_t*)ptrs[6]; p.ldr = p.N1; p.gamma = 1.f;
    }
    std::vector<Candidate> cands;
    for (int i = 0; i < (int)tab.size(); ++i)
      if (b2b_supports(tab, i, bp)) cands.push_back({i, 0, 1, 0.f});
    if (cands.empty()) return BOLT_ERR_UNSUPPORTED;
    if (tune_log_enabled())
      std::fprintf(stderr, "[bolt_tune] problem op %d M %d N0 %d K0 %d N1 %d: %zu candidates\n", (int)op, p.M, p.N0, p.K0, p.N1, cands.size());
    s = tune_candidates(cands, [&](const Candidate& c) { return b2b_launch(tab[c.id], bp, stream); }, stream, &win,
                        &tried);
    if (s != BOLT_OK) return s;
    b2b_fill_config(tab[win.id], win.id, &cfg);
  }
  *best = cfg;
  if (best_ms) *best_ms = win.ms;
  if (n_tried) *n_tried = tried;
  std::lock_guard<std::mutex> lock(tune_mutex());
  tune_cache()[key] = TuneVal{cfg, win.ms, tried};
  return BOLT_OK;
}

bolt_status bolt_check_chain(bolt_op op, int32_t n_ops, const void* const* descs, const bolt_config* config) {
  B2bProblem pr;
  bolt_status s = make_chain_problem(op, n_ops, descs, &pr);
  if (s != BOLT_OK) return s;
  int id;
  return resolve_chain(op == BOLT_OP_GEMM_CHAIN3 ? tables().gemm_chain : tables().conv_chain, pr, config, &id);
}

int32_t bolt_chain_instance_supports(bolt_op op, int32_t kernel_id, int32_t n_ops, const void* const* descs) {
  B2bProblem pr;
  if (make_chain_problem(op, n_ops, descs, &pr) != BOLT_OK) return 0;
  const auto& tab = op == BOLT_OP_GEMM_CHAIN3 ? tables().gemm_chain : tables().conv_chain;
  return kernel_id >= 0 && kernel_id < (int)tab.size() && chain_supports(tab, kernel_id, pr);
}

// ptrs: {x, w0, b0, w1, b1, w2, b2, y}
static bolt_status chain_bind(B2bProblem* pr, const void* const* ptrs) {
  for (int i = 0; i < 8; ++i) {
    const bool optional = i == 2 || i == 4 || i == 6;
    if (!ptrs[i] && !optional) return BOLT_ERR_INVALID_ARG;
    if (ptrs[i] && !is_aligned16(ptrs[i])) return BOLT_ERR_ALIGNMENT;
  }
  B2bParams& p = pr->p;
  p.X = (const half_t*)ptrs[0]; p.W0 = (const half_t*)ptrs[1]; p.b0 = (const half_t*)ptrs[2];
  p.W1 = (const half_t*)ptrs[3]; p.b1 = (const half_t*)ptrs[4]; p.W2 = (const half_t*)ptrs[5];
  p.b2 = (const half_t*)ptrs[6]; p.Y = (half_t*)ptrs[7];
  return BOLT_OK;
}

// res: null for the plain chain; else the full matrix of the last epilogue with row stride ldr (0: the last op's N)
static bolt_status chain_call(bolt_op op, int32_t n_ops, const void* const* descs, const void* x,
                              const void* const* weights, const void* const* biases, void* y, const bolt_config* config,
                              void* stream, bool with_res = false, const void* res = nullptr, int32_t ldr = 0,
                              float gamma = 0.f) {
  B2bProblem pr;
  bolt_status s = make_chain_problem(op, n_ops, descs, &pr);
  if (s != BOLT_OK) return s;
  if (!weights) return BOLT_ERR_INVALID_ARG;
  const void* ptrs[8] = {x, weights[0], biases ? biases[0] : nullptr, weights[1], biases ? biases[1] : nullptr,
                         weights[2], biases ? biases[2] : nullptr, y};
  if ((s = chain_bind(&pr, ptrs)) != BOLT_OK) return s;
  if (with_res) {
    if (!res) return BOLT_ERR_INVALID_ARG;
    if (ldr == 0) ldr = pr.p.N2;
    if (ldr < pr.p.N2) return BOLT_ERR_INVALID_ARG;
    if ((ldr & 7) || !is_aligned16(res)) return BOLT_ERR_ALIGNMENT;
    if (ldr > (1 << 21)) return BOLT_ERR_UNSUPPORTED;
    pr.p.res = (const half_t*)res; pr.p.ldr = ldr; pr.p.gamma = gamma;
  }
  const auto& tab = op == BOLT_OP_GEMM_CHAIN3 ? tables().gemm_chain : tables().conv_chain;
  int id;
  if ((s = resolve_chain(tab, pr, config, &id)) != BOLT_OK) return s;
  return chain_launch(tab[id], pr, (hipStream_t)stream);
}

bolt_status bolt_b2b_gemm_chain(int32_t n_ops, const bolt_gemm_desc* const* descs, const void* A0,
                                const void* const* weights, const void* const* biases, void* D,
                                const bolt_config* config, void* stream) {
  return chain_call(BOLT_OP_GEMM_CHAIN3, n_ops, (const void* const*)descs, A0, weights, biases, D, config, stream);
}

bolt_status bolt_b2b_conv_chain(int32_t n_ops, const bolt_conv_desc* const* descs, const void* x,
                                const void* const* weights, const void* const* biases, void* y,
                                const bolt_config* config, void* stream) {
  return chain_call(BOLT_OP_CONV_CHAIN3, n_ops, (const void* const*)descs, x, weights, biases, y, config, stream);
}

bolt_status bolt_b2b_gemm_chain_residual(int32_t n_ops, const bolt_gemm_desc* const* descs, const void* A0,
                                         const void* const* weights, const void* const* biases, const void* C,
                                         int32_t ldc, float gamma, void* D, const bolt_config* config, void* stream) {
  if (ldc <= 0) return BOLT_ERR_INVALID_ARG;
  return chain_call(BOLT_OP_GEMM_CHAIN3, n_ops, (const void* const*)descs, A0, weights, biases, D, config, stream, true,
                    C, ldc, gamma);
}

bolt_status bolt_b2b_conv_chain_residual(int32_t n_ops, const bolt_conv_desc* const* descs, const void* x,
                                         const void* const* weights, const void* const* biases, const void* residual,
                                         float gamma, void* y, const bolt_config* config, void* stream) {
  return chain_call(BOLT_OP_CONV_CHAIN3, n_ops, (const void* const*)descs, x, weights, biases, y, config, stream, true,
                    residual, 0, gamma);
}

bolt_status bolt_tune_chain(bolt_op op, int32_t n_ops, const void* const* descs, const void* const* ptrs, void* stream_v,
                            bolt_config* best, float* best_ms, int32_t* n_tried) {
  if (!ptrs || !best) return BOLT_ERR_INVALID_ARG;
  B2bProblem pr;
  bolt_status s = make_chain_problem(op, n_ops, descs, &pr);
  if (s != BOLT_OK) return s;
  if ((s = chain_bind(&pr, ptrs)) != BOLT_OK) return s;
  hipStream_t stream = (hipStream_t)stream_v;
  const auto& tab = op == BOLT_OP_GEMM_CHAIN3 ? tables().gemm_chain : tables().conv_chain;
  std::vector<Candidate> cands;
  for (int i = 0; i < (int)tab.size(); ++i)
    if (chain_supports(tab, i, pr)) cands.push_back({i, 0, 1, 0.f});
  if (cands.empty()) return BOLT_ERR_UNSUPPORTED;
  Candidate win{};
  int tried = 0;
  if (tune_log_enabled())
    std::fprintf(stderr, "[bolt_tune] problem op %d M %d N0 %d K0 %d N1 %d N2 %d: %zu candidates\n", (int)op, pr.p.M, pr.p.N0,
                 pr.p.K0, pr.p.N1, pr.p.N2, cands.size());
  s = tune_candidates(cands, [&](const Candidate& c) { return chain_launch(tab[c.id], pr, stream); }, stream, &win, &tried);
  if (s != BOLT_OK) return s;
  std::memset(best, 0, sizeof(*best));
  chain_fill_config(tab[win.id], win.id, best);
  if (best_ms) *best_ms = win.ms;
  if (n_tried) *n_tried = tried;
  return BOLT_OK;
}

bolt_status bolt_pad_channels_nhwc(const void* src, void* dst, int64_t pixels, int32_t C, int32_t C_padded,
                                   void* stream) {
  if (!src || !dst || pixels < 0 || C <= 0 || C_padded < C) return BOLT_ERR_INVALID_ARG;
  if (C_padded & 7) return BOLT_ERR_ALIGNMENT;
  if (!is_aligned16(dst)) return BOLT_ERR_ALIGNMENT;
  if (pixels == 0) return BOLT_OK;
  const int64_t total = pixels * (C_padded / 8);
  if (total >= (1ll << 31)) return BOLT_ERR_UNSUPPORTED;
  const int blocks = (int)std::min<int64_t>((total + 255) / 256, kNumCU * 16);
  // 32-bit reads need an even channel count and a 4-byte aligned source
  const bool even = !(C & 1) && !((uintptr_t)src & 3);
  hipLaunchKernelGGL(even ? pad_channels_kernel<true> : pad_channels_kernel<false>, dim3(blocks), dim3(256), 0,
                     (hipStream_t)stream, (const half_t*)src, (half_t*)dst, (int)pixels, C, C_padded);
  return hipGetLastError() == hipSuccess ? BOLT_OK : BOLT_ERR_LAUNCH;
}

static bolt_status check_layout_args(const void* src, const void* dst, int32_t N, int32_t C, int32_t H, int32_t W,
                                     int32_t C8, const void* nhwc_side) {
  if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0 || C8 < C) return BOLT_ERR_INVALID_ARG;
  if ((C8 & 7) || !is_aligned16(nhwc_side) || ((uintptr_t)src & 1) || ((uintptr_t)dst & 1)) return BOLT_ERR_ALIGNMENT;
  if ((int64_t)N * H * W * C8 >= (1ll << 40) || (int64_t)H * W >= (1ll << 30) || N > 65535) return BOLT_ERR_UNSUPPORTED;
  return BOLT_OK;
}

bolt_status bolt_nchw_to_nhwc(const void* src, void* dst, int32_t N, int32_t C, int32_t H, int32_t W, int32_t C_padded,
                              void* stream) {
  bolt_status s = check_layout_args(src, dst, N, C, H, W, C_padded, dst);
  if (s != BOLT_OK) return s;
  const int HW = H * W;
  if (C_padded == 8) {
    const int64_t pixels = (int64_t)N * HW;
    const int blocks = (int)std::min<int64_t>((pixels + 255) / 256, kNumCU * 16);
    hipLaunchKernelGGL(nchw_to_nhwc8_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const half_t*)src,
                       (half_t*)dst, C, HW, pixels);
    return hipGetLastError() == hipSuccess ? BOLT_OK : BOLT_ERR_LAUNCH;
  }
  const dim3 grid(ceil_div(HW, kLayoutTile), ceil_div(C_padded, kLayoutTile), N);
  if (grid.y > 65535) return BOLT_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(nchw_to_nhwc_kernel, grid, dim3(256), 0, (hipStream_t)stream, (const half_t*)src, (half_t*)dst, C, HW,
                     C_padded);
  return hipGetLastError() == hipSuccess ? BOLT_OK : BOLT_ERR_LAUNCH;
}

bolt_status bolt_nhwc_to_nchw(const void* src, void* dst, int32_t N, int32_t C, int32_t H, int32_t W, int32_t C_src,
                              void* stream) {
  bolt_status s = check_layout_args(src, dst, N, C, H, W, C_src, src);
  if (s != BOLT_OK) return s;
  const int HW = H * W;
  const dim3 grid(ceil_div(HW, kLayoutTile), ceil_div(C, kLayoutTile), N);
  if (grid.y > 65535) return BOLT_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(nhwc_to_nchw_kernel, grid, dim3(256), 0, (hipStream_t)stream, (const half_t*)src, (half_t*)dst, C, HW,
                     C_src);
  return hipGetLastError() == hipSuccess ? BOLT_OK : BOLT_ERR_LAUNCH;
}

bolt_status bolt_bias_act(void* D, const void* bias, int64_t M, int32_t N, int32_t ldd, float alpha, float beta,
                          bolt_act act, void* stream) {
  if (M < 0 || N <= 0 || ldd < N || (M > 0 && !D)) return BOLT_ERR_INVALID_ARG;
  if ((int)act < (int)BOLT_ACT_NONE || (int)act > (int)BOLT_ACT_SOFTPLUS) return BOLT_ERR_INVALID_ARG;
  if ((N & 7) || (ldd & 7) || !is_aligned16(D) || (bias && !is_aligned16(bias))) return BOLT_ERR_ALIGNMENT;
  if (M == 0) return BOLT_OK;
  const int64_t total = M * (N / 8);
  const int blocks = (int)std::min<int64_t>((total + 255) / 256, kNumCU * 16);
  hipLaunchKernelGGL(bias_act_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (half_t*)D,
                     (const half_t*)bias, M, N, ldd, alpha, beta, (int)act);
  return hipGetLastError() == hipSuccess ? BOLT_OK : BOLT_ERR_LAUNCH;
}

bolt_status bolt_probe_mfma_peak(int32_t iterations, void* stream_v, float* tflops) {
  if (iterations <= 0 || !tflops) return BOLT_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_v;
  float* sink = (float*)scratch_of_current_device();  // never written in practice (see mfma_peak_kernel)
  if (!sink) return BOLT_ERR_LAUNCH;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  const int blocks = kNumCU * 2;  // 8 waves per CU: 2 per SIMD
  float ms = 0.f;
  bolt_status s = time_launches([&] {
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(blocks), dim3(256), 0, stream, sink, iterations);
    return hipGetLastError() == hipSuccess ? BOLT_OK : BOLT_ERR_LAUNCH;
  }, 1, 3, stream, e0, e1, &ms);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (s != BOLT_OK) return s;
  const double flop = (double)blocks * 4 /*waves*/ * iterations * 16.0 * (2.0 * 16 * 16 * 32);
  *tflops = (float)(flop / (ms * 1e-3) / 1e12);
  return BOLT_OK;
}

bolt_status bolt_probe_copy_bandwidth(void* buffer, size_t bytes, int32_t repeats, void* stream_v, float* gbps) {
  if (!buffer || bytes < 64 || repeats <= 0 || !gbps) return BOLT_ERR_INVALID_ARG;
  if (!is_aligned16(buffer)) return BOLT_ERR_ALIGNMENT;
  hipStream_t stream = (hipStream_t)stream_v;
  const int64_t n16 = (int64_t)(bytes / 2 / 16);
  const floatx4* src = (const floatx4*)buffer;
  floatx4* dst = (floatx4*)buffer + n16;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  float ms = 0.f;
  const int blocks = (int)std::min<int64_t>((n16 + 255) / 256, kNumCU * 32);
  bolt_status s = time_launches([&] {
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, stream, src, dst, n16);
    return hipGetLastError() == hipSuccess ? BOLT_OK : BOLT_ERR_LAUNCH;
  }, 1, repeats, stream, e0, e1, &ms);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (s != BOLT_OK) return s;
  *gbps = (float)(2.0 * n16 * 16 / (ms * 1e-3) / 1e9);
  return BOLT_OK;
}

}  // extern "C"
