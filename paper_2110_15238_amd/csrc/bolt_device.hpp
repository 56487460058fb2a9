// Device-side building blocks shared by every kernel template of the library (gfx950 / CDNA4).
//
// Vocabulary (Section 2.2 / Figure 2 of the paper, mapped to CDNA4): threadblock tile -> workgroup
// tile, warp tile -> wave tile (64 lanes), tensor-core instruction -> v_mfma_f32_32x32x16_f16,
// shared memory -> LDS, register file -> VGPR/AGPR.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

namespace bolt {

typedef _Float16 half_t;
typedef half_t half2v __attribute__((ext_vector_type(2)));
typedef half_t half4 __attribute__((ext_vector_type(4)));
typedef half_t half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2, ACT_HARDSWISH = 3, ACT_SOFTPLUS = 4 };

// One matrix-core instruction: D(32x32) += A(32x16) * B(16x32), FP16 inputs, FP32 accumulate.
// Lane l supplies A[i = l%32][k = 8*(l/32) .. +7] and B[k = 8*(l/32) .. +7][j = l%32];
// it receives D[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32] in accumulator register r (0..15).
__device__ __forceinline__ floatx16 mfma_32x32x16(half8 a, half8 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// The 16 x 16 x 32 form: D(16x16) += A(16x32) * B(32x16).  Lane l supplies A[i = l%16][k = 8*(l/16) .. +7] and
// B[k = 8*(l/16) .. +7][j = l%16]; it receives D[i = 4*(l/16) + r][j = l%16] in register r (0..3).  It does the
// same FLOPs per cycle as the 32 x 32 x 16 form with a quarter of the accumulator traffic per instruction; under
// the chip's power limit an MFMA-only loop on random FP16 operands sustains 1.96 PFLOP/s with it against 1.68.
__device__ __forceinline__ floatx4 mfma_16x16x32(half8 a, half8 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// LDS operand tiles are [rows][BK] halves, K contiguous, addressed in 16-byte chunks of 8 halves.
// The LDS has 64 banks of 4 bytes; 128-bit accesses are served 16 lanes at a time, so 16 lanes
// should land in 16 different 16-byte bank groups, bank group = (byte address / 16) mod 16.
// The chunk index is XOR-swizzled by row bits so that (a) the 16 lanes of a fragment read, which
// touch 16 consecutive rows at one logical chunk, are conflict-free and (b) the 16 lanes of a
// transposing store, which touch rows 8 apart at one logical chunk, conflict only 2-way.
template <int BK>
__device__ __forceinline__ int lds_chunk_offset(int row, int chunk) {
  static_assert(BK == 32 || BK == 64, "BK");
  if constexpr (BK == 32) {
    return row * 32 + ((chunk ^ (((row >> 2) ^ (row >> 4)) & 3)) << 3);
  } else {
    return row * 64 + ((chunk ^ (((row >> 1) ^ (row >> 4)) & 7)) << 3);
  }
}

// Transcendental activations in FP32 with the hardware exp2 / log2 / rcp units.  Their relative error
// (below 1e-5) is far under half an FP16 ulp (4.9e-4), the rounding the result gets anyway.
//
// GELU = v * Phi(v), Phi(v) = erfc(-v / sqrt 2) / 2.  With z = |v| / sqrt 2 and t = 1 / (1 + z / 2),
// erfc(z) = t * Q(t) * exp(-z^2), where Q is a degree-7 polynomial fitted (Chebyshev nodes on t in
// (0, 1], float64 scaled-erfc as the target) to 4.6e-6 relative error.  This form has no cancellation in
// the negative tail, where 1 + erf(v / sqrt 2) would lose every digit.
__device__ __forceinline__ float gelu_fast(float v) {
  const float z = fabsf(v) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(1.f + 0.5f * z);
  float q = 4.458448196e-02f;
  q = q * t + -8.891160022e-02f;
  q = q * t + -6.914768965e-02f;
  q = q * t + 1.436112067e-01f;
  q = q * t + 1.560333553e-01f;
  q = q * t + 2.497963131e-01f;
  q = q * t + 2.819394284e-01f;
  q = q * t + 2.820960852e-01f;
  const float h = 0.5f * t * q * __builtin_amdgcn_exp2f(z * z * -1.44269504088896340736f);  // erfc(z) / 2
  return v * (v < 0.f ? h : 1.f - h);
}

// softplus = max(v, 0) + log1p(e), e = exp(-|v|) in (0, 1]: three series terms while e is small (the
// sum 1 + e would round e away), the log2 unit otherwise.
__device__ __forceinline__ float softplus_fast(float v) {
  const float e = __builtin_amdgcn_exp2f(fabsf(v) * -1.44269504088896340736f);
  const float series = e * (1.f + e * (-0.5f + e * 0.33333333333f));
  const float direct = __builtin_amdgcn_logf(1.f + e) * 0.69314718055994530942f;
  return fmaxf(v, 0.f) + (e < 0.015625f ? series : direct);
}

__device__ __forceinline__ float hardswish_fast(float v) {
  return v * fminf(fmaxf(v + 3.f, 0.f), 6.f) * (1.f / 6.f);
}

// The fully unrolled epilogues call this once per 4 outputs; out of line so that they stay small.
// act is wave-uniform: the switch is scalar branches.
__device__ __attribute__((noinline)) floatx4 apply_act_slow4(floatx4 v, int act) {
  switch (act) {
    case ACT_GELU:
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = gelu_fast(v[e]);
      break;
    case ACT_HARDSWISH:
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = hardswish_fast(v[e]);
      break;
    case ACT_SOFTPLUS:
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = softplus_fast(v[e]);
      break;
    default: break;
  }
  return v;
}

__device__ __forceinline__ float apply_act(float v, int act) {
  switch (act) {
    case ACT_RELU: return v > 0.f ? v : 0.f;
    case ACT_GELU: return gelu_fast(v);
    case ACT_HARDSWISH: return hardswish_fast(v);
    case ACT_SOFTPLUS: return softplus_fast(v);
    default: return v;
  }
}

// Fused epilogue arithmetic (Section 3.1, patterns (i)-(iii)) for one quad of an accumulator
// fragment: 4 consecutive columns n .. n+3 of one output row, registers 4q .. 4q+3.
//   out = act(alpha * acc + beta * bias[n + e]),  converted to FP16 with round-to-nearest-even.
// The caller never passes a null bias: without a bias the pointer addresses 8 zero halves and
// bias_on is 0, which keeps the hot path free of branches (the loads can be scheduled early).
// Columns beyond N take a zero bias; their results are never stored.
// SLOW = false handles "none" and ReLU with a select; SLOW = true calls the transcendental
// activations.  The choice between the two is ONE wave-uniform branch around a whole tile.
struct EpilogueArgs {
  const half_t* bias;
  int bias_on, N;
  float alpha, beta;
  int act;
  float gamma = 0.f;  // scale of the residual quad (Eq. 1 with a full matrix C), epilogue_quad_res only
};

template <bool SLOW, bool RES>
__device__ __forceinline__ half4 epilogue_quad4_impl(floatx4 a4, int n, const EpilogueArgs& ep, half4 res) {
  // columns beyond N (the zero-padded part of a compiled width) take a zero bias: their value is act(0), finite
  // whatever beta * bias is, so a fused op that multiplies them by zero weights never sees inf * 0
  const half4 hb_in = *(const half4*)(ep.bias + (n < ep.N ? n : 0) * ep.bias_on);
  const half4 hb = n < ep.N ? hb_in : half4{0, 0, 0, 0};
  half4 o;
  floatx4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v[e] = ep.alpha * a4[e] + ep.beta * (float)hb[e];
    if constexpr (RES) v[e] += ep.gamma * (float)res[e];
  }
  if constexpr (SLOW) {
    v = apply_act_slow4(v, ep.act);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float r = v[e] > 0.f ? v[e] : 0.f;
      v[e] = ep.act == ACT_RELU ? r : v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (half_t)v[e];
  return o;
}
template <bool SLOW, bool RES>
__device__ __forceinline__ half4 epilogue_quad_impl(const floatx16& acc, int q, int n, const EpilogueArgs& ep, half4 res) {
  const floatx4 a4 = {acc[q * 4], acc[q * 4 + 1], acc[q * 4 + 2], acc[q * 4 + 3]};
  return epilogue_quad4_impl<SLOW, RES>(a4, n, ep, res);
}
template <bool SLOW>
__device__ __forceinline__ half4 epilogue_quad(const floatx16& acc, int q, int n, const EpilogueArgs& ep) {
  const half4 none = {0, 0, 0, 0};
  return epilogue_quad_impl<SLOW, false>(acc, q, n, ep, none);
}
// The same with a residual: out = act(alpha * acc + beta * bias[n + e] + gamma * res[e]) (Eq. 1, C a full matrix).
template <bool SLOW>
__device__ __forceinline__ half4 epilogue_quad_res(const floatx16& acc, int q, int n, const EpilogueArgs& ep, half4 res) {
  return epilogue_quad_impl<SLOW, true>(acc, q, n, ep, res);
}

// XOR term of the FP16 C tile staged in LDS ([rows][BN], 16-byte chunks): physical chunk = chunk ^ term(row).
// The term walks through all 16 bank groups (256 bytes) over 16 consecutive rows whatever the row length,
// so the 8-byte accumulator-quad writes of 32 rows conflict two ways (rows r and r + 16) instead of four, and
// the 16-byte reads of the store phase (16 lanes: consecutive chunks of one or two rows) not at all.
template <int CPR>
__device__ __forceinline__ int ctile_swizzle(int row) {
  static_assert(CPR == 4 || CPR == 8 || CPR == 16 || CPR == 32, "chunks per C-tile row");
  return CPR >= 16 ? (row & 15) : CPR == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

// Host side: a kernel that wants more than 64 KiB of dynamic LDS has to opt in once per process.  Every launcher
// owns one of these per kernel; call_once makes the first launch safe from several host threads, and the
// attribute is set before (never as part of) the first launch, so it does not matter whether that launch is
// being captured into a graph.
struct LdsOptIn {
  std::once_flag once;
  hipError_t status = hipSuccess;
  hipError_t ensure(const void* kernel, int bytes) {
    std::call_once(once, [&] { status = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
    return status;
  }
};

// Workgroup id -> output tile.  mode 0: n-tile fastest.  mode g > 0: ids are first regrouped so
// that the ids one XCD receives (hardware deals consecutive ids round-robin over 8 XCDs, each with
// a private L2) are consecutive, then walked in bands of g m-tiles x all n-tiles.
__device__ __forceinline__ void tile_of_workgroup(int bid, int tiles_m, int tiles_n, int mode, int& tm, int& tn) {
  if (mode <= 0) {
    tm = bid / tiles_n;
    tn = bid - tm * tiles_n;
    return;
  }
  const int total = tiles_m * tiles_n;
  const int xcd = bid & 7, idx = bid >> 3;
  const int per = total >> 3, rem = total & 7;
  int pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  const int width = mode * tiles_n;
  const int group = pid / width;
  const int first_m = group * mode;
  const int gsz = (tiles_m - first_m) < mode ? (tiles_m - first_m) : mode;
  const int in_group = pid - group * width;
  tm = first_m + in_group % gsz;
  tn = in_group / gsz;
}

}  // namespace bolt
