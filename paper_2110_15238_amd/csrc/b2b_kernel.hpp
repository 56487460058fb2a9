// Persistent back-to-back GEMM / conv kernels (Section 3.1.1 of the paper).
//
//   D0 = act0(alpha0 * X . W0 + beta0 * b0)   rounded to FP16, never written to global memory
//   D1 = act1(alpha1 * D0 . W1 + beta1 * b1)
//
// Threadblock residence: a workgroup tile covers BM rows and ALL columns of both ops (N0T >= N0,
// N1T >= N1 are compile-time upper bounds; missing weight rows are zero-filled).  Both weight
// matrices are loaded into LDS once per workgroup (160 KB of LDS per CU makes that possible for
// the memory-bound shapes fusion targets) and the workgroup then walks over row tiles
// persistently, streaming only activations.
//
//   b2b_rf_kernel  (RF-resident fusion): waves split the tile along M only, so a wave owns whole
//     rows of D0.  The MFMA computes the transposed product, hence a lane's accumulators are runs
//     of 4 consecutive D0 columns of ONE row: exactly a B-operand fragment of the second MFMA up
//     to a permutation of the reduction index, which is applied to the W1 fragment reads instead.
//     The epilogue of op0 is done on those registers; D0 never leaves the register file.
//   b2b_lds_kernel (LDS-resident fusion): waves tile op0 in 2-D; the FP16 D0 tile is stored to LDS
//     in the swizzled operand layout and re-read as the activation operand of op1 by a different
//     2-D wave tiling, which lifts the "wave tile N = N" restriction.
#pragma once
#include <type_traits>

#include "bolt_device.hpp"
#include "fprop_dma_kernel.hpp"
#include "tile_loaders.hpp"

namespace bolt {

struct B2bParams {
  const half_t* X;
  const half_t* W0;
  const half_t* b0;  // biases are never null inside the kernels (see EpilogueArgs)
  const half_t* W1;
  const half_t* b1;
  half_t* Y;
  int b0_on, b1_on;
  int M, N0, K0, N1;
  int ldx, ldw0, ldw1, ldy;
  float alpha0, beta0, alpha1, beta1;
  int act0, act1;
  int tiles_m;
  ConvGeom cg;  // XMODE 1 only (geometry of op0)
  // third op of a chain (b2b_chain_kernel.hpp); N2 == 0 for the two-op kernels
  const half_t* W2;
  const half_t* b2;
  int b2_on, N2, ldw2;
  float alpha2, beta2;
  int act2;
  // full-matrix C of the last op (Eq. 1), [M][N1] with leading dimension ldr, scaled by gamma; null = none
  const half_t* res;
  int ldr;
  float gamma;
};

template <int N0T>
struct B2bK1 {
  static constexpr int KB1 = N0T < 64 ? N0T : 64;  // K-tile width of op1's LDS operands
  static constexpr int NKT1 = N0T / KB1;
};

// Row-major weights ([K][N]) stay row-major in LDS: W0 as [nk0 * BK][N0T], W1 as [N0T][N1T], fetched with
// direct-to-LDS loads (no registers, no transposes; one memory round trip that the first activation tile shares) and
// read as matrix-core operands with the LDS transpose read (kn_frag_read).  Issues the loads only: the kernels wait
// for them in front of the first workgroup barrier of their tile loop.
template <int BK, int NT, int N0T, int N1T>
__device__ __forceinline__ void b2b_preload_weights_kn(const B2bParams& p, half_t* W0s, half_t* W1s, int tid) {
  const int nk0 = (p.K0 + BK - 1) / BK;
  kn_matrix_to_lds<NT, N0T>(p.W0, p.ldw0, p.K0, p.N0, nk0 * BK, W0s, tid);
  kn_matrix_to_lds<NT, N1T>(p.W1, p.ldw1, p.N0, p.N1, N0T, W1s, tid);
}

// Loads W0 as [nk0][N0T][BK] and W1 as [N0T/KB1][N1T][KB1] into LDS (all threads, then barrier).
template <int BK, int NT, int N0T, int N1T, int WMODE>
__device__ __forceinline__ void b2b_preload_weights(const B2bParams& p, half_t* W0s, half_t* W1s, int tid) {
  if constexpr (WMODE == 1) {
    b2b_preload_weights_kn<BK, NT, N0T, N1T>(p, W0s, W1s, tid);
    return;
  }
  constexpr int KB1 = B2bK1<N0T>::KB1;
  const int nk0 = (p.K0 + BK - 1) / BK;
  {
    WTileLoader<N0T, BK, NT, WMODE> wl;
    wl.init(p.W0, p.ldw0, p.N0, p.K0, 0, tid);
    for (int kt = 0; kt < nk0; ++kt) {
      wl.load(kt);
      wl.store(W0s + kt * N0T * BK);
    }
  }
  {
    WTileLoader<N1T, KB1, NT, WMODE> wl;
    wl.init(p.W1, p.ldw1, p.N1, p.N0, 0, tid);
#pragma unroll
    for (int kt = 0; kt < B2bK1<N0T>::NKT1; ++kt) {
      wl.load(kt);
      wl.store(W1s + kt * N1T * KB1);
    }
  }
  __syncthreads();
}

// Epilogue of op0 in registers (RF-resident fusion): accumulators -> FP16 B-operand fragments of
// op1.  Step t = 2a + h of op1 reduces over D0 columns [32a + 16h, 32a + 16h + 16): lane group g
// holds columns 32a+16h+4g+{0..3} (accumulator quad 2h) and 32a+16h+8+4g+{0..3} (quad 2h+1), and the
// W1 fragment reads apply the same permutation of the reduction index.  Columns >= N0 become 0.
template <int FN0, int FM>
__device__ __forceinline__ void b2b_make_d(const EpilogueArgs& ep, const floatx16 (&acc0)[FN0][FM], half8 (&d0)[FN0 * 2][FM],
                                           int g) {
  auto make = [&](auto slow) {
#pragma unroll
    for (int a = 0; a < FN0; ++a)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int c0 = a * 32 + h * 16 + g * 4;
#pragma unroll
        for (int b = 0; b < FM; ++b) {
          half4 lo = epilogue_quad<decltype(slow)::value>(acc0[a][b], 2 * h, c0, ep);
          half4 hi = epilogue_quad<decltype(slow)::value>(acc0[a][b], 2 * h + 1, c0 + 8, ep);
          const half4 z = {0, 0, 0, 0};
          if (c0 >= ep.N) lo = z;
          if (c0 + 8 >= ep.N) hi = z;
          const half8 d = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          d0[a * 2 + h][b] = d;
        }
      }
  };
  if (ep.act > ACT_RELU) make(std::true_type{});
  else make(std::false_type{});
}
template <int FN0, int FM>
__device__ __forceinline__ void b2b_make_d0(const B2bParams& p, const floatx16 (&acc0)[FN0][FM], half8 (&d0)[FN0 * 2][FM],
                                            int g) {
  b2b_make_d<FN0, FM>(EpilogueArgs{p.b0, p.b0_on, p.N0, p.alpha0, p.beta0, p.act0}, acc0, d0, g);
}

// Epilogue of op1 for a 2-D wave tiling, through LDS: accumulators -> FP16 tile [BM][NOUT_T] in `stage` (16-byte
// chunks XOR-swizzled by row, see ctile_swizzle) -> 16-byte non-temporal row stores, every instruction whole
// 128-byte row segments (one 8-byte store per accumulator quad straight from the MFMA layout is four times the
// instructions at a quarter of the bytes each: measured 1 us more on a 64 x 128 tile).  `stage` may overlay whatever op1 has finished reading: the first
// barrier orders that, the last one lets the next tile re-use the memory.  RES: Eq. 1 with a full matrix C - each
// lane first reads the quad of C that its quad of D will replace (8-byte loads; C may be the output buffer), p.gamma
// scales it.
template <int BM, int NOUT_T, int WTM, int WTN, int NT, bool RES>
__device__ __forceinline__ void b2b_tile_out_2d(half_t* stage, const floatx16 (&acc)[WTN / 32][WTM / 32], const B2bParams& p,
                                                int m0, int wm, int wn, int tid, int n_off = 0) {
  // n_off: the staged tile is columns [n_off, n_off + NOUT_T) of D1 (kernels that take op1 a column chunk at a time)
  constexpr int CPR = NOUT_T / 8, ROWS_PER_PASS = NT / CPR;
  static_assert(NT % CPR == 0 && BM % ROWS_PER_PASS == 0, "C tile store mapping");
  const int lane = tid & 63, g = lane >> 5, l32 = lane & 31;
  const int n_valid = p.N1 - n_off;
  const EpilogueArgs ep{p.b1 + n_off, p.b1_on, n_valid, p.alpha1, p.beta1, p.act1, RES ? p.gamma : 0.f};
  __syncthreads();
  auto to_lds = [&](auto slow) {
#pragma unroll
    for (int a = 0; a < WTN / 32; ++a)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nl = wn * WTN + a * 32 + q * 8 + g * 4;
#pragma unroll
        for (int b = 0; b < WTM / 32; ++b) {
          const int row = wm * WTM + b * 32 + l32;
          half4 o;
          if constexpr (RES) {
            half4 c = {0, 0, 0, 0};
            if (nl < n_valid && m0 + row < p.M) c = *(const half4*)(p.res + (int64_t)(m0 + row) * p.ldr + n_off + nl);
            o = epilogue_quad_res<decltype(slow)::value>(acc[a][b], q, nl, ep, c);
          } else {
            o = epilogue_quad<decltype(slow)::value>(acc[a][b], q, nl, ep);
          }
          *(half4*)(stage + row * NOUT_T + (((nl >> 3) ^ ctile_swizzle<CPR>(row)) << 3) + (nl & 4)) = o;
        }
      }
  };
  if (p.act1 > ACT_RELU) to_lds(std::true_type{});
  else to_lds(std::false_type{});
  __syncthreads();
  const int chunk = tid % CPR, r0 = tid / CPR;
  if (chunk * 8 < n_valid) {
#pragma unroll
    for (int i = 0; i < BM / ROWS_PER_PASS; ++i) {
      const int row = r0 + i * ROWS_PER_PASS;
      if (m0 + row < p.M) {
        const half8 v = *(const half8*)(stage + row * NOUT_T + ((chunk ^ ctile_swizzle<CPR>(row)) << 3));
        __builtin_nontemporal_store(v, (half8*)(p.Y + (int64_t)(m0 + row) * p.ldy + n_off + chunk * 8));
      }
    }
  }
  __syncthreads();
}

template <int BM, int BK, int NWAVES, int N0T, int N1T, int XMODE, int WMODE>
struct B2bRfTraits {
  static constexpr int NT = 64 * NWAVES;
  static constexpr int WTM = BM / NWAVES, FM = WTM / 32;
  static constexpr int FN0 = N0T / 32, FN1 = N1T / 32;
  static constexpr int NC1 = FN1 < 4 ? FN1 : 4;  // op1 accumulators live NC1 column fragments at a time
  static_assert(WTM % 32 == 0 && N0T % 32 == 0 && N1T % 32 == 0 && FN1 % NC1 == 0, "tile shape");
  static int lds_bytes(int K0) {
    const int nk0 = (K0 + BK - 1) / BK;
    return (nk0 * N0T * BK + N0T * N1T + 2 * BM * BK) * 2;
  }
};

template <int BM, int BK, int NWAVES, int N0T, int N1T, int XMODE, int WMODE, bool RES = false>
__global__ __launch_bounds__(64 * NWAVES) void b2b_rf_kernel(const B2bParams p) {
  using T = B2bRfTraits<BM, BK, NWAVES, N0T, N1T, XMODE, WMODE>;
  constexpr int NT = T::NT, WTM = T::WTM, FM = T::FM, FN0 = T::FN0, FN1 = T::FN1, NC1 = T::NC1;
  constexpr int KB1 = B2bK1<N0T>::KB1;

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  const int nk0 = (p.K0 + BK - 1) / BK;
  half_t* W0s = lds;
  half_t* W1s = W0s + nk0 * N0T * BK;
  half_t* Xs = W1s + N0T * N1T;  // [2][BM*BK]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, l32 = lane & 31;
  b2b_preload_weights<BK, NT, N0T, N1T, WMODE>(p, W0s, W1s, tid);
  int w0off[WMODE == 1 ? FN0 : 1], w1off[WMODE == 1 ? FN1 : 1];  // row-major weights: lane offsets of the transpose reads
  if constexpr (WMODE == 1) {
#pragma unroll
    for (int a = 0; a < FN0; ++a) w0off[a] = kn_frag_offset<N0T>(a * 32, lane);
#pragma unroll
    for (int a = 0; a < FN1; ++a) w1off[a] = kn_frag_offset<N1T>(a * 32, lane, 4);
  }

  for (int tile = blockIdx.x; tile < p.tiles_m; tile += gridDim.x) {
    const int m0 = tile * BM;
    XTileLoader<BM, BK, NT, XMODE> xl;
    xl.init(p.X, p.ldx, p.M, p.K0, p.cg, m0, 0, tid);

    floatx16 acc0[FN0][FM];
#pragma unroll
    for (int a = 0; a < FN0; ++a)
#pragma unroll
      for (int b = 0; b < FM; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc0[a][b][r] = 0.f;

    // ---- op0 main loop: X streamed through a double-buffered LDS tile, W0 resident ----------
    xl.load(0, p.cg);
    xl.store(Xs);
    if constexpr (WMODE == 1) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's weight loads have landed
    __syncthreads();
    for (int kt = 0; kt < nk0; ++kt) {
      const int buf = kt & 1;
      const bool more = kt + 1 < nk0;
      if (more) xl.load(kt + 1, p.cg);
      const half_t* xs = Xs + buf * BM * BK;
      const half_t* ws = W0s + kt * N0T * BK;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        half8 xf[FM], wf[FN0];
        const int chunk = ks * 2 + g;
#pragma unroll
        for (int b = 0; b < FM; ++b) xf[b] = *(const half8*)(xs + lds_chunk_offset<BK>(wave * WTM + b * 32 + l32, chunk));
#pragma unroll
        for (int a = 0; a < FN0; ++a) {
          if constexpr (WMODE == 1) wf[a] = kn_frag_read<N0T>(W0s, w0off[a], kt * BK + ks * 16);
          else wf[a] = *(const half8*)(ws + lds_chunk_offset<BK>(a * 32 + l32, chunk));
        }
#pragma unroll
        for (int a = 0; a < FN0; ++a)
#pragma unroll
          for (int b = 0; b < FM; ++b) acc0[a][b] = mfma_32x32x16(wf[a], xf[b], acc0[a][b]);
      }
      if (more) xl.store(Xs + (buf ^ 1) * BM * BK);
      __syncthreads();
    }

    // ---- epilogue0 in registers: accumulators -> FP16 B-operand fragments of op1 ------------
    half8 d0[FN0 * 2][FM];
    b2b_make_d0<FN0, FM>(p, acc0, d0, g);

    // ---- op1: W1 fragments from LDS with the matching reduction-index permutation ------------
#pragma unroll
    for (int c1 = 0; c1 < FN1 / NC1; ++c1) {
      floatx16 acc1[NC1][FM];
#pragma unroll
      for (int a = 0; a < NC1; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc1[a][b][r] = 0.f;
#pragma unroll
      for (int t = 0; t < FN0 * 2; ++t) {
        const int kbase = t * 16;            // first D0 column of this step
        const int kt1 = kbase / KB1;         // LDS k-tile of W1
        const int chunk = (kbase % KB1) / 8; // chunk of columns kbase .. kbase+7 (then +1)
        const half_t* ws = W1s + kt1 * N1T * KB1;
#pragma unroll
        for (int a = 0; a < NC1; ++a) {
          const int row = (c1 * NC1 + a) * 32 + l32;
          half8 wf;
          if constexpr (WMODE == 1) {
            wf = kn_frag_read<N1T>(W1s, w1off[c1 * NC1 + a], kbase, 8);
          } else {
            const half4 lo = *(const half4*)(ws + lds_chunk_offset<KB1>(row, chunk) + g * 4);
            const half4 hi = *(const half4*)(ws + lds_chunk_offset<KB1>(row, chunk + 1) + g * 4);
            wf = half8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          }
#pragma unroll
          for (int b = 0; b < FM; ++b) acc1[a][b] = mfma_32x32x16(wf, d0[t][b], acc1[a][b]);
        }
      }
      // this chunk's [BM][NC1 * 32] columns through a staged tile over the activation buffers
      if (c1 * NC1 * 32 < p.N1) b2b_tile_out_2d<BM, NC1 * 32, WTM, NC1 * 32, NT, RES>(Xs, acc1, p, m0, wave, 0, tid, c1 * NC1 * 32);
    }
  }
}

template <int BM, int BK, int WM0, int WN0, int WM1, int WN1, int N0T, int N1T, int XMODE, int WMODE>
struct B2bLdsTraits {
  static constexpr int NT = 64 * WM0 * WN0;
  static_assert(WM0 * WN0 == WM1 * WN1, "both wave grids use the same waves");
  static constexpr int WTM0 = BM / WM0, WTN0 = N0T / WN0, FM0 = WTM0 / 32, FN0 = WTN0 / 32;
  static constexpr int WTM1 = BM / WM1, WTN1 = N1T / WN1, FM1 = WTM1 / 32, FN1 = WTN1 / 32;
  static_assert(WTM0 % 32 == 0 && WTN0 % 32 == 0 && WTM1 % 32 == 0 && WTN1 % 32 == 0, "tile shape");
  static int lds_bytes(int K0) {
    const int nk0 = (K0 + BK - 1) / BK;
    constexpr int loop_halves = 2 * BM * BK + BM * N0T, out_halves = BM * N1T;  // the output tile overlays X and D0
    return (nk0 * N0T * BK + N0T * N1T + (loop_halves > out_halves ? loop_halves : out_halves)) * 2;
  }
};

template <int BM, int BK, int WM0, int WN0, int WM1, int WN1, int N0T, int N1T, int XMODE, int WMODE, bool RES = false>
__global__ __launch_bounds__(64 * WM0 * WN0) void b2b_lds_kernel(const B2bParams p) {
  using T = B2bLdsTraits<BM, BK, WM0, WN0, WM1, WN1, N0T, N1T, XMODE, WMODE>;
  constexpr int NT = T::NT, FM0 = T::FM0, FN0 = T::FN0, FM1 = T::FM1, FN1 = T::FN1;
  constexpr int WTM0 = T::WTM0, WTN0 = T::WTN0, WTM1 = T::WTM1, WTN1 = T::WTN1;
  constexpr int KB1 = B2bK1<N0T>::KB1, NKT1 = B2bK1<N0T>::NKT1;

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  const int nk0 = (p.K0 + BK - 1) / BK;
  half_t* W0s = lds;
  half_t* W1s = W0s + nk0 * N0T * BK;
  half_t* Xs = W1s + N0T * N1T;    // [2][BM*BK]
  half_t* D0s = Xs + 2 * BM * BK;  // [NKT1][BM*KB1]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, l32 = lane & 31;
  const int wm0 = wave % WM0, wn0 = wave / WM0;
  const int wm1 = wave % WM1, wn1 = wave / WM1;
  b2b_preload_weights<BK, NT, N0T, N1T, WMODE>(p, W0s, W1s, tid);
  int w0off[WMODE == 1 ? FN0 : 1], w1off[WMODE == 1 ? FN1 : 1];  // row-major weights: lane offsets of the transpose reads
  if constexpr (WMODE == 1) {
#pragma unroll
    for (int a = 0; a < FN0; ++a) w0off[a] = kn_frag_offset<N0T>(wn0 * WTN0 + a * 32, lane);
#pragma unroll
    for (int a = 0; a < FN1; ++a) w1off[a] = kn_frag_offset<N1T>(wn1 * WTN1 + a * 32, lane);
  }

  for (int tile = blockIdx.x; tile < p.tiles_m; tile += gridDim.x) {
    const int m0 = tile * BM;
    XTileLoader<BM, BK, NT, XMODE> xl;
    xl.init(p.X, p.ldx, p.M, p.K0, p.cg, m0, 0, tid);

    floatx16 acc0[FN0][FM0];
#pragma unroll
    for (int a = 0; a < FN0; ++a)
#pragma unroll
      for (int b = 0; b < FM0; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc0[a][b][r] = 0.f;

    xl.load(0, p.cg);
    xl.store(Xs);
    if constexpr (WMODE == 1) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's weight loads have landed
    __syncthreads();
    for (int kt = 0; kt < nk0; ++kt) {
      const int buf = kt & 1;
      const bool more = kt + 1 < nk0;
      if (more) xl.load(kt + 1, p.cg);
      const half_t* xs = Xs + buf * BM * BK;
      const half_t* ws = W0s + kt * N0T * BK;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        half8 xf[FM0], wf[FN0];
        const int chunk = ks * 2 + g;
#pragma unroll
        for (int b = 0; b < FM0; ++b) xf[b] = *(const half8*)(xs + lds_chunk_offset<BK>(wm0 * WTM0 + b * 32 + l32, chunk));
#pragma unroll
        for (int a = 0; a < FN0; ++a) {
          if constexpr (WMODE == 1) wf[a] = kn_frag_read<N0T>(W0s, w0off[a], kt * BK + ks * 16);
          else wf[a] = *(const half8*)(ws + lds_chunk_offset<BK>(wn0 * WTN0 + a * 32 + l32, chunk));
        }
#pragma unroll
        for (int a = 0; a < FN0; ++a)
#pragma unroll
          for (int b = 0; b < FM0; ++b) acc0[a][b] = mfma_32x32x16(wf[a], xf[b], acc0[a][b]);
      }
      if (more) xl.store(Xs + (buf ^ 1) * BM * BK);
      __syncthreads();
    }

    // ---- epilogue0 -> FP16 D0 tile in LDS, in the operand layout of op1 ----------------------
    // (the last barrier of the loop above orders this after every read of the previous tile's D0s)
    {
      const EpilogueArgs ep{p.b0, p.b0_on, p.N0, p.alpha0, p.beta0, p.act0};
      auto d0_to_lds = [&](auto slow) {
#pragma unroll
        for (int a = 0; a < FN0; ++a)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int col = wn0 * WTN0 + a * 32 + q * 8 + g * 4;
#pragma unroll
            for (int b = 0; b < FM0; ++b) {
              half4 o = epilogue_quad<decltype(slow)::value>(acc0[a][b], q, col, ep);
              const half4 z = {0, 0, 0, 0};
              if (col >= p.N0) o = z;
              const int row = wm0 * WTM0 + b * 32 + l32;
              *(half4*)(D0s + (col / KB1) * BM * KB1 + lds_chunk_offset<KB1>(row, (col % KB1) / 8) + (col & 4)) = o;
            }
          }
      };
      if (p.act0 > ACT_RELU) d0_to_lds(std::true_type{});
      else d0_to_lds(std::false_type{});
    }
    __syncthreads();

    // ---- op1: both operands from LDS -----------------------------------------------------------
    floatx16 acc1[FN1][FM1];
#pragma unroll
    for (int a = 0; a < FN1; ++a)
#pragma unroll
      for (int b = 0; b < FM1; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc1[a][b][r] = 0.f;
#pragma unroll
    for (int kt1 = 0; kt1 < NKT1; ++kt1) {
      const half_t* xs = D0s + kt1 * BM * KB1;
      const half_t* ws = W1s + kt1 * N1T * KB1;
#pragma unroll
      for (int ks = 0; ks < KB1 / 16; ++ks) {
        half8 xf[FM1], wf[FN1];
        const int chunk = ks * 2 + g;
#pragma unroll
        for (int b = 0; b < FM1; ++b) xf[b] = *(const half8*)(xs + lds_chunk_offset<KB1>(wm1 * WTM1 + b * 32 + l32, chunk));
#pragma unroll
        for (int a = 0; a < FN1; ++a) {
          if constexpr (WMODE == 1) wf[a] = kn_frag_read<N1T>(W1s, w1off[a], kt1 * KB1 + ks * 16);
          else wf[a] = *(const half8*)(ws + lds_chunk_offset<KB1>(wn1 * WTN1 + a * 32 + l32, chunk));
        }
#pragma unroll
        for (int a = 0; a < FN1; ++a)
#pragma unroll
          for (int b = 0; b < FM1; ++b) acc1[a][b] = mfma_32x32x16(wf[a], xf[b], acc1[a][b]);
      }
    }
    b2b_tile_out_2d<BM, N1T, WTM1, WTN1, NT, RES>(Xs, acc1, p, m0, wm1, wn1, tid);
  }
}

struct B2bInstance {
  const char* name;
  int mode;  // 0 RF-resident, 1 LDS-resident
  int bm, bk, waves_m, waves_n, n0t, n1t, xmode, wmode, nthreads;
  int stages;
  int (*lds_bytes)(int K0);
  hipError_t (*launch)(const B2bParams&, int grid, int lds_bytes, hipStream_t);
  // instances whose legality / LDS need depends on the geometry (b2b_halo_kernel.hpp); null otherwise
  bool (*dyn_supports)(const B2bParams&);
  int (*dyn_lds_bytes)(const B2bParams&);
  bool residual;  // has the variant whose last epilogue adds a full matrix C (B2bParams::res)
  // Relative time per unit of tile work of this kernel family on the convolution pairs of Section 4.1.2, as measured
  // (0 = 1.0: the weights-resident kernels); read by the built-in pick rule only, bolt_tune measures.
  float prior;
};

template <typename KernT>
hipError_t b2b_launch_common(KernT kern, LdsOptIn& opt_in, const B2bParams& p, int grid, int nthreads, int lds_bytes,
                             hipStream_t stream) {
  if (hipError_t e = opt_in.ensure((const void*)kern, 160 * 1024); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(nthreads), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int BM, int BK, int NWAVES, int N0T, int N1T, int XMODE, int WMODE>
hipError_t launch_b2b_rf(const B2bParams& p, int grid, int lds_bytes, hipStream_t stream) {
  static LdsOptIn opt_in[2];
  if (p.res)  // the residual epilogue is a kernel of its own (see b2b_tile_out_2d)
    return b2b_launch_common(b2b_rf_kernel<BM, BK, NWAVES, N0T, N1T, XMODE, WMODE, true>, opt_in[1], p, grid, 64 * NWAVES,
                             lds_bytes, stream);
  return b2b_launch_common(b2b_rf_kernel<BM, BK, NWAVES, N0T, N1T, XMODE, WMODE, false>, opt_in[0], p, grid, 64 * NWAVES,
                           lds_bytes, stream);
}

template <int BM, int BK, int WM0, int WN0, int WM1, int WN1, int N0T, int N1T, int XMODE, int WMODE>
hipError_t launch_b2b_lds(const B2bParams& p, int grid, int lds_bytes, hipStream_t stream) {
  static LdsOptIn opt_in[2];
  if (p.res)
    return b2b_launch_common(b2b_lds_kernel<BM, BK, WM0, WN0, WM1, WN1, N0T, N1T, XMODE, WMODE, true>, opt_in[1], p, grid,
                             64 * WM0 * WN0, lds_bytes, stream);
  return b2b_launch_common(b2b_lds_kernel<BM, BK, WM0, WN0, WM1, WN1, N0T, N1T, XMODE, WMODE, false>, opt_in[0], p, grid,
                           64 * WM0 * WN0, lds_bytes, stream);
}

#define BOLT_B2B_RF_INSTANCE(BM, BK, NW, N0T, N1T, XMODE, WMODE)                                         \
  {                                                                                                      \
    "rf_" #BM "x" #BK "_w" #NW "_n" #N0T "_" #N1T, 0, BM, BK, NW, 1, N0T, N1T, XMODE, WMODE, 64 * NW, 2,  \
        &bolt::B2bRfTraits<BM, BK, NW, N0T, N1T, XMODE, WMODE>::lds_bytes,                                \
        &bolt::launch_b2b_rf<BM, BK, NW, N0T, N1T, XMODE, WMODE>, nullptr, nullptr, true                  \
  }
#define BOLT_B2B_LDS_INSTANCE(BM, BK, WM0, WN0, WM1, WN1, N0T, N1T, XMODE, WMODE)                          \
  {                                                                                                      \
    "lds_" #BM "x" #BK "_w" #WM0 "x" #WN0 "_" #WM1 "x" #WN1 "_n" #N0T "_" #N1T, 1, BM, BK, WM0, WN0, N0T, \
        N1T, XMODE, WMODE, 64 * WM0 * WN0, 2,                                                            \
        &bolt::B2bLdsTraits<BM, BK, WM0, WN0, WM1, WN1, N0T, N1T, XMODE, WMODE>::lds_bytes,               \
        &bolt::launch_b2b_lds<BM, BK, WM0, WN0, WM1, WN1, N0T, N1T, XMODE, WMODE>, nullptr, nullptr, true \
  }

}  // namespace bolt
