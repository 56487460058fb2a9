// Back-to-back fusion on top of the multi-stage direct-to-LDS main loop (Section 3.1.1,
// RF-resident fusion).  One workgroup owns BM rows and all N0 and N1 columns (threadblock
// residence); waves split the tile along M only, so the accumulators of op0, after the epilogue
// of op0 and rounding to FP16, are re-used in registers as the activation operand of op1.
//   op0: X (GEMM rows or implicit im2col) and W0 k-tiles stream through NS LDS stages;
//   op1: W1 (all of it, [N1][N0] K-contiguous) is fetched to LDS once, at kernel start, so the
//        second GEMM runs entirely out of registers and LDS;
//   epilogue: D1 tile -> FP16 -> LDS -> 16-byte coalesced row stores.
// Unlike the weights-resident kernels of b2b_kernel.hpp this kernel is not persistent: 2 workgroups fit on a compute unit and
// cover each other's prologue / epilogue.  Weights K-contiguous (conv KRSC, GEMM B as [N][K]) or, for GEMM pairs, row-major (WKN).
#pragma once
#include "b2b_kernel.hpp"
#include "fprop_dma_kernel.hpp"

namespace bolt {

template <int BM, int BK, int NW, int N0T, int N1T, int XMODE, int NS>
struct B2bDmaTraits {
  static constexpr int NT = 64 * NW;
  static constexpr int WTM = BM / NW, FM = WTM / 32;
  static constexpr int FN0 = N0T / 32, FN1 = N1T / 32;
  static constexpr int KB1 = N0T < 64 ? N0T : 64, NKT1 = N0T / KB1;
  static constexpr int STAGE_HALVES = (BM + N0T) * BK;
  static constexpr int PIPE_BYTES = (NS * STAGE_HALVES + N0T * N1T) * 2;
  static constexpr int CTILE_BYTES = BM * N1T * 2;
  static constexpr int LDS_BYTES = PIPE_BYTES > CTILE_BYTES ? PIPE_BYTES : CTILE_BYTES;
  static constexpr int CPR = N1T / 8;
  static constexpr int ROWS_PER_PASS = NT / CPR;
  static_assert(WTM % 32 == 0 && N0T % 32 == 0 && N1T % 32 == 0, "tile shape");
  static_assert(NT % CPR == 0 && BM % ROWS_PER_PASS == 0, "C tile store mapping");
  // waves per SIMD the register allocation must leave room for: as many workgroups as LDS admits
  static constexpr int WGS_PER_CU = (160 * 1024) / LDS_BYTES < 1 ? 1 : (160 * 1024) / LDS_BYTES;
  static constexpr int MIN_WAVES = (WGS_PER_CU * NW + 3) / 4 > 2 ? 2 : (WGS_PER_CU * NW + 3) / 4;
  static int lds_bytes(int) { return LDS_BYTES; }
};

// ---- building blocks shared by the two-op kernel below and the three-op chain (b2b_chain_kernel.hpp) ----

// Weights of a later op, W [n_valid][k_valid] with leading dimension ld, K-contiguous: all of it goes to LDS
// once as [NKT][NOUT_T][KB] k-tiles of width KB = min(NIN_T, 64); missing rows and columns are zero-filled.
// WKN: W is row-major [k_valid][n_valid] instead and stays so in LDS, as [NIN_T][NOUT_T] (kn_matrix_to_lds).
template <int NOUT_T, int NIN_T, int NW, bool WKN = false>
__device__ __forceinline__ void b2b_issue_weights(const half_t* W, int ld, int n_valid, int k_valid, half_t* Ws,
                                                  const ConvGeom& cg, int wave, int lane) {
  if constexpr (WKN) {
    kn_matrix_to_lds<64 * NW, NOUT_T>(W, ld, k_valid, n_valid, NIN_T, Ws, wave * 64 + lane);
    return;
  }
  constexpr int KB = NIN_T < 64 ? NIN_T : 64, NKT = NIN_T / KB;
  DmaTileLoader<NOUT_T, KB, NW, 0> wl;
  const int64_t bytes = ((int64_t)(n_valid - 1) * ld + k_valid) * 2;
  wl.init(W, (unsigned)(bytes < 0x7fffffff ? bytes : 0x7fffffff), ld, n_valid, k_valid, cg, 0, 0, wave, lane);
#pragma unroll
  for (int kt = 0; kt < NKT; ++kt) wl.issue(kt, Ws + kt * NOUT_T * KB, cg);
}

// op0: acc0 = X tile (GEMM rows or implicit im2col) x W0^T over K0, NS-deep direct-to-LDS pipeline with the
// fragments double-buffered across the k-tile barrier.  On return every load this wave has issued, the
// resident weights of the later ops included, has landed (the loop's final wait is vmcnt 0).
// WKN: W0 is row-major [K0][N0]; its k-tiles go to LDS as they lie in memory and are read with the LDS
// transpose read (DmaKnTileLoader).
template <int BM, int BK, int NW, int N0T, int XMODE, int NS, bool WKN = false>
__device__ __forceinline__ void b2b_dma_op0(const B2bParams& p, half_t* lds, int m0, int wave, int lane,
                                            floatx16 (&acc0)[N0T / 32][BM / NW / 32]) {
  constexpr int WTM = BM / NW, FM = WTM / 32, FN0 = N0T / 32, STAGE = (BM + N0T) * BK, KS = BK / 16;
  using XL = DmaTileLoader<BM, BK, NW, XMODE>;
  using WL = std::conditional_t<WKN, DmaKnTileLoader<BK, N0T, NW>, DmaTileLoader<N0T, BK, NW, 0>>;
  constexpr int L = XL::NI + WL::NI;
  static_assert((NS - 1) * L < 64, "vmcnt range");
  static_assert(KS % 2 == 0, "fragment double buffering");
  const int g = lane >> 5, l32 = lane & 31;
  const int n_tiles = (p.K0 + BK - 1) / BK;
  XL xl;
  WL wl;
  if constexpr (XMODE == 0) {
    const int64_t rem = ((int64_t)(p.M - m0 - 1) * p.ldx + p.K0) * 2;
    xl.init(p.X + (int64_t)m0 * p.ldx, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff), p.ldx, p.M - m0, p.K0, p.cg, m0, 0,
            wave, lane);
  } else {
    const int64_t bytes = (int64_t)p.cg.H * p.cg.Wi * p.cg.C * 2 * (int64_t)(p.M / (p.cg.P * p.cg.Q));
    xl.init(p.X, (unsigned)bytes, 0, p.M - m0, p.K0, p.cg, m0, 0, wave, lane);
  }
  int w0off[WKN ? FN0 : 1];
  if constexpr (WKN) {
    wl.init(p.W0, (unsigned)(((p.K0 - 1) * p.ldw0 + p.N0) * 2), p.ldw0, p.N0, p.K0, wave, lane);  // (under 2 GiB: host check)
#pragma unroll
    for (int a = 0; a < FN0; ++a) w0off[a] = kn_frag_offset<N0T>(a * 32, lane);
  } else {
    const int64_t bytes = ((int64_t)(p.N0 - 1) * p.ldw0 + p.K0) * 2;
    wl.init(p.W0, (unsigned)(bytes < 0x7fffffff ? bytes : 0x7fffffff), p.ldw0, p.N0, p.K0, p.cg, 0, 0, wave, lane);
  }
#pragma unroll
  for (int a = 0; a < FN0; ++a)
#pragma unroll
    for (int b = 0; b < FM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc0[a][b][r] = 0.f;

  auto issue = [&](int kt, int stage) {
    half_t* s = lds + stage * STAGE;
    xl.issue(kt, s, p.cg);
    wl.issue(kt, s + BM * BK, p.cg);
  };
  half8 xf[2][FM], wf[2][FN0];
  auto read_frags = [&](int stage, int ks, half8 (&x)[FM], half8 (&w)[FN0]) {
    const half_t* xs = lds + stage * STAGE;
    const half_t* ws = xs + BM * BK;
    const int chunk = ks * 2 + g;
#pragma unroll
    for (int b = 0; b < FM; ++b) x[b] = *(const half8*)(xs + dma_chunk_offset<BK>(wave * WTM + b * 32 + l32, chunk));
#pragma unroll
    for (int a = 0; a < FN0; ++a) {
      if constexpr (WKN) w[a] = kn_frag_read<N0T>(ws, w0off[a], ks * 16);
      else w[a] = *(const half8*)(ws + dma_chunk_offset<BK>(a * 32 + l32, chunk));
    }
  };
#pragma unroll
  for (int s = 0; s < NS; ++s)
    if (s < n_tiles) issue(s, s);
  if (n_tiles >= NS) barrier_after_loads<(NS - 1) * L>();
  else barrier_after_loads<0>();
  read_frags(0, 0, xf[0], wf[0]);
  int stage = 0;
  for (int it = 0; it < n_tiles; ++it) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) {
        read_frags(stage, ks + 1, xf[(ks + 1) & 1], wf[(ks + 1) & 1]);
      } else {
        __builtin_amdgcn_sched_barrier(0);
        if (n_tiles - 2 - it >= NS - 2) barrier_after_reads_and_loads<(NS - 2) * L>();
        else barrier_after_reads_and_loads<0>();
        if (it + NS < n_tiles) issue(it + NS, stage);
        stage = stage + 1 == NS ? 0 : stage + 1;
        read_frags(stage, 0, xf[0], wf[0]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int a = 0; a < FN0; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b) acc0[a][b] = mfma_32x32x16(wf[ks & 1][a], xf[ks & 1][b], acc0[a][b]);
    }
  }
}

// A later op entirely out of registers and LDS: acc[NOUT_T columns] = d (FP16 fragments of the previous
// op's output, NIN_T columns) x Ws^T, Ws as b2b_issue_weights leaves it.  Step t reduces over input columns
// [16t, 16t + 16); the fragment reads apply the permutation of the reduction index that b2b_make_d documents.
// WKN: Ws holds the row-major matrix as [NIN_T][NOUT_T]; the transpose read gathers the same permuted rows.
template <int NIN_T, int NOUT_T, int FM, bool WKN = false>
__device__ __forceinline__ void b2b_rf_gemm(const half_t* Ws, const half8 (&d)[NIN_T / 16][FM],
                                            floatx16 (&acc)[NOUT_T / 32][FM], int l32, int g) {
  constexpr int KB = NIN_T < 64 ? NIN_T : 64, FNO = NOUT_T / 32;
  int woff[WKN ? FNO : 1];
  if constexpr (WKN) {
#pragma unroll
    for (int a = 0; a < FNO; ++a) woff[a] = kn_frag_offset<NOUT_T>(a * 32, g * 32 + l32, 4);
  }
#pragma unroll
  for (int a = 0; a < FNO; ++a)
#pragma unroll
    for (int b = 0; b < FM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
#pragma unroll
  for (int t = 0; t < NIN_T / 16; ++t) {
    const int kbase = t * 16;
    const half_t* ws = Ws + (kbase / KB) * NOUT_T * KB;
    const int chunk = (kbase % KB) / 8;
#pragma unroll
    for (int a = 0; a < FNO; ++a) {
      const int row = a * 32 + l32;
      half8 w;
      if constexpr (WKN) {
        w = kn_frag_read<NOUT_T>(Ws, woff[a], kbase, 8);
      } else {
        const half4 lo = *(const half4*)(ws + dma_chunk_offset<KB>(row, chunk) + g * 4);
        const half4 hi = *(const half4*)(ws + dma_chunk_offset<KB>(row, chunk + 1) + g * 4);
        w = half8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      }
#pragma unroll
      for (int b = 0; b < FM; ++b) acc[a][b] = mfma_32x32x16(w, d[t][b], acc[a][b]);
    }
  }
}

// Last epilogue: accumulators -> FP16 tile [BM][NOUT_T] in LDS (over whatever the main loop left there) ->
// 16-byte coalesced non-temporal row stores.  Every wave must be done with the LDS it overwrites.
// RES (Eq. 1's C as a full matrix): the [BM][NOUT_T] tile of `res` is first brought into the same LDS slots,
// direct-to-LDS with the row swizzle applied to which global chunk a lane fetches, and every lane reads the
// quad it is about to overwrite; ep.gamma scales it.  A compile-time switch, so the plain kernels keep
// their register allocation.
template <int BM, int NW, int NOUT_T, bool RES = false>
__device__ __forceinline__ void b2b_tile_out(half_t* lds, const floatx16 (&acc)[NOUT_T / 32][BM / NW / 32],
                                             const EpilogueArgs& ep, half_t* Y, int ldy, int M, int m0, int wave, int tid,
                                             const half_t* res = nullptr, int ldr = 0) {
  constexpr int NT = 64 * NW, WTM = BM / NW, FM = WTM / 32, FNO = NOUT_T / 32;
  constexpr int CPR = NOUT_T / 8, ROWS_PER_PASS = NT / CPR;
  static_assert(NT % CPR == 0 && BM % ROWS_PER_PASS == 0, "C tile store mapping");
  const int lane = tid & 63, g = lane >> 5, l32 = lane & 31;
  barrier_after_lds_writes();
  if constexpr (RES) {
    constexpr int RPI = 64 / CPR;  // tile rows per load instruction (1024 contiguous LDS bytes)
    static_assert(CPR <= 64 && BM % RPI == 0, "residual tile rows per load instruction");
    const int64_t rem = ((int64_t)(M - m0 - 1) * ldr + ep.N) * 2;
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(res + (int64_t)m0 * ldr, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff));
    for (int i = wave; i < BM / RPI; i += NW) {
      const int row = i * RPI + lane / CPR;
      const int c = (lane % CPR) ^ ctile_swizzle<CPR>(row);
      const bool ok = m0 + row < M && c * 8 < ep.N;
      const unsigned off = ok ? (unsigned)((row * ldr + c * 8) * 2) : kInvalidOffset;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rr, BOLT_LDS_PTR(lds + i * RPI * NOUT_T), 16, off, 0, 0, 0);
    }
    barrier_after_loads<0>();
  }
  auto tile_to_lds = [&](auto slow) {
#pragma unroll
    for (int a = 0; a < FNO; ++a)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nl = a * 32 + q * 8 + g * 4;
#pragma unroll
        for (int b = 0; b < FM; ++b) {
          const int row = wave * WTM + b * 32 + l32;
          const int at = row * NOUT_T + (((nl >> 3) ^ ctile_swizzle<CPR>(row)) << 3) + (nl & 4);
          if constexpr (RES) {
            half4* slot = (half4*)(lds + at);
            *slot = epilogue_quad_res<decltype(slow)::value>(acc[a][b], q, nl, ep, *slot);
          } else {
            // (written as one expression: naming the pointer first costs the 128-wide instances a workgroup per CU)
            *(half4*)(lds + row * NOUT_T + (((nl >> 3) ^ ctile_swizzle<CPR>(row)) << 3) + (nl & 4)) =
                epilogue_quad<decltype(slow)::value>(acc[a][b], q, nl, ep);
          }
        }
      }
  };
  if (ep.act > ACT_RELU) tile_to_lds(std::true_type{});
  else tile_to_lds(std::false_type{});
  barrier_after_lds_writes();
  const int chunk = tid % CPR, r0 = tid / CPR;
  const int n = chunk * 8;
  if (n < ep.N) {
#pragma unroll
    for (int i = 0; i < BM / ROWS_PER_PASS; ++i) {
      const int row = r0 + i * ROWS_PER_PASS;
      if (m0 + row < M) {
        const half8 v = *(const half8*)(lds + row * NOUT_T + ((chunk ^ ctile_swizzle<CPR>(row)) << 3));
        __builtin_nontemporal_store(v, (half8*)(Y + (int64_t)(m0 + row) * ldy + n));
      }
    }
  }
}

template <int BM, int BK, int NW, int N0T, int N1T, int XMODE, int NS, bool RES = false, bool WKN = false>
__global__ __launch_bounds__(64 * NW, (B2bDmaTraits<BM, BK, NW, N0T, N1T, XMODE, NS>::MIN_WAVES)) void b2b_dma_kernel(
    const B2bParams p) {
  using T = B2bDmaTraits<BM, BK, NW, N0T, N1T, XMODE, NS>;
  constexpr int FM = T::FM, FN0 = T::FN0, FN1 = T::FN1;

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* W1s = lds + NS * T::STAGE_HALVES;  // [NKT1][N1T*KB1]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, l32 = lane & 31;
  const int m0 = blockIdx.x * BM;

  // W1 first: these are the oldest loads, any later wait for an operand tile covers them
  b2b_issue_weights<N1T, N0T, NW, WKN>(p.W1, p.ldw1, p.N1, p.N0, W1s, p.cg, wave, lane);

  floatx16 acc0[FN0][FM];
  b2b_dma_op0<BM, BK, NW, N0T, XMODE, NS, WKN>(p, lds, m0, wave, lane, acc0);

  // epilogue0 in registers: accumulators -> FP16 B-operand fragments of op1 (b2b_make_d0)
  half8 d0[FN0 * 2][FM];
  b2b_make_d0<FN0, FM>(p, acc0, d0, g);

  // op1: all N1 columns accumulate in registers
  floatx16 acc1[FN1][FM];
  b2b_rf_gemm<N0T, N1T, FM, WKN>(W1s, d0, acc1, l32, g);

  // epilogue1 through LDS (over the dead stages and W1)
  const EpilogueArgs ep{p.b1, p.b1_on, p.N1, p.alpha1, p.beta1, p.act1, RES ? p.gamma : 0.f};
  b2b_tile_out<BM, NW, N1T, RES>(lds, acc1, ep, p.Y, p.ldy, p.M, m0, wave, tid, p.res, p.ldr);
}

template <int BM, int BK, int NW, int N0T, int N1T, int XMODE, int NS, bool WKN = false>
hipError_t launch_b2b_dma(const B2bParams& p, int /*grid*/, int lds_bytes, hipStream_t stream) {
  static LdsOptIn opt_in[2];
  // the residual epilogue is a kernel of its own (see b2b_tile_out)
  if (p.res)
    return b2b_launch_common(b2b_dma_kernel<BM, BK, NW, N0T, N1T, XMODE, NS, true, WKN>, opt_in[1], p, p.tiles_m, 64 * NW,
                             lds_bytes, stream);
  return b2b_launch_common(b2b_dma_kernel<BM, BK, NW, N0T, N1T, XMODE, NS, false, WKN>, opt_in[0], p, p.tiles_m, 64 * NW,
                           lds_bytes, stream);
}

// mode 0 = RF-resident fusion
#define BOLT_B2B_DMA_INSTANCE(BM, BK, NW, N0T, N1T, NS, XMODE)                                            \
  {                                                                                                       \
    "b2bdma_" #BM "x" #BK "_w" #NW "_n" #N0T "_" #N1T "_s" #NS, 0, BM, BK, NW, 1, N0T, N1T, XMODE, 0, 64 * NW, \
        NS, &bolt::B2bDmaTraits<BM, BK, NW, N0T, N1T, XMODE, NS>::lds_bytes,                                \
        &bolt::launch_b2b_dma<BM, BK, NW, N0T, N1T, XMODE, NS>, nullptr, nullptr, true, 0.5f               \
  }

// The GEMM pair with row-major weights (wmode 1) on the same kernel.
#define BOLT_B2B_DMA_KN_INSTANCE(BM, BK, NW, N0T, N1T, NS)                                                \
  {                                                                                                       \
    "b2bdmakn_" #BM "x" #BK "_w" #NW "_n" #N0T "_" #N1T "_s" #NS, 0, BM, BK, NW, 1, N0T, N1T, 0, 1, 64 * NW,  \
        NS, &bolt::B2bDmaTraits<BM, BK, NW, N0T, N1T, 0, NS>::lds_bytes,                                    \
        &bolt::launch_b2b_dma<BM, BK, NW, N0T, N1T, 0, NS, true>, nullptr, nullptr, true, 0.5f             \
  }

}  // namespace bolt
