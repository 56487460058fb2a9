// Persistent fusion of a chain of three ops (Section 3.1.1: the two-op pipeline "duplicated" once
// more): op0 is a GEMM or an implicit-GEMM convolution, op1 and op2 are GEMMs / 1x1 convolutions
// whose whole weight matrices stay in LDS.  One workgroup owns BM rows and all N0, N1 and N2
// columns (threadblock residence for every op of the chain); D0 and D1 never leave the registers
// of the wave that computed them (RF-resident fusion): after each epilogue the FP16 results are
// re-used as the activation fragments of the next MFMA chain, exactly as in b2b_dma_kernel.hpp.
// K-contiguous weights only (conv KRSC, GEMM B as [N][K]).
#pragma once
#include "b2b_dma_kernel.hpp"
#include "b2b_halo_kernel.hpp"

namespace bolt {

template <int BM, int BK, int NW, int N0T, int N1T, int N2T, int XMODE, int NS>
struct B2bChainTraits {
  static constexpr int WTM = BM / NW, FM = WTM / 32;
  static constexpr int STAGE_HALVES = (BM + N0T) * BK;
  static constexpr int PIPE_BYTES = (NS * STAGE_HALVES + N0T * N1T + N1T * N2T) * 2;
  static constexpr int CTILE_BYTES = BM * N2T * 2;
  static constexpr int LDS_BYTES = PIPE_BYTES > CTILE_BYTES ? PIPE_BYTES : CTILE_BYTES;
  static_assert(WTM % 32 == 0 && N0T % 32 == 0 && N1T % 32 == 0 && N2T % 32 == 0, "tile shape");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  static int lds_bytes(int) { return LDS_BYTES; }
};

// RES: the last epilogue adds gamma * C, C a full M x N2 matrix (Eq. 1 with C0 a matrix, taken by the op whose output
// is stored); its tile comes through LDS as in b2b_tile_out.
// WKN: GEMM chain whose three weight matrices are row-major [K][N] (see DmaKnTileLoader / kn_matrix_to_lds).
template <int BM, int BK, int NW, int N0T, int N1T, int N2T, int XMODE, int NS, bool RES = false, bool WKN = false>
__global__ __launch_bounds__(64 * NW) void b2b_chain_kernel(const B2bParams p) {
  using T = B2bChainTraits<BM, BK, NW, N0T, N1T, N2T, XMODE, NS>;
  constexpr int FM = T::FM;

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* W1s = lds + NS * T::STAGE_HALVES;  // [N0T / KB1][N1T * KB1]
  half_t* W2s = W1s + N0T * N1T;             // [N1T / KB2][N2T * KB2]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, l32 = lane & 31;
  const int m0 = blockIdx.x * BM;

  // resident weights first: the oldest loads, covered by the main loop's final wait
  b2b_issue_weights<N1T, N0T, NW, WKN>(p.W1, p.ldw1, p.N1, p.N0, W1s, p.cg, wave, lane);
  b2b_issue_weights<N2T, N1T, NW, WKN>(p.W2, p.ldw2, p.N2, p.N1, W2s, p.cg, wave, lane);

  floatx16 acc0[N0T / 32][FM];
  b2b_dma_op0<BM, BK, NW, N0T, XMODE, NS, WKN>(p, lds, m0, wave, lane, acc0);

  half8 d0[N0T / 16][FM];
  b2b_make_d<N0T / 32, FM>(EpilogueArgs{p.b0, p.b0_on, p.N0, p.alpha0, p.beta0, p.act0}, acc0, d0, g);
  floatx16 acc1[N1T / 32][FM];
  b2b_rf_gemm<N0T, N1T, FM, WKN>(W1s, d0, acc1, l32, g);

  half8 d1[N1T / 16][FM];
  b2b_make_d<N1T / 32, FM>(EpilogueArgs{p.b1, p.b1_on, p.N1, p.alpha1, p.beta1, p.act1}, acc1, d1, g);
  floatx16 acc2[N2T / 32][FM];
  b2b_rf_gemm<N1T, N2T, FM, WKN>(W2s, d1, acc2, l32, g);

  const EpilogueArgs ep{p.b2, p.b2_on, p.N2, p.alpha2, p.beta2, p.act2, RES ? p.gamma : 0.f};
  b2b_tile_out<BM, NW, N2T, RES>(lds, acc2, ep, p.Y, p.ldy, p.M, m0, wave, tid, p.res, p.ldr);
}

// The same chain with a stride-1 "same" convolution as op0 on the halo main loop of conv_halo_kernel.hpp (the
// activation halo goes to LDS once per 64-channel chunk instead of one gathered k-tile per filter tap), as
// b2b_halo_kernel.hpp does for the fused pair.  W1 and W2 sit behind the halo buffers and the W0 stages.
template <int BM, int NW, int N0T, int N1T, int N2T, int NS, int XI>
struct B2bChainHaloTraits {
  using Halo = ConvHaloTraits<BM, N0T, NW, 1, NS, XI, 1>;
  static constexpr int WTM = BM / NW, FM = WTM / 32;
  static_assert(WTM % 32 == 0 && N0T % 32 == 0 && N1T % 32 == 0 && N2T % 32 == 0, "tile shape");
  static bool supports(const B2bParams& p) { return Halo::supports(B2bHaloTraits<BM, NW, N0T, N1T, NS, XI>::as_fprop(p)); }
  static int lds_bytes(const B2bParams& p) {
    const int pipe = (Halo::group_halves(p.cg) + N0T * N1T + N1T * N2T) * 2;
    const int ctile = BM * N2T * 2;
    return pipe > ctile ? pipe : ctile;
  }
};

template <int BM, int NW, int N0T, int N1T, int N2T, int NS, int XI, bool RES = false>
__global__ __launch_bounds__(64 * NW, 2) void b2b_chain_halo_kernel(const B2bParams p) {
  using T = B2bChainHaloTraits<BM, NW, N0T, N1T, N2T, NS, XI>;
  constexpr int FM = T::FM;

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* W1s = lds + T::Halo::group_halves(p.cg);  // [N0T / KB1][N1T * KB1]
  half_t* W2s = W1s + N0T * N1T;                    // [N1T / KB2][N2T * KB2]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, l32 = lane & 31;
  const int m0 = blockIdx.x * BM;

  // resident weights first: the oldest loads, the main loop's first wait covers them
  b2b_issue_weights<N1T, N0T, NW>(p.W1, p.ldw1, p.N1, p.N0, W1s, p.cg, wave, lane);
  b2b_issue_weights<N2T, N1T, NW>(p.W2, p.ldw2, p.N2, p.N1, W2s, p.cg, wave, lane);

  floatx16 acc0[N0T / 32][FM];
  {
    const HaloArgs h{p.X, p.W0, p.N0, p.M, p.K0, p.ldw0, p.cg, m0};
    conv_halo_mainloop<BM, N0T, NW, 1, NS, XI, 1>(h, lds, acc0);
  }

  half8 d0[N0T / 16][FM];
  b2b_make_d<N0T / 32, FM>(EpilogueArgs{p.b0, p.b0_on, p.N0, p.alpha0, p.beta0, p.act0}, acc0, d0, g);
  floatx16 acc1[N1T / 32][FM];
  b2b_rf_gemm<N0T, N1T, FM>(W1s, d0, acc1, l32, g);

  half8 d1[N1T / 16][FM];
  b2b_make_d<N1T / 32, FM>(EpilogueArgs{p.b1, p.b1_on, p.N1, p.alpha1, p.beta1, p.act1}, acc1, d1, g);
  floatx16 acc2[N2T / 32][FM];
  b2b_rf_gemm<N1T, N2T, FM>(W2s, d1, acc2, l32, g);

  const EpilogueArgs ep{p.b2, p.b2_on, p.N2, p.alpha2, p.beta2, p.act2, RES ? p.gamma : 0.f};
  b2b_tile_out<BM, NW, N2T, RES>(lds, acc2, ep, p.Y, p.ldy, p.M, m0, wave, tid, p.res, p.ldr);
}

struct ChainInstance {
  const char* name;
  int bm, bk, waves, n0t, n1t, n2t, xmode, stages, lds_bytes;
  hipError_t (*launch)(const B2bParams&, hipStream_t);
  // instances whose legality / LDS need depends on the geometry (the halo chains); null otherwise
  bool (*dyn_supports)(const B2bParams&);
  int (*dyn_lds_bytes)(const B2bParams&);
  int wmode;  // 0: weights stored [N][K] (reduction index contiguous), 1: row-major [K][N] (GEMM chains)
};

template <int BM, int BK, int NW, int N0T, int N1T, int N2T, int XMODE, int NS, bool WKN = false>
hipError_t launch_b2b_chain(const B2bParams& p, hipStream_t stream) {
  static LdsOptIn opt_in[2];
  constexpr int kLds = B2bChainTraits<BM, BK, NW, N0T, N1T, N2T, XMODE, NS>::LDS_BYTES;
  if (p.res)  // the residual epilogue is a kernel of its own (see b2b_tile_out)
    return b2b_launch_common(b2b_chain_kernel<BM, BK, NW, N0T, N1T, N2T, XMODE, NS, true, WKN>, opt_in[1], p, p.tiles_m,
                             64 * NW, kLds, stream);
  return b2b_launch_common(b2b_chain_kernel<BM, BK, NW, N0T, N1T, N2T, XMODE, NS, false, WKN>, opt_in[0], p, p.tiles_m,
                           64 * NW, kLds, stream);
}

template <int BM, int NW, int N0T, int N1T, int N2T, int NS, int XI>
hipError_t launch_b2b_chain_halo(const B2bParams& p, hipStream_t stream) {
  static LdsOptIn opt_in[2];
  const int lds = B2bChainHaloTraits<BM, NW, N0T, N1T, N2T, NS, XI>::lds_bytes(p);
  if (p.res)
    return b2b_launch_common(b2b_chain_halo_kernel<BM, NW, N0T, N1T, N2T, NS, XI, true>, opt_in[1], p, p.tiles_m, 64 * NW,
                             lds, stream);
  return b2b_launch_common(b2b_chain_halo_kernel<BM, NW, N0T, N1T, N2T, NS, XI, false>, opt_in[0], p, p.tiles_m, 64 * NW,
                           lds, stream);
}

#define BOLT_B2B_CHAIN_HALO_INSTANCE(BM, NW, N0T, N1T, N2T, NS, XI)                                             \
  {                                                                                                            \
    "chainhalo_" #BM "_w" #NW "_n" #N0T "_" #N1T "_" #N2T "_s" #NS "_x" #XI, BM, 64, NW, N0T, N1T, N2T, 1, NS, 0, \
        &bolt::launch_b2b_chain_halo<BM, NW, N0T, N1T, N2T, NS, XI>,                                             \
        &bolt::B2bChainHaloTraits<BM, NW, N0T, N1T, N2T, NS, XI>::supports,                                      \
        &bolt::B2bChainHaloTraits<BM, NW, N0T, N1T, N2T, NS, XI>::lds_bytes                                      \
  }

#define BOLT_B2B_CHAIN_INSTANCE(BM, BK, NW, N0T, N1T, N2T, NS, XMODE)                                          \
  {                                                                                                            \
    "chain_" #BM "x" #BK "_w" #NW "_n" #N0T "_" #N1T "_" #N2T "_s" #NS, BM, BK, NW, N0T, N1T, N2T, XMODE, NS,     \
        bolt::B2bChainTraits<BM, BK, NW, N0T, N1T, N2T, XMODE, NS>::LDS_BYTES,                                   \
        &bolt::launch_b2b_chain<BM, BK, NW, N0T, N1T, N2T, XMODE, NS>, nullptr, nullptr                          \
  }

// The GEMM chain with row-major weights.
#define BOLT_B2B_CHAIN_KN_INSTANCE(BM, BK, NW, N0T, N1T, N2T, NS)                                              \
  {                                                                                                            \
    "chainkn_" #BM "x" #BK "_w" #NW "_n" #N0T "_" #N1T "_" #N2T "_s" #NS, BM, BK, NW, N0T, N1T, N2T, 0, NS,       \
        bolt::B2bChainTraits<BM, BK, NW, N0T, N1T, N2T, 0, NS>::LDS_BYTES,                                       \
        &bolt::launch_b2b_chain<BM, BK, NW, N0T, N1T, N2T, 0, NS, true>, nullptr, nullptr, 1                     \
  }

}  // namespace bolt
