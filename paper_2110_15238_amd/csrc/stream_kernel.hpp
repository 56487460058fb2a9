// Persistent, weights-resident streaming kernel for the back-to-back GEMM fusion of Section 3.1.1
// with row-major weights ([K][N], transposed on their way into LDS).
//
//   D0 = act0(alpha0 * X . W0 + beta0 * b0)          (Eq. 1)
//   D1 = act1(alpha1 * fp16(D0) . W1 + beta1 * b1)   (Eq. 2)
//
// A workgroup keeps W0 and W1 in LDS for its whole life and walks over BM-row tiles of X,
// persistently (grid = number of compute units x residency).  Threadblock residence: the tile
// spans all N0 (and N1) columns; RF-resident fusion: waves split the tile along M only, the
// FP16-rounded D0 accumulators are re-used in registers as the operand of the second MFMA chain.
//
// What differs from the paper's CUTLASS design, for this chip:
//   * both weight matrices are resident in the 160 KB LDS instead of being re-streamed per tile;
//   * activation tiles stream global -> LDS directly (buffer_load ... lds), NS k-tiles deep, and
//     the stream does NOT drain at row-tile boundaries: the loads of the next row tile are in
//     flight while the epilogue / second GEMM of the current one runs;
//   * the MFMA computes the transposed product so that a lane's accumulators are runs of D0
//     columns of one row (see b2b_kernel.hpp), which is what makes the register hand-over cheap.
#pragma once
#include "b2b_kernel.hpp"
#include "fprop_dma_kernel.hpp"

namespace bolt {

// s_waitcnt vmcnt(n) for a wave-uniform run-time n in [0, 63], rounded DOWN to a multiple of 4
// above 8 (waiting for a few more operations than necessary is always safe).
__device__ __forceinline__ void wait_vmcnt_upto(int n) {
#define BOLT_VM_CASE(v) \
  case v: __builtin_amdgcn_s_waitcnt(((v) & 0xF) | (((v) >> 4) << 14) | 0x0F70); break;
  if (n > 63) n = 63;
  if (n > 8) n &= ~3;
  switch (n) {
    BOLT_VM_CASE(0) BOLT_VM_CASE(1) BOLT_VM_CASE(2) BOLT_VM_CASE(3) BOLT_VM_CASE(4) BOLT_VM_CASE(5) BOLT_VM_CASE(6)
    BOLT_VM_CASE(7) BOLT_VM_CASE(8) BOLT_VM_CASE(12) BOLT_VM_CASE(16) BOLT_VM_CASE(20) BOLT_VM_CASE(24)
    BOLT_VM_CASE(28) BOLT_VM_CASE(32) BOLT_VM_CASE(36) BOLT_VM_CASE(40) BOLT_VM_CASE(44) BOLT_VM_CASE(48)
    BOLT_VM_CASE(52) BOLT_VM_CASE(56) BOLT_VM_CASE(60)
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;
  }
#undef BOLT_VM_CASE
}

template <int BM, int BK, int NW, int N0T, int N1T, int NS>
struct StreamTraits {
  static constexpr int NT = 64 * NW;
  static constexpr int WTM = BM / NW, FM = WTM / 32;
  static constexpr int FN0 = N0T / 32, FN1 = N1T / 32;
  static constexpr int NC1 = FN1 < 4 ? FN1 : 4;
  static constexpr int KB1 = N0T < 64 ? N0T : 64;
  static constexpr int NKT1 = N0T / KB1;
  static constexpr int STORES = FM * FN1 * 4;  // store instructions per wave per row tile
  static_assert(WTM % 32 == 0 && N0T % 32 == 0 && N1T % 32 == 0 && N1T > 0, "tile shape");
  static_assert(FN1 % NC1 == 0, "op1 column chunks");
  static_assert(NS >= 2 && NS <= 8, "stages");
  static int lds_bytes(int K0) {
    const int nk0 = (K0 + BK - 1) / BK;
    return (nk0 * N0T * BK + N0T * N1T + NS * BM * BK) * 2;
  }
};

template <int BM, int BK, int NW, int N0T, int N1T, int NS>
__global__ __launch_bounds__(64 * NW) void stream_kernel(const B2bParams p) {
  using T = StreamTraits<BM, BK, NW, N0T, N1T, NS>;
  constexpr int NT = T::NT, WTM = T::WTM, FM = T::FM, FN0 = T::FN0, FN1 = T::FN1, NC1 = T::NC1;
  constexpr int KB1 = T::KB1, NKT1 = T::NKT1, KS = BK / 16;
  using XL = DmaTileLoader<BM, BK, NW, 0>;
  constexpr int L = XL::NI;
  static_assert(KS % 2 == 0, "fragment double buffering");

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  const int nk0 = (p.K0 + BK - 1) / BK;
  half_t* W0s = lds;                      // [nk0][N0T*BK]
  half_t* W1s = W0s + nk0 * N0T * BK;     // [NKT1][N1T*KB1]
  half_t* Xs = W1s + N0T * N1T;           // [NS][BM*BK]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, l32 = lane & 31;
  const int G = gridDim.x;
  const int n_mine = (int)blockIdx.x < p.tiles_m ? (p.tiles_m - (int)blockIdx.x + G - 1) / G : 0;
  if (n_mine == 0) return;
  const int S = n_mine * nk0;  // length of this workgroup's stream of k-tiles

  // ---- weights -> LDS, once ----------------------------------------------------------------
  {
    WTileLoader<N0T, BK, NT, 1> wl;
    wl.init(p.W0, p.ldw0, p.N0, p.K0, 0, tid);
    for (int kt = 0; kt < nk0; ++kt) {
      wl.load(kt);
      wl.store(W0s + kt * N0T * BK);
    }
  }
  {
    WTileLoader<N1T, KB1, NT, 1> wl;
    wl.init(p.W1, p.ldw1, p.N1, p.N0, 0, tid);
#pragma unroll
    for (int kt = 0; kt < NKT1; ++kt) {
      wl.load(kt);
      wl.store(W1s + kt * N1T * KB1);
    }
  }

  // ---- the load side of the stream ---------------------------------------------------------------
  XL xl;
  int l_tile = blockIdx.x, l_k = 0, fill = 0, issued = 0;
  auto init_loader = [&](int tile) {
    const int m0 = tile * BM;
    const int64_t rem = ((int64_t)(p.M - m0 - 1) * p.ldx + p.K0) * 2;
    xl.init(p.X + (int64_t)m0 * p.ldx, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff), p.ldx, p.M - m0, p.K0, p.cg, m0, 0,
            wave, lane);
  };
  auto issue_next = [&]() {  // issue stream item `issued` into stage `fill`
    xl.issue(l_k, Xs + fill * BM * BK, p.cg);
    fill = fill + 1 == NS ? 0 : fill + 1;
    ++issued;
    if (++l_k == nk0) {
      l_k = 0;
      l_tile += G;
      if (issued < S) init_loader(l_tile);
    }
  };
  init_loader(l_tile);
#pragma unroll
  for (int s = 0; s < NS; ++s)
    if (s < S) issue_next();
  // everything issued before stream item 1 (the weights, item 0) must have landed
  wait_vmcnt_upto((S < NS ? S - 1 : NS - 1) * L);
  barrier_after_lds_writes();

  half8 xf[2][FM], wf[2][FN0];
  auto read_frags = [&](int stage, int kt, int ks, half8 (&x)[FM], half8 (&w)[FN0]) {
    const half_t* xs = Xs + stage * BM * BK;
    const half_t* ws = W0s + kt * N0T * BK;
    const int chunk = ks * 2 + g;
#pragma unroll
    for (int b = 0; b < FM; ++b) x[b] = *(const half8*)(xs + dma_chunk_offset<BK>(wave * WTM + b * 32 + l32, chunk));
#pragma unroll
    for (int a = 0; a < FN0; ++a) w[a] = *(const half8*)(ws + lds_chunk_offset<BK>(a * 32 + l32, chunk));
  };
  read_frags(0, 0, 0, xf[0], wf[0]);

  int stage = 0, s = 0;
  // bit i of hist: stream item s-1-i was the last k-tile of a row tile whose epilogue issued exactly
  // T::STORES store instructions in this wave.  That is only certain when no store can be skipped:
  // every row of the wave's slice and every column of the compiled width is valid.  Otherwise the
  // stores are not counted, which only makes the wait below longer.
  unsigned hist = 0;
  const bool all_cols = p.N1 == N1T;
  for (int j = 0; j < n_mine; ++j) {
    const int m0 = ((int)blockIdx.x + j * G) * BM;
    floatx16 acc0[FN0][FM];
#pragma unroll
    for (int a = 0; a < FN0; ++a)
#pragma unroll
      for (int b = 0; b < FM; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc0[a][b][r] = 0.f;

    for (int kt = 0; kt < nk0; ++kt) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (ks + 1 < KS) {
          read_frags(stage, kt, ks + 1, xf[(ks + 1) & 1], wf[(ks + 1) & 1]);
        } else {
          // end of stream item s: wait until item s+1 has landed.  Operations issued after its loads
          // may stay in flight: the loads of items s+2 .. s+NS-1 and the stores of the epilogues that
          // ran since (vector memory operations retire in issue order).
          __builtin_amdgcn_sched_barrier(0);
          const int newer = S - 2 - s < NS - 2 ? (S - 2 - s < 0 ? 0 : S - 2 - s) : NS - 2;
          const int n_epi = __builtin_popcount(hist & ((1u << (NS - 1)) - 1));
          wait_vmcnt_upto(newer * L + n_epi * T::STORES);
          __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's reads of item s are complete
          raw_barrier();
          if (issued < S) issue_next();  // refills the stage item s was read from
          hist = (hist << 1) | ((kt + 1 == nk0 && all_cols && m0 + (wave + 1) * WTM <= p.M) ? 1u : 0u);
          stage = stage + 1 == NS ? 0 : stage + 1;
          ++s;
          read_frags(stage, kt + 1 == nk0 ? 0 : kt + 1, 0, xf[0], wf[0]);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int a = 0; a < FN0; ++a)
#pragma unroll
          for (int b = 0; b < FM; ++b) acc0[a][b] = mfma_32x32x16(wf[ks & 1][a], xf[ks & 1][b], acc0[a][b]);
      }
    }

    const int mrow = m0 + wave * WTM + l32;
    // ---- epilogue0 in registers: accumulators -> FP16 B-operand fragments of op1 ------------
    half8 d0[FN0 * 2][FM];
    b2b_make_d0<FN0, FM>(p, acc0, d0, g);
    // ---- op1: W1 fragments from LDS with the matching reduction-index permutation ----------
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
        const int kbase = t * 16;
        const int kt1 = kbase / KB1;
        const int chunk = (kbase % KB1) / 8;
        const half_t* ws = W1s + kt1 * N1T * KB1;
#pragma unroll
        for (int a = 0; a < NC1; ++a) {
          const int row = (c1 * NC1 + a) * 32 + l32;
          const half4 lo = *(const half4*)(ws + lds_chunk_offset<KB1>(row, chunk) + g * 4);
          const half4 hi = *(const half4*)(ws + lds_chunk_offset<KB1>(row, chunk + 1) + g * 4);
          const half8 w1 = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
          for (int b = 0; b < FM; ++b) acc1[a][b] = mfma_32x32x16(w1, d0[t][b], acc1[a][b]);
        }
      }
      b2b_store_tile<NC1, FM>(p, acc1, mrow, c1 * NC1 * 32 + g * 4);
    }
  }
}

template <int BM, int BK, int NW, int N0T, int N1T, int NS>
hipError_t launch_stream(const B2bParams& p, int grid, int lds_bytes, hipStream_t stream) {
  static LdsOptIn opt_in;
  return b2b_launch_common(stream_kernel<BM, BK, NW, N0T, N1T, NS>, opt_in, p, grid, 64 * NW, lds_bytes, stream);
}

// mode 0 = RF-resident fusion; GEMM rows (x mode 0), row-major weights (w mode 1)
#define BOLT_STREAM_INSTANCE(BM, BK, NW, N0T, N1T, NS)                                                  \
  {                                                                                                     \
    "stream_" #BM "x" #BK "_w" #NW "_n" #N0T "_" #N1T "_s" #NS, 0, BM, BK, NW, 1, N0T, N1T, 0, 1, 64 * NW, \
        NS, &bolt::StreamTraits<BM, BK, NW, N0T, N1T, NS>::lds_bytes,                                   \
        &bolt::launch_stream<BM, BK, NW, N0T, N1T, NS>                                                  \
  }

}  // namespace bolt
