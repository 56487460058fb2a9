// Back-to-back fusion of a stride-1 "same" convolution (e.g. 3x3 / pad 1) with a 1x1 convolution
// (Section 3.1.1, RF-resident fusion; the bottleneck pair of Section 4.1.2), on top of the halo
// main loop of conv_halo_kernel.hpp: the activation halo of the first convolution is fetched to
// LDS once per 64-channel chunk, its weights stream per filter tap, W1 is fetched once at kernel
// start, and the accumulators of op0 become the activation operand of op1 in registers exactly
// as in b2b_dma_kernel.hpp (waves split the tile along M only).
#pragma once
#include "b2b_dma_kernel.hpp"
#include "conv_halo_kernel.hpp"

namespace bolt {

template <int BM, int NW, int N0T, int N1T, int NS, int XI>
struct B2bHaloTraits {
  using Halo = ConvHaloTraits<BM, N0T, NW, 1, NS, XI, 1>;
  static constexpr int NT = 64 * NW;
  static constexpr int WTM = BM / NW, FM = WTM / 32;
  static constexpr int FN0 = N0T / 32, FN1 = N1T / 32;
  static constexpr int KB1 = N0T < 64 ? N0T : 64, NKT1 = N0T / KB1;
  static constexpr int CPR = N1T / 8;
  static constexpr int ROWS_PER_PASS = NT / CPR;
  static_assert(WTM % 32 == 0 && N0T % 32 == 0 && N1T % 32 == 0, "tile shape");
  static_assert(NT % CPR == 0 && BM % ROWS_PER_PASS == 0, "C tile store mapping");
  static FpropParams as_fprop(const B2bParams& p) {  // the view of op0 that the halo legality rules read
    FpropParams f{};
    f.M = p.M; f.N = p.N0; f.K = p.K0; f.cg = p.cg;
    return f;
  }
  static bool supports(const B2bParams& p) { return Halo::supports(as_fprop(p)); }
  static int lds_bytes(const B2bParams& p) {
    const int pipe = (Halo::group_halves(p.cg) + N0T * N1T) * 2;
    const int ctile = BM * N1T * 2;
    return pipe > ctile ? pipe : ctile;
  }
};

template <int BM, int NW, int N0T, int N1T, int NS, int XI, bool RES = false>
__global__ __launch_bounds__(64 * NW, 2) void b2b_halo_kernel(const B2bParams p) {
  using T = B2bHaloTraits<BM, NW, N0T, N1T, NS, XI>;
  constexpr int NT = T::NT, WTM = T::WTM, FM = T::FM, FN0 = T::FN0, FN1 = T::FN1;
  constexpr int KB1 = T::KB1, NKT1 = T::NKT1;

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* W1s = lds + T::Halo::group_halves(p.cg);  // [NKT1][N1T * KB1], behind the halo buffers and W0 stages

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, l32 = lane & 31;
  const int m0 = blockIdx.x * BM;

  // W1 first: these are the oldest loads, the main loop's first wait covers them
  {
    DmaTileLoader<N1T, KB1, NW, 0> w1l;
    const int64_t bytes = ((int64_t)(p.N1 - 1) * p.ldw1 + p.N0) * 2;
    w1l.init(p.W1, (unsigned)(bytes < 0x7fffffff ? bytes : 0x7fffffff), p.ldw1, p.N1, p.N0, p.cg, 0, 0, wave, lane);
#pragma unroll
    for (int kt = 0; kt < NKT1; ++kt) w1l.issue(kt, W1s + kt * N1T * KB1, p.cg);
  }

  floatx16 acc0[FN0][FM];
  {
    const HaloArgs h{p.X, p.W0, p.N0, p.M, p.K0, p.ldw0, p.cg, m0};
    conv_halo_mainloop<BM, N0T, NW, 1, NS, XI, 1>(h, lds, acc0);
  }

  // ---- epilogue0 in registers: accumulators -> FP16 B-operand fragments of op1 ----------------
  half8 d0[FN0 * 2][FM];
  b2b_make_d0<FN0, FM>(p, acc0, d0, g);

  // ---- op1: all N1 columns accumulate in registers; W1 fragments carry the matching permutation
  floatx16 acc1[FN1][FM];
  b2b_rf_gemm<N0T, N1T, FM>(W1s, d0, acc1, l32, g);

  // ---- epilogue1: registers -> FP16 D1 tile in LDS (over the dead buffers and W1) -> global -----
  const EpilogueArgs ep{p.b1, p.b1_on, p.N1, p.alpha1, p.beta1, p.act1, RES ? p.gamma : 0.f};
  b2b_tile_out<BM, NW, N1T, RES>(lds, acc1, ep, p.Y, p.ldy, p.M, m0, wave, tid, p.res, p.ldr);
}

template <int BM, int NW, int N0T, int N1T, int NS, int XI>
hipError_t launch_b2b_halo(const B2bParams& p, int /*grid*/, int lds_bytes, hipStream_t stream) {
  static LdsOptIn opt_in[2];
  if (p.res)  // the residual epilogue is a kernel of its own (see b2b_tile_out)
    return b2b_launch_common(b2b_halo_kernel<BM, NW, N0T, N1T, NS, XI, true>, opt_in[1], p, p.tiles_m, 64 * NW, lds_bytes,
                             stream);
  return b2b_launch_common(b2b_halo_kernel<BM, NW, N0T, N1T, NS, XI, false>, opt_in[0], p, p.tiles_m, 64 * NW, lds_bytes,
                           stream);
}

// The same pair with op1 taken in chunks of 64 output columns, for wide second ops (N1 = 256: the bottleneck pair
// 64 -> 256 of Section 4.1.2).  A resident W1 of 64 x 256 costs 32 KB and its accumulators 128 registers per 32 rows,
// which limits the kernel above to 128-row tiles with 32 x 64 wave tiles (every wave re-reads all of W0 per filter
// tap: LDS-bound) and two rounds of workgroups.  Here only two chunks of W1 have LDS of their own; the others land in
// the W0 stages once the main loop has retired them, each chunk's 64 accumulator columns leave through a [BM][64]
// staging tile over the dead halo buffer before the next chunk is computed, so 256-row tiles with 64 x 64 wave
// tiles fit twice on a compute unit and config 4's 392 tiles run in one round.
template <int BM, int NW, int N0T, int N1T, int NS, int XI>
struct B2bHaloChunkedTraits {
  using Halo = ConvHaloTraits<BM, N0T, NW, 1, NS, XI, 1>;
  static constexpr int NC = 64;                 // columns of op1 per chunk
  static constexpr int NCHUNK = N1T / NC;
  static constexpr int OWN = NCHUNK < 2 ? NCHUNK : 2;  // chunks with LDS of their own (fetched before the main loop)
  static constexpr int SLOT = NC * N0T;         // halves of one chunk of W1 = one W0 stage
  static constexpr int WTM = BM / NW, FM = WTM / 32, FN0 = N0T / 32;
  static_assert(N1T % NC == 0 && NCHUNK - OWN <= NS, "the late chunks of W1 re-use the W0 stages");
  static_assert(WTM % 32 == 0 && N0T % 32 == 0, "tile shape");
  static bool supports(const B2bParams& p) { return Halo::supports(B2bHaloTraits<BM, NW, N0T, N1T, NS, XI>::as_fprop(p)); }
  static int lds_bytes(const B2bParams& p) { return (Halo::group_halves(p.cg) + OWN * SLOT) * 2; }  // >= the [BM][64] staging tile
};

template <int BM, int NW, int N0T, int N1T, int NS, int XI, bool RES = false>
__global__ __launch_bounds__(64 * NW, 2) void b2b_halo_chunked_kernel(const B2bParams p) {
  using T = B2bHaloChunkedTraits<BM, NW, N0T, N1T, NS, XI>;
  constexpr int FM = T::FM, FN0 = T::FN0, NC = T::NC, NCHUNK = T::NCHUNK, OWN = T::OWN, SLOT = T::SLOT;

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* own = lds + T::Halo::group_halves(p.cg);            // chunks 0 .. OWN-1 of W1
  half_t* stages = own - NS * N0T * 64;                        // the W0 stages of the main loop: chunks OWN .. of W1

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, l32 = lane & 31;
  const int m0 = blockIdx.x * BM;
  auto issue_chunk = [&](int c, half_t* dst) {  // rows [c * NC, ...) of W1; rows past N1 are zero-filled
    const int left = p.N1 - c * NC;
    b2b_issue_weights<NC, N0T, NW>(p.W1 + (int64_t)c * NC * p.ldw1, p.ldw1, left > 0 ? (left < NC ? left : NC) : 1, left > 0 ? p.N0 : 0,
                                   dst, p.cg, wave, lane);
  };

  // the first chunks of W1: the oldest loads, the main loop's first wait covers them
#pragma unroll
  for (int c = 0; c < OWN; ++c) issue_chunk(c, own + c * SLOT);

  floatx16 acc0[FN0][FM];
  {
    const HaloArgs h{p.X, p.W0, p.N0, p.M, p.K0, p.ldw0, p.cg, m0};
    conv_halo_mainloop<BM, N0T, NW, 1, NS, XI, 1>(h, lds, acc0);
  }
  // every wave has passed the main loop's last barrier, which follows the last read of a W0 stage that is used
#pragma unroll
  for (int c = OWN; c < NCHUNK; ++c) issue_chunk(c, stages + (c - OWN) * SLOT);

  half8 d0[FN0 * 2][FM];
  b2b_make_d0<FN0, FM>(p, acc0, d0, g);

#pragma unroll
  for (int c = 0; c < NCHUNK; ++c) {
    if (c * NC >= p.N1) break;  // uniform over the workgroup
    floatx16 acc1[NC / 32][FM];
    b2b_rf_gemm<N0T, NC, FM>(c < OWN ? own + c * SLOT : stages + (c - OWN) * SLOT, d0, acc1, l32, g);
    // this wave's share of the late chunks has landed; the barrier that opens b2b_tile_out publishes it
    if (c == 0 && NCHUNK > OWN) __builtin_amdgcn_s_waitcnt(0x0F70);
    const EpilogueArgs ep{p.b1 + c * NC, p.b1_on, p.N1 - c * NC, p.alpha1, p.beta1, p.act1, RES ? p.gamma : 0.f};
    b2b_tile_out<BM, NW, NC, RES>(lds, acc1, ep, p.Y + c * NC, p.ldy, p.M, m0, wave, tid, RES ? p.res + c * NC : nullptr, p.ldr);
  }
}

template <int BM, int NW, int N0T, int N1T, int NS, int XI>
hipError_t launch_b2b_halo_chunked(const B2bParams& p, int /*grid*/, int lds_bytes, hipStream_t stream) {
  static LdsOptIn opt_in[2];
  if (p.res)
    return b2b_launch_common(b2b_halo_chunked_kernel<BM, NW, N0T, N1T, NS, XI, true>, opt_in[1], p, p.tiles_m, 64 * NW,
                             lds_bytes, stream);
  return b2b_launch_common(b2b_halo_chunked_kernel<BM, NW, N0T, N1T, NS, XI, false>, opt_in[0], p, p.tiles_m, 64 * NW,
                           lds_bytes, stream);
}

#define BOLT_B2B_HALO_CHUNKED_INSTANCE(BM, NW, N0T, N1T, NS, XI)                                               \
  {                                                                                                            \
    "b2bhalo_c64_" #BM "_w" #NW "_n" #N0T "_" #N1T "_s" #NS "_x" #XI, 0, BM, 64, NW, 1, N0T, N1T, 1, 0, 64 * NW,  \
        NS, nullptr, &bolt::launch_b2b_halo_chunked<BM, NW, N0T, N1T, NS, XI>,                                   \
        &bolt::B2bHaloChunkedTraits<BM, NW, N0T, N1T, NS, XI>::supports,                                         \
        &bolt::B2bHaloChunkedTraits<BM, NW, N0T, N1T, NS, XI>::lds_bytes, true, 0.3f                             \
  }

// mode 0 = RF-resident fusion; legality and LDS need depend on the geometry (dyn hooks)
#define BOLT_B2B_HALO_INSTANCE(BM, NW, N0T, N1T, NS, XI)                                                  \
  {                                                                                                       \
    "b2bhalo_" #BM "_w" #NW "_n" #N0T "_" #N1T "_s" #NS "_x" #XI, 0, BM, 64, NW, 1, N0T, N1T, 1, 0, 64 * NW, \
        NS, nullptr, &bolt::launch_b2b_halo<BM, NW, N0T, N1T, NS, XI>,                                     \
        &bolt::B2bHaloTraits<BM, NW, N0T, N1T, NS, XI>::supports,                                          \
        &bolt::B2bHaloTraits<BM, NW, N0T, N1T, NS, XI>::lds_bytes, true, 0.4f                              \
  }

}  // namespace bolt
