// Two-wave-group ("ping-pong") GEMM / implicit-GEMM convolution kernel for problems that fill the chip.
//
// The tiling is that of Section 2.2 (workgroup tile -> wave tile -> matrix-core instruction) with the
// template parameters of Section 3.2.2; what is new against fprop_dma_kernel is how the two waves that share a
// SIMD take turns.  The workgroup computes a 256 x 256 tile with 8 waves: waves 0-3 (group 0) and waves 4-7
// (group 1), wave w and wave w + 4 on the same SIMD, each wave a 128 x 64 part.  A wave alternates between
//   M phases: read the operand fragments of one 64-deep k-tile from LDS into registers and issue this wave's
//             share of the direct-to-LDS loads of a later k-tile, and
//   C phases: issue the 32 MFMAs of that k-tile, nothing else,
// with a workgroup barrier after every phase, and group 1 runs one phase behind group 0.  So at any time one
// wave of a SIMD feeds the matrix pipe from registers while the other one waits on LDS and on the address
// path: an in-order wave that stalls on a read or on a full load queue never holds back an MFMA.  (Load
// instructions in front of the MFMAs of a C phase do exactly that: the address path takes 16 cycles per
// instruction, a k-tile is 64 of them, and the wave issues in order.)  Every wave executes the same number of
// barriers: group 1 one more in front, group 0 one more behind.
//
// Slot s = the time between two barriers: group 0 runs M(t) in slot 2t and C(t) in slot 2t + 1, group 1 runs
// M(t) in slot 2t + 1 and C(t) in slot 2t + 2.  The 160 KB of LDS hold two stages of the weight tile (32 KB
// each) and three of the activation tile.  Group 0 loads the weight tiles, group 1 the activation tiles, each in
// its M phases only:
//   W(t+1) goes to the stage of W(t-1), last read in slot 2t - 1; group 0 issues it in M(t) (slot 2t), waits for
//          it at the end of C(t) (slot 2t + 1), it is first read in slot 2t + 2;
//   X(t+2) goes to the stage of X(t-1); group 1 issues it in M(t) (slot 2t + 1), waits for X(t+1) - everything
//          but its newest 8 loads - at the end of the same phase; X(t+2) is first read in slot 2t + 4.
// Loads of tiles beyond the reduction are issued all the same: their offsets fall outside the buffer, the
// hardware writes zeros into a stage nobody reads any more, and the wait counts stay uniform.
#pragma once
#include <type_traits>
#include <utility>

#include "fprop_dma_kernel.hpp"

namespace bolt {

struct FpropPpTraits {
  static constexpr int BM = 256, BN = 256, BK = 64;
  static constexpr int NT = 512;
  static constexpr int WTM = 128, WTN = 64;  // group g owns rows [128 g, 128 g + 128), wave q of a group 64 columns
  static constexpr int W_STAGES = 2, X_STAGES = 3;
  static constexpr int W_HALVES = BN * BK, X_HALVES = BM * BK;  // one stage
  static constexpr int PIPE_BYTES = (W_STAGES * W_HALVES + X_STAGES * X_HALVES) * 2;
  static constexpr int CTILE_BYTES = BM * BN * 2;
  static constexpr int LDS_BYTES = PIPE_BYTES > CTILE_BYTES ? PIPE_BYTES : CTILE_BYTES;
  static constexpr int CPR = BN / 8;
  static constexpr int STORE_THREADS = NT;
  static constexpr int ROWS_PER_PASS = NT / CPR;
  static_assert(PIPE_BYTES <= 160 * 1024, "stages must fit the 160 KB LDS");
};

template <typename F, int... I>
__device__ __forceinline__ void pp_static_for(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}

// ABL: ablation bits for measurements only (results are wrong with any of them set; every access stays in
// bounds and every wave still reaches every barrier): 1 = no global loads in the steady state,
// 2 = no fragment reads in the steady state, 4 = no MFMAs, 8 = every workgroup computes tile (0, 0).
// MI: the matrix-core instruction, 32 (32 x 32 x 16) or 16 (16 x 16 x 32, see mfma_16x16x32).
// PK: reduction depth of one phase, 64 (one M and one C phase per k-tile) or 32 (two of each: half the fragment
//     registers, which the implicit-GEMM gather needs for its per-row state, and twice the barriers).  With two
//     phases per tile the loads still go out in the first M phase of a tile and the waits stay where they are.
template <int XMODE, int MI = 16, int PK = 64, bool RES = false, int ABL = 0>
__global__ __launch_bounds__(512) void fprop_pp_kernel(const FpropParams p) {
  using T = FpropPpTraits;
  static_assert(MI == 16 || MI == 32, "matrix-core instruction");
  static_assert(PK == 32 || PK == 64, "phase depth");
  constexpr int BM = T::BM, BN = T::BN, BK = T::BK, WTM = T::WTM, WTN = T::WTN;
  constexpr int FM = WTM / MI, FN = WTN / MI;  // fragments per wave tile along M and N
  constexpr int MK = MI == 32 ? 16 : 32;       // reduction depth of one instruction
  constexpr int P = BK / PK;                   // phases per k-tile
  constexpr int KS = PK / MK;                  // k-steps per phase
  constexpr int KL = MK / 8;                   // lane groups along k: lane l reads chunk k * KL + l / MI of row l % MI
  using acc_t = std::conditional_t<MI == 32, floatx16, floatx4>;
  using XL = DmaTileLoader<BM, BK, 4, XMODE>;
  using WL = DmaTileLoader<BN, BK, 4, 0>;
  constexpr int L = 8;  // load instructions per wave per k-tile
  static_assert(XL::NI == L && WL::NI == L, "each group moves one operand tile with 8 instructions per wave");

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* const wring = lds;
  half_t* const xring = lds + T::W_STAGES * T::W_HALVES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, wq = wave & 3;  // wave group (phase offset and operand it loads), wave inside the group
  const int wm = grp, wn = wq;
  const int g = lane / MI, lr = lane % MI;
  int tm, tn;
  tile_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, p.swizzle, tm, tn);
  if (ABL & 8) tm = tn = 0;
  const int m0 = tm * BM, n0 = tn * BN;
  const int n_tiles = (p.K + BK - 1) / BK;

  XL xl;
  WL wl;
  if (grp == 1) {
    if constexpr (XMODE == 0) {
      const int64_t rem = ((int64_t)(p.M - m0 - 1) * p.ldx + p.K) * 2;
      xl.init(p.X + (int64_t)m0 * p.ldx, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff), p.ldx, p.M - m0, p.K, p.cg, m0, 0,
              wq, lane);
    } else {
      const int64_t bytes = (int64_t)p.cg.H * p.cg.Wi * p.cg.C * 2 * (int64_t)(p.M / (p.cg.P * p.cg.Q));
      xl.init(p.X, (unsigned)bytes, 0, p.M - m0, p.K, p.cg, m0, 0, wq, lane);
    }
  } else {
    const int64_t rem = ((int64_t)(p.N - n0 - 1) * p.ldw + p.K) * 2;
    wl.init(p.W + (int64_t)n0 * p.ldw, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff), p.ldw, p.N - n0, p.K, p.cg, n0, 0, wq,
            lane);
  }

  acc_t acc[FN][FM];
#pragma unroll
  for (int a = 0; a < FN; ++a)
#pragma unroll
    for (int b = 0; b < FM; ++b)
#pragma unroll
      for (int r = 0; r < (MI == 32 ? 16 : 4); ++r) acc[a][b][r] = 0.f;

  half8 xf[KS][FM], wf[KS][FN];
  constexpr int NREAD = KS * (FM + FN);  // fragment reads per phase
  auto read_one = [&](const half_t* xs, const half_t* ws, int h, auto rc) {
    constexpr int r = decltype(rc)::value, k = r / (FM + FN), i = r % (FM + FN);
    const int chunk = (h * KS + k) * KL + g;
    if constexpr (i < FM) xf[k][i] = *(const half8*)(xs + dma_chunk_offset<BK>(wm * WTM + i * MI + lr, chunk));
    else wf[k][i - FM] = *(const half8*)(ws + dma_chunk_offset<BK>(wn * WTN + (i - FM) * MI + lr, chunk));
  };
  // An M phase that also loads: the L load instructions of k-tile kt (into dst) interleaved with the phase's fragment
  // reads, so that the address path and the LDS pipe work side by side.
  auto m_phase_loads = [&](auto& loader, half_t* dst, int kt, const half_t* xs, const half_t* ws, bool first) {
    pp_static_for([&](auto jc) {
      constexpr int j = decltype(jc)::value, r0 = j * NREAD / L, r1 = (j + 1) * NREAD / L;
      if constexpr (!(ABL & 1)) loader.template issue_part<j, j + 1>(kt, dst, p.cg);
      if (!(ABL & 2) || first)
        pp_static_for([&](auto ic) { read_one(xs, ws, 0, std::integral_constant<int, r0 + decltype(ic)::value>{}); },
                      std::make_integer_sequence<int, r1 - r0>{});
    }, std::make_integer_sequence<int, L>{});
    if constexpr (!(ABL & 1)) loader.advance(p.cg);
    if constexpr (!(ABL & 3)) {
      pp_static_for([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                        // one load
        __builtin_amdgcn_sched_group_barrier(0x100, (j + 1) * NREAD / L - j * NREAD / L, 0);      // its share of reads
      }, std::make_integer_sequence<int, L>{});
    }
  };
  auto m_phase_reads = [&](const half_t* xs, const half_t* ws, int h) {
    if constexpr (!(ABL & 2))
      pp_static_for([&](auto ic) { read_one(xs, ws, h, ic); }, std::make_integer_sequence<int, NREAD>{});
  };
  auto c_phase = [&]() {
    pp_static_for([&](auto ic) {
      constexpr int i = decltype(ic)::value, k = i / (FM * FN), a = (i / FM) % FN, b = i % FM;
      if constexpr (!(ABL & 4)) {
        if constexpr (MI == 32) acc[a][b] = mfma_32x32x16(wf[k][a], xf[k][b], acc[a][b]);
        else acc[a][b] = mfma_16x16x32(wf[k][a], xf[k][b], acc[a][b]);
      }
    }, std::make_integer_sequence<int, KS * FM * FN>{});
  };
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  // gfx9 s_waitcnt encoding: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8]
  auto wait_reads = [] { __builtin_amdgcn_s_waitcnt(0xC07F); };            // lgkmcnt(0)
  auto wait_loads_0 = [] { __builtin_amdgcn_s_waitcnt(0x0F70); };          // vmcnt(0)
  auto wait_loads_L = [] { __builtin_amdgcn_s_waitcnt(0x0F70 | L); };      // vmcnt(L): all but the newest tile

  // ---- prologue: W(0), X(0), X(1); tile 0 landed for everyone; group 1 drops one slot behind --------------------
  if (grp == 0) {
    wl.issue(0, wring, p.cg);
    if (ABL & 1) wl.issue(1, wring + T::W_HALVES, p.cg);  // every stage holds real data
    wait_loads_0();
  } else {
    xl.issue(0, xring, p.cg);
    xl.issue(1, xring + T::X_HALVES, p.cg);
    if (ABL & 1) xl.issue(2, xring + 2 * T::X_HALVES, p.cg);
    if (ABL & 1) wait_loads_0();
    wait_loads_L();
  }
  raw_barrier();
  if (grp == 1) raw_barrier();

  int ws_cur = 0, xs_cur = 0;  // stages of W(t) and X(t)
  for (int t = 0; t < n_tiles; ++t) {
    const int ws_next = ws_cur ^ 1;                          // stage of W(t+1) = stage of W(t-1)
    const int xs_fill = xs_cur == 0 ? 2 : xs_cur - 1;        // stage of X(t+2) = stage of X(t-1)
    const half_t* xs = xring + xs_cur * T::X_HALVES;
    const half_t* ws = wring + ws_cur * T::W_HALVES;
#pragma unroll
    for (int h = 0; h < P; ++h) {
      // ---- M phase ----------------------------------------------------------------------------------------
      fence();
      if (h == 0) {
        if (grp == 0) m_phase_loads(wl, wring + ws_next * T::W_HALVES, t + 1, xs, ws, t == 0);
        else m_phase_loads(xl, xring + xs_fill * T::X_HALVES, t + 2, xs, ws, t == 0);
      } else {
        m_phase_reads(xs, ws, h);
      }
      wait_reads();
      if (h == P - 1 && grp == 1) {
        if constexpr (ABL & 1) wait_loads_0();
        else wait_loads_L();  // X(t+1) has landed
      }
      fence();
      raw_barrier();
      // ---- C phase ----------------------------------------------------------------------------------------
      fence();
      __builtin_amdgcn_s_setprio(1);
      c_phase();
      __builtin_amdgcn_s_setprio(0);
      if (h == P - 1 && grp == 0) wait_loads_0();  // W(t+1) has landed
      fence();
      raw_barrier();
    }
    ws_cur = ws_next;
    xs_cur = xs_cur == 2 ? 0 : xs_cur + 1;
  }
  if (grp == 0) raw_barrier();
  wait_loads_0();  // nothing of this wave is still on its way into LDS

  if constexpr (MI == 32) {
    fprop_tile_out<RES, BM, BN, WTM, WTN, T::STORE_THREADS, T::ROWS_PER_PASS>(lds, acc, p, m0, n0, wm, wn, true, tid);
  } else {
    // 16 x 16 accumulators: lane l holds columns 4 (l / 16) .. +3 of row l % 16 of its fragment, one quad
    fprop_tile_out_with<RES, BM, BN, T::STORE_THREADS, T::ROWS_PER_PASS>(lds, p, m0, n0, true, tid, [&](auto slow, const EpilogueArgs& ep) {
#pragma unroll
      for (int a = 0; a < FN; ++a) {
        const int nl = wn * WTN + a * 16 + g * 4;  // column inside the tile
#pragma unroll
        for (int b = 0; b < FM; ++b) {
          const int row = wm * WTM + b * 16 + lr;
          half4* slot = (half4*)(lds + row * BN + (((nl >> 3) ^ ctile_swizzle<T::CPR>(row)) << 3) + (nl & 4));
          if constexpr (RES) *slot = epilogue_quad4_impl<decltype(slow)::value, true>(acc[a][b], n0 + nl, ep, *slot);
          else *slot = epilogue_quad4_impl<decltype(slow)::value, false>(acc[a][b], n0 + nl, ep, half4{0, 0, 0, 0});
        }
      }
    });
  }
}

template <int XMODE, int MI = 16, int PK = 64, int ABL = 0>
hipError_t launch_fprop_pp(const FpropParams& p, hipStream_t stream) {
  using T = FpropPpTraits;
  auto kern = p.res ? fprop_pp_kernel<XMODE, MI, PK, true, ABL> : fprop_pp_kernel<XMODE, MI, PK, false, ABL>;
  static bool attr_set[2] = {false, false};
  if (!attr_set[p.res ? 1 : 0]) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set[p.res ? 1 : 0] = true;
  }
  dim3 grid(p.tiles_m * p.tiles_n, 1, 1);
  hipLaunchKernelGGL(kern, grid, dim3(T::NT), T::LDS_BYTES, stream, p);
  return hipGetLastError();
}

// In the instance table: 8 waves as 2 (M) x 4 (N), two LDS stages of weights,
// three of activations (reported as 2), no split-K.
#define BOLT_FPROP_PP_INSTANCE(XMODE, MI, PK)                                                               \
  {                                                                                                         \
    "pp_256x256x64_w2x4_mi" #MI "_pk" #PK, 256, 256, 64, 2, 4, XMODE, 0, 2, bolt::FpropPpTraits::LDS_BYTES,  \
        &bolt::launch_fprop_pp<XMODE, MI, PK>, 0, nullptr, nullptr, nullptr, nullptr, 0, MI, true           \
  }

}  // namespace bolt
