// Two-wave-group ("ping-pong"), persistent GEMM / implicit-GEMM convolution kernel for problems that fill the chip.
//
// The tiling is that of Section 2.2 (workgroup tile -> wave tile -> matrix-core instruction) with the
// template parameters of Section 3.2.2; what is new against fprop_dma_kernel is how the two waves that share a
// SIMD take turns, which matrix-core instruction is used, and that a workgroup walks over several output tiles.
//
// Wave groups.  The workgroup computes a 256 x 256 tile with 8 waves: waves 0-3 (group 0) and waves 4-7
// (group 1), wave w and wave w + 4 on the same SIMD, each wave a 128 x 64 part.  A wave alternates between
//   M phases: read the operand fragments of one 64-deep k-tile from LDS into registers and issue this wave's
//             share of the direct-to-LDS loads of a later k-tile, and
//   C phases: issue the MFMAs of that k-tile, nothing else,
// with a workgroup barrier after every phase, and group 1 runs one phase behind group 0.  So at any time one
// wave of a SIMD feeds the matrix pipe from registers while the other one waits on LDS and on the address
// path: an in-order wave that stalls on a read or on a full load queue never holds back an MFMA.  (Load
// instructions in front of the MFMAs of a C phase do exactly that: the address path takes 16 cycles per
// instruction, a k-tile is 64 of them, and the wave issues in order.)  Every wave executes the same number of
// barriers: group 1 one more in front of the k loop, group 0 one more behind it.
//
// Slot s = the time between two barriers: group 0 runs M(t) in slot 2t and C(t) in slot 2t + 1, group 1 runs
// M(t) in slot 2t + 1 and C(t) in slot 2t + 2.  The 160 KB of LDS hold two stages of the weight tile (32 KB
// each) and three of the activation tile.  Group 0 loads the weight tiles, group 1 the activation tiles, each in
// its M phases only:
//   W(t+1) goes to the stage of W(t-1), last read in slot 2t - 1; group 0 issues it in M(t) (slot 2t), waits for
//          it at the end of C(t) (slot 2t + 1), it is first read in slot 2t + 2;
//   X(t+2) goes to the stage of X(t-1); group 1 issues it in M(t) (slot 2t + 1), waits for X(t+1) - everything
//          but its newest 8 loads - at the end of the same phase; X(t+2) is first read in slot 2t + 4.
// Loads of k-tiles beyond the reduction are issued all the same: their offsets fall outside the buffer, the
// hardware writes zeros into a stage nobody reads any more, and the wait counts stay uniform.
//
// Persistence.  The grid has one workgroup per compute unit (fewer for small problems); workgroup w computes the
// output tiles w, w + grid, ...  When the k loop of a tile ends, the loads of the first k-tiles of the next tile
// (W(0), X(0), X(1): 96 KB) go out before the epilogue starts, and the epilogue stages the FP16 output through
// the 64 KB of LDS they leave free (the second weight stage and the third activation stage), one wave group's
// 128 rows at a time.  So the matrix pipe idles for the epilogue arithmetic only, not for the first loads of a
// tile and not for the output stores, which drain while the next tile is computed.
//
// Counting outstanding loads (s_waitcnt vmcnt(N)) stays valid with the output stores of the previous tile still
// in flight: loads complete in order among themselves, so "at most N operations outstanding" implies "at most N
// loads outstanding", whatever the stores do; the stores only make a wait more conservative.
#pragma once
#include <type_traits>
#include <utility>

#include "fprop_dma_kernel.hpp"

namespace bolt {

struct FpropPpTraits {
  static constexpr int BN = 256, BK = 64;
  static constexpr int NT = 512;
  static constexpr int WTN = 64;  // wave q of a group owns 64 columns; group g owns half of the tile's rows
  static constexpr int W_STAGES = 2, X_STAGES = 3;
  static constexpr int W_HALVES = BN * BK, X_HALVES = 256 * BK;  // one stage (an activation stage has room for 256 rows)
  static constexpr int LDS_BYTES = (W_STAGES * W_HALVES + X_STAGES * X_HALVES) * 2;
  static constexpr int CPR = BN / 8;  // 16-byte chunks per output row
  static_assert(LDS_BYTES <= 160 * 1024, "stages must fit the 160 KB LDS");
  static_assert(W_HALVES == 64 * BN && X_HALVES == 64 * BN, "a free stage holds 64 output rows");
};

template <typename F, int... I>
__device__ __forceinline__ void pp_static_for(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}

// MI: the matrix-core instruction, 32 (32 x 32 x 16) or 16 (16 x 16 x 32, see mfma_16x16x32).
// PK: reduction depth of one phase, 64 (one M and one C phase per k-tile) or 32 (two of each: half the fragment
//     registers and twice the barriers).  With two phases per tile the loads still go out in the first M phase of
//     a tile and the waits stay where they are.
// BM: rows of the output tile, 256 or 224 (two wave groups of 128 or 112 rows).  The narrower tile exists for the
//     tuner: 256 compute units each take whole tiles, and a problem of 6.1 rounds of 256-row tiles is 7.0 rounds of
//     224-row tiles that are 12.5 % shorter.
// The transpose-read swizzle of a row-major [64][256] weight tile for the 16 x 16 x 32 operand layout: a half-wave reads
// rows {0..3} and {8..11} (+16 for the other half) x 32 bytes, so chunk bits 2-3 take row bits 0-1 and chunk bit 1 takes row
// bit 3; the 8 rows x 2 chunks then fall into 16 different bank groups (rows are multiples of 256 bytes).
__device__ __forceinline__ int pp_kn_swizzle(int k) { return ((k & 3) << 2) | (((k >> 3) & 1) << 1); }

// WKN (GEMM only): the weights are row-major [K][N]; their k-tiles go to LDS as they lie in memory and the operand is
// gathered by the LDS transpose read (see DmaKnTileLoader in fprop_dma_kernel.hpp for the instruction's semantics).
template <int XMODE, int MI = 16, int PK = 64, bool RES = false, int BM = 256, bool WKN = false>
__global__ __launch_bounds__(512) void fprop_pp_kernel(const FpropParams p) {
  using T = FpropPpTraits;
  static_assert(!WKN || (XMODE == 0 && MI == 16), "row-major weights: GEMM rows, 16 x 16 x 32 instruction");
  static_assert(MI == 16 || MI == 32, "matrix-core instruction");
  static_assert(PK == 32 || PK == 64, "phase depth");
  static_assert(XMODE == 0 || XMODE == 1, "row-major matrix or implicit im2col");
  static_assert(BM <= 256 && (BM / 2) % MI == 0, "two wave groups of whole fragments");
  constexpr int BN = T::BN, BK = T::BK, WTM = BM / 2, WTN = T::WTN, CPR = T::CPR;
  constexpr int FM = WTM / MI, FN = WTN / MI;  // fragments per wave tile along M and N
  constexpr int MK = MI == 32 ? 16 : 32;       // reduction depth of one instruction
  constexpr int P = BK / PK;                   // phases per k-tile
  constexpr int KS = PK / MK;                  // k-steps per phase
  constexpr int KL = MK / 8;                   // lane groups along k: lane l reads chunk k * KL + l / MI of row l % MI
  using acc_t = std::conditional_t<MI == 32, floatx16, floatx4>;
  constexpr int L = 8;  // load instructions per wave per k-tile: 4 waves move 256 rows, 8 rows per instruction

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* const wring = lds;
  half_t* const xring = lds + T::W_STAGES * T::W_HALVES;
  // the two stages that hold nothing while the first k-tiles of the next output tile are on their way
  half_t* const free0 = wring + T::W_HALVES;
  half_t* const free1 = xring + 2 * T::X_HALVES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, wq = wave & 3;  // wave group (phase offset and operand it loads), wave inside the group
  const int wm = grp, wn = wq;
  const int g = lane / MI, lr = lane % MI;
  const int n_tiles = (p.K + BK - 1) / BK;
  const int total = p.tiles_m * p.tiles_n;

  // ---- this wave's loader ----------------------------------------------------------------------------------------
  // A wave moves rows (j * 4 + wq) * 8 + lane / 8, j = 0 .. 7, of ONE operand tile (group 0: weights, group 1:
  // activations); lane % 8 picks the 16-byte chunk of the 128-byte row, swizzled as in dma_chunk_offset.  Per row it
  // keeps one register, st[j]:
  //   matrix rows (weights; activations of a GEMM): the row's byte offset from the tile's first row, or the
  //     invalid offset for rows beyond the matrix (adding the k offset to it keeps it out of range);
  //   implicit im2col: pix0 << 10 | mask, where pix0 = (img * H + ih0) * W + iw0 is the linear pixel index of the
  //     window origin (negative when the origin lies above or left of the first image) and bit r * S + s of mask
  //     says that tap (r, s) of this output pixel reads padding (all taps for rows beyond M; bit 9 is always
  //     set and stands for every k-tile past the end of the reduction).  Four vector instructions turn it into
  //     the load offset of a tap; the tap and channel offsets themselves are wave-uniform, because a k-tile of
  //     64 channels lies inside one filter tap (C % 64 == 0).
  const int lrow = lane >> 3;
  const int lc16 = ((lane & 7) ^ dma_swizzle<BK>(wq * 8 + lrow)) << 4;  // byte offset of this lane's chunk in a row
  int st[L];
  __amdgpu_buffer_rsrc_t rsrc;
  const int k_limit_bytes = p.K * 2;
  int cur_r, cur_s, cur_c;  // conv: filter tap and first channel of the next k-tile to issue
  int m0, n0;               // the output tile whose operands the loader addresses

  auto setup_tile = [&](int tile) {
    int tm, tn;
    tile_of_workgroup(tile, p.tiles_m, p.tiles_n, p.swizzle, tm, tn);
    m0 = tm * BM;
    n0 = tn * BN;
    cur_r = cur_s = cur_c = 0;
    if (WKN && grp == 0) {
      // instruction j of this wave fills tile rows (k) 2 (4 j + wq) and the next: lane / 32 picks the row, lane % 32 the
      // 16-byte slot, which holds the row's chunk slot ^ swizzle(row).  st[j] = byte offset of that chunk from (row 0,
      // column n0), or the invalid offset for columns beyond N.
      const int64_t rem = ((int64_t)(p.K - 1) * p.ldw + (p.N - n0)) * 2;  // (the host keeps the matrix under 2 GiB)
      rsrc = make_rsrc(p.W + n0, (unsigned)rem);
#pragma unroll
      for (int j = 0; j < L; ++j) {
        const int krow = (j * 4 + wq) * 2 + (lane >> 5);
        const int c = (lane & 31) ^ pp_kn_swizzle(krow);
        st[j] = n0 + c * 8 < p.N ? krow * p.ldw * 2 + c * 16 : (int)kInvalidOffset;
      }
    } else if (grp == 0 || XMODE == 0) {
      const half_t* base = grp == 0 ? p.W + (int64_t)n0 * p.ldw : p.X + (int64_t)m0 * p.ldx;
      const int ld = grp == 0 ? p.ldw : p.ldx, rows_valid = grp == 0 ? p.N - n0 : p.M - m0;
      const int64_t rem = ((int64_t)(rows_valid - 1) * ld + p.K) * 2;
      rsrc = make_rsrc(base, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff));
#pragma unroll
      for (int j = 0; j < L; ++j) {
        const int row = (j * 4 + wq) * 8 + lrow;
        st[j] = row < rows_valid && (grp == 0 || row < BM) ? row * ld * 2 : (int)kInvalidOffset;
      }
    } else {
      const int64_t bytes = (int64_t)p.cg.H * p.cg.Wi * p.cg.C * 2 * (int64_t)(p.M / (p.cg.P * p.cg.Q));
      rsrc = make_rsrc(p.X, (unsigned)bytes);
      // the wave's rows are 32 output pixels apart: one division for the first, carries for the others
      const int PQ = p.cg.P * p.cg.Q;
      const int mfirst = m0 + wq * 8 + lrow;
      int img = mfirst / PQ;
      const int rem = mfirst - img * PQ;
      int op = rem / p.cg.Q, oq = rem - op * p.cg.Q;
#pragma unroll
      for (int j = 0; j < L; ++j) {
        int pix0 = 0, mask = 0x3ff;
        if (mfirst + j * 32 < p.M && wq * 8 + lrow + j * 32 < BM) {
          const int ih0 = op * p.cg.stride_h - p.cg.pad_h, iw0 = oq * p.cg.stride_w - p.cg.pad_w;
          pix0 = (img * p.cg.H + ih0) * p.cg.Wi + iw0;
          int rows_in = 0, cols_in = 0;  // bit r: window row r inside the image; bit s: window column s inside
          for (int r = 0; r < p.cg.R; ++r) rows_in |= (int)((unsigned)(ih0 + r) < (unsigned)p.cg.H) << r;
          for (int c = 0; c < p.cg.S; ++c) cols_in |= (int)((unsigned)(iw0 + c) < (unsigned)p.cg.Wi) << c;
          for (int r = 0; r < p.cg.R; ++r)
            if ((rows_in >> r) & 1) mask &= ~(cols_in << (r * p.cg.S));
        }
        st[j] = (pix0 << 10) | mask;
        oq += 32;
        while (oq >= p.cg.Q) {
          oq -= p.cg.Q;
          ++op;
        }
        while (op >= p.cg.P) {
          op -= p.cg.P;
          ++img;
        }
      }
    }
  };

  // per k-tile, for the gather: bit of the current tap in the masks, and this lane's byte offset of
  // (tap, first channel) relative to a window origin; for the weights of a convolution: byte offset of the
  // k-tile's first column, (tap * C + channel) * 2.
  // The k-tiles of a convolution are walked tap-fastest (all R * S taps of channels [c, c + 64), then the next 64
  // channels): the activation tiles of one channel block are the same pixels shifted by a tap, so all but the
  // first come out of the L2 instead of the memory-side cache - with the channel block fastest the re-use distance
  // is C / 64 k-tiles of every compute unit of the XCD, more than its L2 holds.
  int tap_bit = 0, tap_off = 0, w_kb = 0;
  auto set_tap = [&](int kt) {
    const int tap = cur_r * p.cg.S + cur_s;
    tap_bit = kt < n_tiles ? tap : 9;
    tap_off = ((cur_r * p.cg.Wi + cur_s) * p.cg.C + cur_c) * 2 + lc16;
    w_kb = kt < n_tiles ? (tap * p.cg.C + cur_c) * 2 : k_limit_bytes;
  };
  // Issue instruction j of k-tile kt into the 32 KB stage at dst.  Tiles are issued in increasing order.
  // gather: compile-time copy of "XMODE == 1 && grp == 1" where the caller knows it, so that the two groups of a
  // convolution get straight-line code of their own instead of a branch per load
  auto issue_one = [&](auto jc, int kt, half_t* dst, auto gather) {
    constexpr int j = decltype(jc)::value;
    half_t* slot = dst + (j * 4) * 8 * BK + wq * 8 * BK;
    unsigned off;
    // (the empty asm keeps the compiler from hoisting anything derived from st[j] out of the k loop - the unpacked
    // fields, st[j] + lc16: more than one register per row would not fit)
    int sj = st[j];
    asm volatile("" : "+v"(sj));
    if constexpr (decltype(gather)::value == 1) {
      const unsigned inv = __builtin_amdgcn_ubfe((unsigned)sj, (unsigned)tap_bit, 1u);
      off = (unsigned)(__mul24(sj >> 10, p.cg.C * 2) + tap_off) | (inv << 31);
    } else if constexpr (decltype(gather)::value == 2) {
      // row-major weights: k-tile kt starts 64 rows further down; rows at or beyond K are out of range
      const int krow = kt * BK + (j * 4 + wq) * 2 + (lane >> 5);
      off = ((unsigned)sj + (unsigned)(kt * BK * p.ldw * 2)) | (krow < p.K ? 0u : kInvalidOffset);
    } else {
      const int kb = (XMODE == 1 ? w_kb : kt * (BK * 2)) + lc16;
      off = ((unsigned)sj + (unsigned)kb) | (kb < k_limit_bytes ? 0u : kInvalidOffset);
    }
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, BOLT_LDS_PTR(slot), 16, off, 0, 0, 0);
  };
  auto advance_tile = [&]() {
    if (XMODE == 1) {
      if (++cur_s == p.cg.S) {
        cur_s = 0;
        if (++cur_r == p.cg.R) {
          cur_r = 0;
          cur_c += BK;
        }
      }
    }
  };
  auto issue_tile = [&](int kt, half_t* dst, auto gather) {
    if (XMODE == 1) set_tap(kt);
    pp_static_for([&](auto jc) { issue_one(jc, kt, dst, gather); }, std::make_integer_sequence<int, L>{});
    advance_tile();
  };
  using Gather = std::integral_constant<int, XMODE == 1 ? 1 : 0>;  // group 1 of a convolution
  using Rows = std::integral_constant<int, 0>;                    // matrix rows
  using WRows = std::integral_constant<int, WKN ? 2 : 0>;         // the weight tile: [N][K] rows, or row-major [K][N]
  // the first k-tiles of an output tile: W(0) by group 0, X(0) and X(1) by group 1
  auto issue_first_tiles = [&]() {
    if (grp == 0) {
      issue_tile(0, wring, WRows{});
    } else {
      issue_tile(0, xring, Gather{});
      issue_tile(1, xring + T::X_HALVES, Gather{});
    }
  };

  acc_t acc[FN][FM];
  half8 xf[KS][FM], wf[KS][FN];
  constexpr int NREAD = KS * (FM + FN);  // fragment reads per phase
  // row-major weights: this lane's offset (halves) inside the [64][256] tile for fragment column 0 of its wave and k-step
  // 0: row 8 g + (lr / 4), columns wn * 64 + 4 (lr % 4) .. +3.  Fragment column i flips chunk bits 1-2 (i * 16 halves),
  // k-step k adds 32 rows, the second transpose read 4 rows.
  int kn_off = 0;
  if constexpr (WKN) {
    const int r4 = lr >> 2, q4 = lr & 3;
    kn_off = (g * 8 + r4) * BN + (((wn * 8 + (q4 >> 1)) ^ pp_kn_swizzle(g * 8 + r4)) << 3) + (q4 & 1) * 4;
  }
  auto read_one = [&](const half_t* xs, const half_t* ws, int h, auto rc) {
    constexpr int r = decltype(rc)::value, k = r / (FM + FN), i = r % (FM + FN);
    const int chunk = (h * KS + k) * KL + g;
    if constexpr (i < FM) xf[k][i] = *(const half8*)(xs + dma_chunk_offset<BK>(wm * WTM + i * MI + lr, chunk));
    else if constexpr (WKN) {
      int ko = kn_off;  // (the empty asm keeps the per-fragment addresses from being hoisted out of the k loop: one register, not eight)
      asm volatile("" : "+v"(ko));
      wf[k][i - FM] = kn_frag_read<BN>(ws, ko ^ ((i - FM) * 16), (h * KS + k) * MK);
    }
    else wf[k][i - FM] = *(const half8*)(ws + dma_chunk_offset<BK>(wn * WTN + (i - FM) * MI + lr, chunk));
  };
  // LDS read instructions of fragment reads [r0, r1) of a phase (a row-major weight fragment takes two)
  constexpr auto ds_reads = [](int r0, int r1) constexpr {
    int n = 0;
    for (int r = r0; r < r1; ++r) n += (WKN && r % (FM + FN) >= FM) ? 2 : 1;
    return n;
  };
  // An M phase that also loads: the L load instructions of k-tile kt (into dst) interleaved with the phase's fragment
  // reads, so that the address path and the LDS pipe work side by side.
  auto m_phase_loads = [&](half_t* dst, int kt, const half_t* xs, const half_t* ws, auto gather) {
    if (XMODE == 1) set_tap(kt);
    pp_static_for([&](auto jc) {
      constexpr int j = decltype(jc)::value, r0 = j * NREAD / L, r1 = (j + 1) * NREAD / L;
      issue_one(jc, kt, dst, gather);
      pp_static_for([&](auto ic) { read_one(xs, ws, 0, std::integral_constant<int, r0 + decltype(ic)::value>{}); },
                    std::make_integer_sequence<int, r1 - r0>{});
    }, std::make_integer_sequence<int, L>{});
    advance_tile();
    pp_static_for([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                        // one load
      __builtin_amdgcn_sched_group_barrier(0x100, ds_reads(j * NREAD / L, (j + 1) * NREAD / L), 0);  // its share of reads
    }, std::make_integer_sequence<int, L>{});
  };
  auto m_phase_reads = [&](const half_t* xs, const half_t* ws, int h) {
    pp_static_for([&](auto ic) { read_one(xs, ws, h, ic); }, std::make_integer_sequence<int, NREAD>{});
  };
  auto c_phase = [&]() {
    pp_static_for([&](auto ic) {
      constexpr int i = decltype(ic)::value, k = i / (FM * FN), a = (i / FM) % FN, b = i % FM;
      if constexpr (MI == 32) acc[a][b] = mfma_32x32x16(wf[k][a], xf[k][b], acc[a][b]);
      else acc[a][b] = mfma_16x16x32(wf[k][a], xf[k][b], acc[a][b]);
    }, std::make_integer_sequence<int, KS * FM * FN>{});
  };
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  // gfx9 s_waitcnt encoding: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8]
  auto wait_reads = [] { __builtin_amdgcn_s_waitcnt(0xC07F); };            // lgkmcnt(0)
  auto wait_loads_0 = [] { __builtin_amdgcn_s_waitcnt(0x0F70); };          // vmcnt(0)
  auto wait_loads_L = [] { __builtin_amdgcn_s_waitcnt(0x0F70 | L); };      // vmcnt(L): all but the newest tile

  // ---- the epilogue of one tile (Section 3.1, patterns (i)-(iii)) -------------------------------------------------
  // Each wave group moves its own 128 rows through its own free stage (group 0: free0, group 1: free1), 64 rows at
  // a time: its waves write their accumulators as FP16 quads into the stage (16-byte chunks XOR-swizzled by row as
  // in fprop_tile_out), then its 256 threads move whole 16-byte row pieces to global memory with non-temporal
  // stores.  Both groups run the same steps side by side, so the workgroup barriers between the steps cost no idle
  // group.  With a residual, the 64 rows of C are first fetched into the same LDS locations.
  // The bias does not wait for the epilogue: the accumulators of a tile start at (beta / alpha) * bias instead of
  // zero, so that alpha * accumulator is alpha * sum + beta * bias (Eq. 1 with C0 the broadcast bias).  The bias quads
  // of this lane's columns are requested just before the first k-tiles of the tile and awaited together with them; a
  // load inside the epilogue would have to wait for everything requested before it, the 96 KB of the next tile's
  // first k-tiles included.  With alpha == 0 the accumulators start at zero and the epilogue fetches the bias itself.
  constexpr int NBQ = MI == 32 ? FN * 4 : FN;  // quads of 4 columns per lane
  half4 bias_q[NBQ];
  const bool bias_in_acc = p.alpha != 0.f;
  auto quad_col = [&](int i, int gl) { return MI == 32 ? wn * WTN + (i >> 2) * 32 + (i & 3) * 8 + gl * 4 : wn * WTN + i * 16 + gl * 4; };
  auto load_bias = [&](int en0) {
#pragma unroll
    for (int i = 0; i < NBQ; ++i) {
      const int n = en0 + quad_col(i, g);
      bias_q[i] = *(const half4*)(p.bias + (n < p.N ? n : 0) * p.bias_on);
    }
  };
  auto quad_out = [&](floatx4 v, half4 hb, half4 res, auto slow, auto with_bias) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = p.alpha * v[e];
      if constexpr (decltype(with_bias)::value) v[e] += p.beta * (float)hb[e];
      if constexpr (RES) v[e] += p.gamma * (float)res[e];
    }
    if constexpr (decltype(slow)::value) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = p.act == ACT_RELU ? (v[e] > 0.f ? v[e] : 0.f) : v[e];
      v = apply_act_slow4(v, p.act);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float r = v[e] > 0.f ? v[e] : 0.f;
        v[e] = p.act == ACT_RELU ? r : v[e];
      }
    }
    half4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (half_t)v[e];
    return o;
  };
  auto epilogue = [&](int em0, int en0) {
    // (everything the epilogue derives from the lane id is invariant across output tiles; the empty asm keeps the
    // compiler from hoisting those addresses out of the tile loop and holding them in registers through the k loop)
    int elane = lane;
    asm volatile("" : "+v"(elane));
    const int eg = elane / MI, elr = elane % MI, gtid = wq * 64 + elane;  // thread index inside the wave group
    half_t* const stage = grp == 0 ? free0 : free1;
    const int r_half = em0 + grp * WTM;  // first output row of this group
    if (!bias_in_acc) load_bias(en0);
    constexpr int BPS = 64 / MI;         // fragment rows (b) per 64-row sub-pass
    auto write_quads = [&](auto sc, auto slow, auto with_bias) {
      constexpr int sp = decltype(sc)::value;
#pragma unroll
      for (int i = 0; i < NBQ; ++i) {
        const int nl = quad_col(i, eg);
#pragma unroll
        for (int bb = 0; bb < BPS; ++bb) {
          const int b = sp * BPS + bb, srow = bb * MI + elr;
          if (b >= FM) continue;  // the last sub-pass of a 112-row group holds 48 rows
          half4* slot = (half4*)(stage + srow * BN + (((nl >> 3) ^ ctile_swizzle<CPR>(srow)) << 3) + (nl & 4));
          floatx4 v;
          if constexpr (MI == 32) {
            const int a = i >> 2, q4 = i & 3;
            v = floatx4{acc[a][b][q4 * 4], acc[a][b][q4 * 4 + 1], acc[a][b][q4 * 4 + 2], acc[a][b][q4 * 4 + 3]};
          } else {
            v = acc[i][b];
          }
          half4 res = {0, 0, 0, 0};
          if constexpr (RES) res = *slot;
          *slot = quad_out(v, bias_q[i], res, slow, with_bias);
        }
      }
    };
    pp_static_for([&](auto sc) {
      constexpr int sp = decltype(sc)::value;
      const int r_base = r_half + sp * 64;  // first output row of this sub-pass
      barrier_after_lds_writes();           // the previous sub-pass has been read out (first: the k loop's reads)
      if constexpr (RES) {
        // direct-to-LDS, 16 bytes per lane, two rows of 256 columns per instruction; rows beyond M and columns
        // beyond N are zero-filled
        const int64_t rem = ((int64_t)(p.M - r_base - 1) * p.ldr + p.N) * 2;
        const __amdgpu_buffer_rsrc_t rr =
            make_rsrc(p.res + (int64_t)r_base * p.ldr, rem <= 0 ? 0u : (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff));
        for (int i = wq; i < 32; i += 4) {
          const int srow = i * 2 + (elane >> 5);
          const int c = (elane & 31) ^ ctile_swizzle<CPR>(srow);
          const bool ok = r_base + srow < p.M && sp * 64 + srow < WTM && en0 + c * 8 < p.N;
          const unsigned off = ok ? (unsigned)((srow * p.ldr + en0 + c * 8) * 2) : kInvalidOffset;
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rr, BOLT_LDS_PTR(stage + i * 2 * BN), 16, off, 0, 0, 0);
        }
        barrier_after_loads<0>();
      }
      if (!bias_in_acc) write_quads(sc, std::true_type{}, std::true_type{});  // rare: slow path for every activation
      else if (p.act > ACT_RELU) write_quads(sc, std::true_type{}, std::false_type{});
      else write_quads(sc, std::false_type{}, std::false_type{});
      barrier_after_lds_writes();
      const int chunk = gtid % CPR, r0 = gtid / CPR;  // 8 rows per sweep of the group's 256 threads
      const int n = en0 + chunk * 8;
      if (n < p.N) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int srow = r0 + i * 8;
          if (r_base + srow < p.M && sp * 64 + srow < WTM) {
            const half8 v = *(const half8*)(stage + srow * BN + ((chunk ^ ctile_swizzle<CPR>(srow)) << 3));
            __builtin_nontemporal_store(v, (half8*)(p.Y + (int64_t)(r_base + srow) * p.ldy + n));
          }
        }
      }
    }, std::make_integer_sequence<int, 2>{});
  };

  // ---- the first output tile of this workgroup ---------------------------------------------------------------------
  int tile = blockIdx.x;
  setup_tile(tile);
  load_bias(n0);
  issue_first_tiles();

  while (true) {
    // tile 0 of the reduction has landed for everyone (group 1: X(1) may still fly), and with it the older bias
    // quads; group 1 drops one slot behind
    if (grp == 0) wait_loads_0();
    else wait_loads_L();
    wait_reads();  // and this wave's LDS reads of the previous epilogue have returned
    const float bias_scale = bias_in_acc ? p.beta / p.alpha : 0.f;
#pragma unroll
    for (int i = 0; i < NBQ; ++i)
#pragma unroll
      for (int b = 0; b < FM; ++b)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v = (float)bias_q[i][e] * bias_scale;
          if constexpr (MI == 32) acc[i >> 2][b][(i & 3) * 4 + e] = v;
          else acc[i][b][e] = v;
        }
    raw_barrier();
    if (grp == 1) raw_barrier();

    int ws_cur = 0, xs_cur = 0;  // stages of W(t) and X(t)
    for (int t = 0; t < n_tiles; ++t) {
      const int ws_next = ws_cur ^ 1;                    // stage of W(t+1) = stage of W(t-1)
      const int xs_fill = xs_cur == 0 ? 2 : xs_cur - 1;  // stage of X(t+2) = stage of X(t-1)
      const half_t* xs = xring + xs_cur * T::X_HALVES;
      const half_t* ws = wring + ws_cur * T::W_HALVES;
#pragma unroll
      for (int h = 0; h < P; ++h) {
        // ---- M phase --------------------------------------------------------------------------------------
        fence();
        if (h == 0) {
          if constexpr (XMODE == 0 && !WKN) {
            // both groups run the same code on their own rows, offsets and stage
            m_phase_loads(grp == 0 ? wring + ws_next * T::W_HALVES : xring + xs_fill * T::X_HALVES, t + 1 + grp, xs, ws, Rows{});
          } else if constexpr (XMODE == 0) {
            if (grp == 0) m_phase_loads(wring + ws_next * T::W_HALVES, t + 1, xs, ws, WRows{});
            else m_phase_loads(xring + xs_fill * T::X_HALVES, t + 2, xs, ws, Rows{});
          } else {
            if (grp == 0) m_phase_loads(wring + ws_next * T::W_HALVES, t + 1, xs, ws, Rows{});
            else m_phase_loads(xring + xs_fill * T::X_HALVES, t + 2, xs, ws, Gather{});
          }
        } else {
          m_phase_reads(xs, ws, h);
        }
        wait_reads();
        if (h == P - 1 && grp == 1) wait_loads_L();  // X(t+1) has landed
        fence();
        raw_barrier();
        // ---- C phase --------------------------------------------------------------------------------------
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
    // Nothing of this workgroup is on its way into LDS any more (the zero-filled tiles past the end included),
    // and nobody reads a stage: the first k-tiles of the next output tile may go out.
    wait_loads_0();
    raw_barrier();
    const int em0 = m0, en0 = n0;
    tile += gridDim.x;
    const bool more = tile < total;
    if (more) {
      setup_tile(tile);
      load_bias(n0);
      issue_first_tiles();
    }
    epilogue(em0, en0);
    if (!more) break;
  }
}

template <int XMODE, int MI = 16, int PK = 64, int BM = 256, bool WKN = false>
hipError_t launch_fprop_pp(const FpropParams& p, hipStream_t stream) {
  using T = FpropPpTraits;
  auto kern = p.res ? fprop_pp_kernel<XMODE, MI, PK, true, BM, WKN> : fprop_pp_kernel<XMODE, MI, PK, false, BM, WKN>;
  static LdsOptIn opt_in[2];
  if (hipError_t e = opt_in[p.res ? 1 : 0].ensure((const void*)kern, T::LDS_BYTES); e != hipSuccess) return e;
  // one workgroup per compute unit; 256 is a multiple of the 8 XCDs, so the tiles w, w + 256, ... of a workgroup
  // stay on the XCD that tile_of_workgroup assumes for them
  constexpr int kComputeUnits = 256;
  const int tiles = p.tiles_m * p.tiles_n;
  dim3 grid(tiles < kComputeUnits ? tiles : kComputeUnits, 1, 1);
  hipLaunchKernelGGL(kern, grid, dim3(T::NT), T::LDS_BYTES, stream, p);
  return hipGetLastError();
}

// What the packed per-row state of the implicit-GEMM loader can express.
inline bool fprop_pp_conv_supports(const FpropParams& p) {
  const int64_t batch = p.M / ((int64_t)p.cg.P * p.cg.Q);
  const int64_t pixels = batch * p.cg.H * p.cg.Wi, origin = (int64_t)p.cg.pad_h * p.cg.Wi + p.cg.pad_w;
  return p.cg.C % 64 == 0 && p.cg.R * p.cg.S <= 9 && pixels + origin < (1 << 21) && p.cg.C < (1 << 22);
}
inline int fprop_pp_lds_bytes(const FpropParams&) { return FpropPpTraits::LDS_BYTES; }

// In the instance table: 8 waves as 2 (M) x 4 (N), two LDS stages of weights, three of activations (reported as 2),
// no split-K.
#define BOLT_FPROP_PP_INSTANCE(XMODE, MI, PK, BM)                                                           \
  {                                                                                                         \
    "pp_" #BM "x256x64_w2x4_mi" #MI "_pk" #PK, BM, 256, 64, 2, 4, XMODE, 0, 2, bolt::FpropPpTraits::LDS_BYTES, \
        &bolt::launch_fprop_pp<XMODE, MI, PK, BM>,                                                          \
        XMODE == 1 ? &bolt::fprop_pp_conv_supports : nullptr, XMODE == 1 ? &bolt::fprop_pp_lds_bytes : nullptr, 0, MI, true \
  }

// The GEMM form for row-major weights (wmode 1).
#define BOLT_FPROP_PP_KN_INSTANCE(MI, PK, BM)                                                                \
  {                                                                                                         \
    "ppkn_" #BM "x256x64_w2x4_mi" #MI "_pk" #PK, BM, 256, 64, 2, 4, 0, 1, 2, bolt::FpropPpTraits::LDS_BYTES,    \
        &bolt::launch_fprop_pp<0, MI, PK, BM, true>, nullptr, nullptr, 0, MI, true, false, true               \
  }

}  // namespace bolt
