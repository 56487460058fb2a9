// Implicit-GEMM convolution for stride-1 "same" filters (output extent = input extent, e.g. the
// 3x3 / pad 1 layers of Section 4.1.1), with the activation halo re-used out of LDS.
//
// The generic implicit-GEMM kernel streams an im2col k-tile per filter tap: a 3x3 filter fetches
// every input pixel nine times through the L1/L2 path.  For stride 1 and "same" padding the
// im2col row of output pixel m at tap (r, s) is simply input pixel m + (r - pad_h) * W + (s - pad_w)
// in the flattened (n, h, w) pixel index, so a tile of BM consecutive output pixels needs the
// contiguous pixel range [m0 - halo, m0 + BM + halo), halo = pad_h * W + pad_w, ONCE per 64-channel
// chunk.  That range is loaded to LDS once and every tap reads its MFMA fragments from it at a
// shifted row; taps that fall outside the image (zero padding, image boundaries inside the flat
// range) are masked per lane.  Weights stream as before, one [BN x 64] k-tile per (tap, chunk).
//
// Everything else (transposed-product MFMA layout, 64-bank swizzle, direct-to-LDS loads with
// hardware zero fill, NS-stage weight pipeline with one barrier per item, register double-buffered
// fragments, LDS-staged coalesced epilogue) is shared with fprop_dma_kernel.hpp.
#pragma once
#include "fprop_dma_kernel.hpp"

namespace bolt {

// KG k-groups: set g of WAVES_M x WAVES_N waves reduces over the 64-channel chunks g, g + KG, ... with
// its own halo buffers and weight stages; the sets' accumulators are summed through LDS in a fixed
// order before the epilogue (as in fprop_dma_kernel.hpp).
template <int BM, int BN, int WAVES_M, int WAVES_N, int NS, int XI, int KG = 1>
struct ConvHaloTraits {
  static constexpr int BK = 64;
  static constexpr int NW = WAVES_M * WAVES_N;  // waves per k-group
  static constexpr int NT = 64 * NW * KG;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int FM = WTM / 32, FN = WTN / 32;
  static constexpr int CPR = BN / 8;
  static constexpr int STORE_THREADS = NT / CPR <= BM ? NT : BM * CPR;
  static constexpr int ROWS_PER_PASS = STORE_THREADS / CPR;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(STORE_THREADS % CPR == 0 && BM % ROWS_PER_PASS == 0 && NT <= 1024, "C tile store mapping");
  static_assert(BM >= 16 * XI, "surplus row groups map onto distinct real ones");
  static_assert(NW % 2 == 0, "swizzle term of a lane must not depend on the row group");
  // X parts of the next channel chunk are issued at the first T - NS + 1 taps of a chunk, XI
  // instructions per wave each; the halo must fit in those.
  static bool supports(const FpropParams& p) {
    const ConvGeom& g = p.cg;
    const int T = g.R * g.S;
    if (g.stride_h != 1 || g.stride_w != 1 || g.P != g.H || g.Q != g.Wi) return false;
    if (2 * g.pad_h != g.R - 1 || 2 * g.pad_w != g.S - 1) return false;
    if (g.C % (64 * KG) != 0 || T > 32 || T < NS) return false;
    const int hb8 = halo_rows(g);
    return (T - NS + 1) * XI * NW * 8 >= hb8;
  }
  static __host__ __device__ int halo_rows(const ConvGeom& g) {  // LDS rows (pixels) of one halo buffer, multiple of 8
    const int hb = BM + 2 * (g.pad_h * g.Wi + g.pad_w);
    return (hb + 7) / 8 * 8;
  }
  // Rows from one halo buffer to the next: with two buffers the second starts on a 16-row boundary
  // so that a row's swizzle term is the same in both.
  static __host__ __device__ int buffer_stride(const ConvGeom& g) {
    return g.C > 64 * KG ? (halo_rows(g) + 15) / 16 * 16 : halo_rows(g);
  }
  static __host__ __device__ int group_halves(const ConvGeom& g) {  // LDS of one k-group: halo buffers, zero row, weight stages
    const int nbuf = g.C > 64 * KG ? 2 : 1;
    return (nbuf * buffer_stride(g) + 1) * 64 + NS * BN * 64;
  }
  static int lds_bytes(const FpropParams& p) {
    const int pipe = KG * group_halves(p.cg) * 2;
    const int ctile = BM * BN * 2, reduce = (KG - 1) * BM * BN * 4;
    return pipe > ctile ? (pipe > reduce ? pipe : reduce) : (ctile > reduce ? ctile : reduce);
  }
};

// What the main loop needs to know about the problem (the single convolution and the fused pair share it).
struct HaloArgs {
  const half_t* X;  // NHWC input
  const half_t* W;  // row 0 of this tile's weights, [w_rows][K] with leading dimension ldw
  int w_rows;       // valid weight rows (output channels) from W on
  int M, K, ldw;    // output pixels (= input pixels), R*S*C, weight leading dimension
  ConvGeom cg;
  int m0;           // first output pixel of the tile
};

// Prologue and main loop: on return acc holds this k-group's partial sums of the BM x BN tile and
// every load has landed.  `lds` is the workgroup's dynamic LDS; k-group kg uses
// [kg * group_halves, (kg + 1) * group_halves).
template <int BM, int BN, int WAVES_M, int WAVES_N, int NS, int XI, int KG>
__device__ __forceinline__ void conv_halo_mainloop(const HaloArgs& h, half_t* lds,
                                                   floatx16 (&acc)[BN / WAVES_N / 32][BM / WAVES_M / 32]) {
  using T_ = ConvHaloTraits<BM, BN, WAVES_M, WAVES_N, NS, XI, KG>;
  constexpr int BK = 64, NW = T_::NW, WTM = T_::WTM, WTN = T_::WTN, FM = T_::FM, FN = T_::FN, KS = 4;
  using WL = DmaTileLoader<BN, BK, NW, 0>;
  static_assert(NS >= 2 && NS <= 4, "the wait selection below handles up to two issue points in flight");
  static_assert((NS - 1) * (WL::NI + XI) < 64, "vmcnt range");

  const ConvGeom& cg = h.cg;
  const int taps = cg.R * cg.S;
  const int nchunks_all = cg.C / 64;      // 64-channel chunks of the input
  const int nchunks = nchunks_all / KG;   // ... of which this k-group takes kg, kg + KG, ...
  const int halo = cg.pad_h * cg.Wi + cg.pad_w;
  const int hb8 = (BM + 2 * halo + 7) / 8 * 8;  // rows of one halo buffer
  const int bstride = T_::buffer_stride(cg);     // rows between the two buffers
  const int nbuf = nchunks > 1 ? 2 : 1;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = wave_all / NW, wave = wave_all - kg * NW;
  half_t* Xh = lds + kg * T_::group_halves(cg);  // [nbuf][hb8 * 64], then one row of zeros
  const int zero_row = nbuf * bstride;     // what a lane reads for a filter tap outside the image
  half_t* Ws = Xh + (zero_row + 1) * 64;   // [NS][BN * 64]

  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int g = lane >> 5, l32 = lane & 31;
  const int m0 = h.m0;
  const int total_px = h.M;  // stride 1, same padding: output pixels == input pixels
  const int S_items = nchunks * taps;
  const int xparts = (hb8 / 8 + XI * NW - 1) / (XI * NW);  // issue points that carry halo loads (<= taps - NS + 1)

  // ---- loaders ---------------------------------------------------------------------------------
  WL wl;
  {
    const int64_t rem = ((int64_t)(h.w_rows - 1) * h.ldw + h.K) * 2;
    wl.init(h.W, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff), h.ldw, h.w_rows, h.K, cg, 0, 0, wave, lane);
  }
  const __amdgpu_buffer_rsrc_t xrsrc = make_rsrc(h.X, (unsigned)((int64_t)total_px * cg.C * 2));
  const int lrow = lane >> 3;
  const int xlc = (lane & 7) ^ dma_swizzle<BK>(wave * 8 + lrow);  // logical chunk this lane fetches
  // X part `part` (0 .. xparts-1) of channel chunk `chunk` into halo buffer `buf`: XI instructions,
  // each filling 8 LDS rows per wave.  Row groups past the halo (only in the last part) re-load the
  // last group: the instruction count of a part must not depend on the wave.
  auto issue_x_part = [&](int chunk, int part, int buf) {
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      int group = (part * XI + i) * NW + wave;  // group of 8 LDS rows
      if (group * 8 >= hb8) {  // the highest real groups of this wave's parity: same swizzle term
        const int top = hb8 / 8 - 1;
        group = top - ((top ^ wave) & 1) - 2 * i;
      }
      const int row = group * 8 + lrow;
      const int px = m0 - halo + row;
      const bool ok = px >= 0 && px < total_px;
      const unsigned off = ok ? (unsigned)(px * cg.C + (kg + chunk * KG) * 64 + xlc * 8) * 2u : kInvalidOffset;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, BOLT_LDS_PTR(Xh + buf * bstride * 64 + group * 512), 16, off, 0,
                                               0, 0);
    }
  };
  // Issue point at the end of item (chunk ac, tap at_): first, at the first xparts taps of a chunk,
  // one part of the NEXT chunk's halo into the buffer the previous chunk no longer reads; then the W
  // tile of item u into `stage`.  The order matters: an X part is older than the first W tile that is
  // waited for at the chunk boundary, so that wait covers it (vector memory operations retire in
  // issue order).  Returns whether X loads were issued: the waits count instructions.
  int w_tap = 0, w_chunk = 0;  // (tap, chunk) of the next W tile to fetch; its k-tile is tap * nchunks + chunk
  auto issue_w = [&](int stage) {
    wl.issue(w_tap * nchunks_all + kg + w_chunk * KG, Ws + stage * BN * 64, cg);
    if (++w_tap == taps) {
      w_tap = 0;
      ++w_chunk;
    }
  };
  auto issue_point = [&](int ac, int at_, int stage) -> bool {
    const bool with_x = at_ < xparts && ac + 1 < nchunks;  // wave-uniform
    if (with_x) issue_x_part(ac + 1, at_, (ac + 1) & 1);
    issue_w(stage);
    return with_x;
  };
  // Waits until at most the loads of the `NS - 2` most recent issue points are in flight; xhist bit k
  // says whether the issue point k+1 items ago carried X loads.
  auto wait_and_barrier = [&](unsigned xhist) {
    if constexpr (NS == 2) {
      barrier_after_reads_and_loads<0>();
    } else {
      const int j = __builtin_popcount(xhist & ((1u << (NS - 2)) - 1u));
      if (j == 0) barrier_after_reads_and_loads<(NS - 2) * WL::NI>();
      else if (NS == 3 || j == 1) barrier_after_reads_and_loads<(NS - 2) * WL::NI + XI>();
      else barrier_after_reads_and_loads<(NS - 2) * WL::NI + 2 * XI>();
    }
  };

  // ---- per-lane validity of every tap for the FM output pixels this lane feeds -------------------
  unsigned tapmask[FM];
#pragma unroll
  for (int b = 0; b < FM; ++b) {
    const int m = m0 + wm * WTM + b * 32 + l32;
    unsigned mask = 0;
    if (m < h.M) {
      const int hw = cg.H * cg.Wi;
      const int rem = m - (m / hw) * hw;
      const int op = rem / cg.Wi, oq = rem - op * cg.Wi;
      const int ih0 = op - cg.pad_h, iw0 = oq - cg.pad_w;
      const int r_lo = ih0 < 0 ? -ih0 : 0, r_hi = cg.H - ih0 < cg.R ? cg.H - ih0 : cg.R;
      const int s_lo = iw0 < 0 ? -iw0 : 0, s_hi = cg.Wi - iw0 < cg.S ? cg.Wi - iw0 : cg.S;
      if (s_hi > s_lo) {
        const unsigned rowbits = ((s_hi >= 32 ? 0u : 1u << s_hi) - 1u) & ~((1u << s_lo) - 1u);
        for (int r = r_lo; r < r_hi; ++r) mask |= rowbits << (r * cg.S);
      }
    }
    tapmask[b] = mask;
  }
  if (wave == 0 && lane < 8) *(half8*)(Xh + zero_row * 64 + lane * 8) = half8{0, 0, 0, 0, 0, 0, 0, 0};

#pragma unroll
  for (int a = 0; a < FN; ++a)
#pragma unroll
    for (int b = 0; b < FM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  // Fragments are double-buffered in registers in groups of G k-steps, as in fprop_dma_kernel.hpp.
  constexpr int G = FM * FN >= BOLT_FRAG_DEPTH ? 1 : (BOLT_FRAG_DEPTH / (FM * FN) < KS ? BOLT_FRAG_DEPTH / (FM * FN) : KS);
  constexpr int NG = KS / G;
  static_assert(KS % G == 0 && (NG == 1 || NG % 2 == 0), "register sets alternate per group");
  half8 xf[2][G][FM], wf[2][G][FN];
  // LDS row (over both halo buffers) each of this lane's FM fragments reads for the item being read:
  // its own pixel shifted by the tap, or the row of zeros where the tap falls outside the image.
  int xrow[FM];
  auto set_rows = [&](int buf, int toff, int tap) {
#pragma unroll
    for (int b = 0; b < FM; ++b)
      xrow[b] = (tapmask[b] >> tap) & 1u ? buf * bstride + wm * WTM + b * 32 + l32 + toff : zero_row;
  };
  auto read_group = [&](int stage, int grp, half8 (&x)[G][FM], half8 (&w)[G][FN]) {
    const half_t* ws = Ws + stage * BN * 64;
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const int chunk = (grp * G + k) * 2 + g;
#pragma unroll
      for (int b = 0; b < FM; ++b) x[k][b] = *(const half8*)(Xh + dma_chunk_offset<BK>(xrow[b], chunk));
#pragma unroll
      for (int a = 0; a < FN; ++a) w[k][a] = *(const half8*)(ws + dma_chunk_offset<BK>(wn * WTN + a * 32 + l32, chunk));
    }
  };
  auto mfma_group = [&](const half8 (&x)[G][FM], const half8 (&w)[G][FN]) {
#pragma unroll
    for (int k = 0; k < G; ++k)
#pragma unroll
      for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b) acc[a][b] = mfma_32x32x16(w[k][a], x[k][b], acc[a][b]);
  };

  // ---- prologue: all of chunk 0's halo, then the first NS items ---------------------------------------
  // (S_items >= taps >= NS is a condition of support)
  for (int part = 0; part < xparts; ++part) issue_x_part(0, part, 0);
#pragma unroll
  for (int s = 0; s < NS; ++s) issue_w(s);
  barrier_after_reads_and_loads<(NS - 1) * WL::NI>();  // lgkmcnt 0 too: the zero row's ds_write is done
  set_rows(0, 0, 0);
  read_group(0, 0, xf[0], wf[0]);

  int stage = 0;
  int chunk = 0, tap = 0, fr = 0, fs = 0;  // item in progress: channel chunk, filter tap = fr * S + fs
  unsigned xhist = 0;
  auto tile_body = [&](int s, auto par) {
    constexpr int P = decltype(par)::value;
    auto group = [&](auto jc) {
      constexpr int j = decltype(jc)::value;
      constexpr int cur = (P + j) & 1, nxt = cur ^ 1;
      __builtin_amdgcn_sched_barrier(0);
      if (j + 1 < NG) {
        read_group(stage, j + 1, xf[nxt], wf[nxt]);
      } else {
        // end of item s: item s+1's W tile (and, being older, every X part it may need) has landed
        if (S_items - 2 - s >= NS - 2) wait_and_barrier(xhist);
        else barrier_after_reads_and_loads<0>();
        bool with_x = false;
        if (s + NS < S_items) with_x = issue_point(chunk, tap, stage);
        xhist = (xhist << 1) | (with_x ? 1u : 0u);
        stage = stage + 1 == NS ? 0 : stage + 1;
        ++tap;
        if (++fs == cg.S) {
          fs = 0;
          ++fr;
        }
        if (tap == taps) {
          tap = fr = fs = 0;
          ++chunk;
        }
        set_rows(chunk < nchunks ? chunk & 1 : 0, fr * cg.Wi + fs, tap);  // (after the last item: never used)
        read_group(stage, 0, xf[nxt], wf[nxt]);
      }
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(xf[cur], wf[cur]);
    };
    group(std::integral_constant<int, 0>{});
    if constexpr (NG > 1) group(std::integral_constant<int, 1>{});
    if constexpr (NG > 2) {
      group(std::integral_constant<int, 2>{});
      group(std::integral_constant<int, 3>{});
    }
  };
  if constexpr (NG % 2 == 0) {
    for (int s = 0; s < S_items; ++s) tile_body(s, std::integral_constant<int, 0>{});
  } else {
    int s = 0;
    for (; s + 1 < S_items; s += 2) {
      tile_body(s, std::integral_constant<int, 0>{});
      tile_body(s + 1, std::integral_constant<int, 1>{});
    }
    if (s < S_items) tile_body(s, std::integral_constant<int, 0>{});
  }

}

template <int BM, int BN, int WAVES_M, int WAVES_N, int NS, int XI, int KG = 1, bool RES = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * KG) void conv_halo_kernel(const FpropParams p) {
  using T_ = ConvHaloTraits<BM, BN, WAVES_M, WAVES_N, NS, XI, KG>;
  constexpr int NW = T_::NW, WTM = T_::WTM, WTN = T_::WTN, FM = T_::FM, FN = T_::FN;
  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = wave_all / NW, wave = wave_all - kg * NW;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int g = lane >> 5, l32 = lane & 31;
  int tm, tn;
  tile_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, p.swizzle, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  floatx16 acc[FN][FM];
  {
    const HaloArgs h{p.X, p.W + (int64_t)n0 * p.ldw, p.N - n0, p.M, p.K, p.ldw, p.cg, m0};
    conv_halo_mainloop<BM, BN, WAVES_M, WAVES_N, NS, XI, KG>(h, lds, acc);
  }

  // ---- k-groups: sum the accumulators through LDS, group 0 carries on ------------------------------
  if constexpr (KG > 1) {
    float* red = reinterpret_cast<float*>(lds);  // [KG-1][NW][FN*FM*16][64 lanes]
    barrier_after_lds_writes();                  // every wave has finished reading halo and weight stages
    if (kg > 0) {
      float* mine = red + ((kg - 1) * NW + wave) * (FN * FM * 16 * 64) + lane;
#pragma unroll
      for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) mine[((a * FM + b) * 16 + r) * 64] = acc[a][b][r];
    }
    barrier_after_lds_writes();
    if (kg == 0) {
      for (int o = 0; o < KG - 1; ++o) {  // fixed order: the result does not depend on timing
        const float* theirs = red + (o * NW + wave) * (FN * FM * 16 * 64) + lane;
#pragma unroll
        for (int a = 0; a < FN; ++a)
#pragma unroll
          for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] += theirs[((a * FM + b) * 16 + r) * 64];
      }
    }
  }

  // ---- epilogue: registers -> FP16 C tile in LDS -> coalesced stores (fprop_dma_kernel.hpp) ----------------
  fprop_tile_out<RES, BM, BN, WTM, WTN, T_::STORE_THREADS, T_::ROWS_PER_PASS>(lds, acc, p, m0, n0, wm, wn, kg == 0, tid);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int NS, int XI, int KG = 1>
hipError_t launch_conv_halo(const FpropParams& p, hipStream_t stream) {
  using T_ = ConvHaloTraits<BM, BN, WAVES_M, WAVES_N, NS, XI, KG>;
  // the residual epilogue is a kernel of its own (fprop_tile_out in fprop_dma_kernel.hpp)
  auto kern = p.res ? conv_halo_kernel<BM, BN, WAVES_M, WAVES_N, NS, XI, KG, true>
                    : conv_halo_kernel<BM, BN, WAVES_M, WAVES_N, NS, XI, KG, false>;
  static LdsOptIn opt_in[2];
  if (hipError_t e = opt_in[p.res ? 1 : 0].ensure((const void*)kern, 160 * 1024); e != hipSuccess) return e;
  dim3 grid(p.tiles_m * p.tiles_n, 1, 1);
  hipLaunchKernelGGL(kern, grid, dim3(T_::NT), T_::lds_bytes(p), stream, p);
  return hipGetLastError();
}

#define BOLT_CONV_HALO_INSTANCE(BM, BN, WM, WN, NS, XI)                                                 \
  {                                                                                                     \
    "halo_" #BM "x" #BN "_w" #WM "x" #WN "_s" #NS "_x" #XI, BM, BN, 64, WM, WN, 1, 0, NS, 0,              \
        &bolt::launch_conv_halo<BM, BN, WM, WN, NS, XI>,                                                 \
        &bolt::ConvHaloTraits<BM, BN, WM, WN, NS, XI>::supports,                                         \
        &bolt::ConvHaloTraits<BM, BN, WM, WN, NS, XI>::lds_bytes                                         \
  }

#define BOLT_CONV_HALO_KG_INSTANCE(BM, BN, WM, WN, NS, XI, KG)                                          \
  {                                                                                                     \
    "halo_" #BM "x" #BN "_w" #WM "x" #WN "_s" #NS "_x" #XI "_kg" #KG, BM, BN, 64, WM, WN, 1, 0, NS, 0,    \
        &bolt::launch_conv_halo<BM, BN, WM, WN, NS, XI, KG>,                                             \
        &bolt::ConvHaloTraits<BM, BN, WM, WN, NS, XI, KG>::supports,                                     \
        &bolt::ConvHaloTraits<BM, BN, WM, WN, NS, XI, KG>::lds_bytes, KG                                 \
  }

}  // namespace bolt
