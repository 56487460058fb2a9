// First-layer convolution: few input channels (C <= 4, e.g. the 3 colour planes of an image), read where the model
// keeps them - NHWC with the channels NOT padded, or NCHW - with the layout transformation and the channel padding of
// Section 3.2.3 folded into the kernel's loader instead of running as passes of their own (the paper puts the
// transformation into the generated code of the first layer and pads to alignment 8 because unaligned vector
// accesses are slow; here global memory is read in aligned dwords whatever the run's start, and the 2-byte
// granularity lives in register shifts and LDS writes).
//
// One workgroup (4 waves) computes 128 consecutive output pixels of ONE output row for 64 output channels:
//   * staging: the R input rows that row needs are copied into LDS as R rows of interleaved halves,
//     row[r][j * C + c] = x[img][ih0 + r][iw_lo + j][c], zero outside the image, over the columns the tile's windows
//     touch.  In NHWC a row is one contiguous run in global memory (a straight copy, 16 bytes per LDS write); in
//     NCHW it is C runs, interleaved by 2-byte LDS writes.
//   * the reduction index is ordered (r, s, c) as in the weights, with the S * C halves of a filter row padded to
//     NF = ceil(S * C / 8) fragments of 8: fragment f = (r, fr) of output pixel q is the 8 consecutive halves at
//     row[r][q * stride_w * C + 8 * fr] - aligned 4-byte LDS reads when stride_w is 2 - and the same 8 halves
//     w[k][r][8 * fr ..] of every output channel's weights.  What a fragment reads past S * C belongs to the
//     neighbouring pixels; a mask zeroes it (its weights are zero as well, but 0 * inf is not 0).
//   * the weights are the A operand of v_mfma_f32_16x16x32_f16 (T k-steps x 4 blocks of 16 channels): at kernel
//     start the workgroup writes them to LDS in fragment order, where they stay; a lane reads its fragments of a
//     k-step with four conflict-free 16-byte reads.  Row i of block b is output channel
//     32 * (b / 2) + 8 * (i / 4) + 4 * (b % 2) + i % 4, so that a lane ends up with two runs of 8 consecutive
//     channels of its pixel (two 16-byte stores) and the four lanes of a pixel write 64 contiguous bytes per store.
// Workgroups are persistent over the output rows (grid = three per compute unit, what the registers allow), which amortises the weight set-up;
// the global loads of a workgroup's next tile are in flight while it multiplies and stores the current one.
// Vector ALU work is what bounds this kernel (a 64-lane instruction takes 4 cycles): index arithmetic is per
// 8-half item, never per half.
#pragma once
#include "fprop_dma_kernel.hpp"

namespace bolt {

template <int T, int SW>
struct ConvSmallCTraits {
  static constexpr int NT = 256, QT = 128, BN = 64;
  static constexpr int FRAGS = 4 * T;               // fragments (r, fr) a k loop of T steps covers
  static constexpr int W_HALVES = FRAGS * 64 * 8;   // weights in fragment order
  static constexpr int M_HALVES = FRAGS * 8;        // one mask per fragment
  static constexpr int IN_CAP = 6656;               // halves of staged input rows
  static constexpr int NI = (IN_CAP / 8 + FRAGS + 255) / 256;  // staging items per thread
  static constexpr int LDS_BYTES = (W_HALVES + M_HALVES + IN_CAP) * 2;
  static __host__ __device__ int nf(const ConvGeom& g) { return (g.S * g.C + 7) / 8; }
  // halves of a staged row that the tile's fragments read, rounded up to whole items
  static __host__ __device__ int xlen(const ConvGeom& g) { return ((QT - 1) * SW * g.C + 8 * nf(g) + 7) & ~7; }
  // row stride: room for the last NCHW item of every channel (8 columns past the last one needed)
  static __host__ __device__ int rstride(const ConvGeom& g) { return xlen(g) + 8 * g.C; }
  static bool supports(const FpropParams& p) {
    const ConvGeom& g = p.cg;
    return g.C <= 4 && g.stride_w == SW && g.R * nf(g) <= FRAGS && g.R * rstride(g) <= IN_CAP;
  }
  static int lds_bytes(const FpropParams&) { return LDS_BYTES; }
};

// x_nchw (FpropParams::x_nchw): the input is [N][C][H][W] instead of [N][H][W][C]
template <int T, int SW>
__global__ __launch_bounds__(256, 3) void conv_smallc_kernel(const FpropParams p) {
  using Tr = ConvSmallCTraits<T, SW>;
  constexpr int QT = Tr::QT, NI = Tr::NI;
  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* const wfrag = lds;                               // the weights in fragment order, for the whole kernel
  half_t* const mtab = lds + Tr::W_HALVES;                 // fragment masks
  half_t* const rows = lds + Tr::W_HALVES + Tr::M_HALVES;  // the staged input rows of the current tile

  const ConvGeom& cg = p.cg;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = lane >> 4, l16 = lane & 15;  // k-group (fragment within a k-step) and pixel / channel row of this lane
  const int n0 = blockIdx.y * Tr::BN;
  const int SC = cg.S * cg.C;
  const int NF = Tr::nf(cg), nfrag = cg.R * NF, XLEN = Tr::xlen(cg), RS = Tr::rstride(cg);
  // small exact divisions: v / d = (int)((v + 0.5f) * (1 / d)) for v < 2^16, d < 2^10
  auto fdiv = [](int v, float rcp) { return (int)(((float)v + 0.5f) * rcp); };
  const float rcp_nf = 1.0f / (float)NF, rcp_c = 1.0f / (float)cg.C;

  const int tiles_q = (cg.Q + QT - 1) / QT;
  const int total = (p.M / cg.Q) * tiles_q;  // output rows of the whole batch x column tiles

  // ---- staging --------------------------------------------------------------------------------------------------
  // What a tile needs lies in global memory as contiguous runs: one per input row in NHWC (XLEN halves), one per
  // (input row, channel) in NCHW (XLEN / C columns).  A work item is 8 consecutive halves of a run; a run starts at
  // any 2-byte boundary, so the item is fetched as the 5 ALIGNED dwords that cover it (2-byte global loads are served
  // at a fraction of the rate) and shifted into place in registers.  Item w belongs to thread w % 256.
  //   fetch:   global memory -> 5 registers per item, all loads together; a dword outside the tensor or of a row
  //            outside the image gets an offset beyond the buffer and reads as zero.
  //   scatter: one tile later (the loads of tile i + 1 fly while tile i is multiplied and stored): columns outside
  //            the image are zeroed, then NHWC: one 16-byte LDS write; NCHW: 8 2-byte writes, C halves apart.
  const int ipr = p.x_nchw ? ((XLEN + cg.C - 1) / cg.C + 7) / 8 : XLEN / 8;  // items per run
  const int nseg = p.x_nchw ? cg.R * cg.C : cg.R;
  const float rcp_ipr = 1.0f / (float)ipr;
  const int stride_r = p.x_nchw ? cg.Wi : cg.Wi * cg.C, stride_c = p.x_nchw ? cg.H * cg.Wi : 0;
  const int unit = p.x_nchw ? 1 : cg.C;  // halves per column inside a run
  // (rounded up to whole dwords: the last element of a tensor with an odd element count shares its dword with two
  // bytes that still lie inside the caller's allocation - x is 16-byte aligned and allocations are multiples of 4)
  const __amdgpu_buffer_rsrc_t xrsrc = make_rsrc(p.X, ((unsigned)((int64_t)(p.M / (cg.P * cg.Q)) * cg.H * cg.Wi * cg.C * 2) + 3u) & ~3u);
  unsigned v[NI][5];
  struct TileAt { int orow, q0, iw_lo, ih0, base; };
  auto locate = [&](int tile) {
    TileAt t;
    const int qt = tile % tiles_q;
    t.orow = tile / tiles_q;  // img * P + p
    const int img = t.orow / cg.P, op = t.orow - img * cg.P;
    t.q0 = qt * QT;
    t.iw_lo = t.q0 * SW - cg.pad_w;
    t.ih0 = op * cg.stride_h - cg.pad_h;
    t.base = p.x_nchw ? (img * cg.C * cg.H + t.ih0) * cg.Wi + t.iw_lo : ((img * cg.H + t.ih0) * cg.Wi + t.iw_lo) * cg.C;
    return t;
  };
  // What does not depend on the tile is worked out once per item i of this thread and kept in two registers:
  //   rel[i]: first half of the item relative to the tile's first half in the tensor (TileAt::base);
  //   dsx[i]: LDS half index of its destination | filter row r << 16 | first half inside the run x0 << 21, or -1 for
  //           an item past the last run.
  int rel[NI], dsx[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int w = tid + 256 * i, seg = fdiv(w, rcp_ipr), x0 = (w - seg * ipr) * 8;
    const int r = p.x_nchw ? fdiv(seg, rcp_c) : seg, c = p.x_nchw ? seg - r * cg.C : 0;
    rel[i] = r * stride_r + c * stride_c + x0;
    dsx[i] = seg < nseg ? (r * RS + (p.x_nchw ? x0 * cg.C + c : x0)) | (r << 16) | (x0 << 21) : -1;
  }
  auto fetch = [&](const TileAt& t) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int gi = t.base + rel[i];
      const int a4 = (gi >> 1) * 4;  // byte offset of the dword that holds half gi (floor)
      const bool ok = (dsx[i] >= 0) & ((unsigned)(t.ih0 + ((dsx[i] >> 16) & 31)) < (unsigned)cg.H);
      // One 16-byte load and one 4-byte load per item: consecutive lanes hold consecutive items, so the wide loads of
      // a wave cover one contiguous kilobyte (five strided dword loads would keep the address path five times as
      // busy).  An item that starts in front of the tensor (the first rows of the first image, left of the image)
      // takes single dwords instead: those in front hold only columns that scatter() zeroes, any address does.
      if (a4 >= 0) {
        const auto q4 = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, ok ? (unsigned)a4 : kInvalidOffset, 0, 0);
        v[i][0] = q4[0]; v[i][1] = q4[1]; v[i][2] = q4[2]; v[i][3] = q4[3];
        v[i][4] = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, ok ? (unsigned)a4 + 16u : kInvalidOffset, 0, 0);
      } else {
#pragma unroll
        for (int n = 0; n < 5; ++n) {
          const int off = a4 + 4 * n;
          v[i][n] = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, ok ? (unsigned)(off > 0 ? off : 0) : kInvalidOffset, 0, 0);
        }
      }
    }
  };
  auto scatter = [&](const TileAt& t) {
    // columns [lo, hi) of a run, in halves of the run, lie inside the image
    const int lo = (t.iw_lo < 0 ? -t.iw_lo : 0) * unit, hi = (cg.Wi - t.iw_lo) * unit;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const unsigned sh = (unsigned)((t.base + rel[i]) & 1) * 16u;
      unsigned o[4];
#pragma unroll
      for (int n = 0; n < 4; ++n) o[n] = __builtin_amdgcn_alignbit(v[i][n + 1], v[i][n], sh);
      const int x0 = dsx[i] >> 21;
      if ((x0 < lo) | (x0 + 8 > hi)) {  // an item on the image's edge: zero the halves outside
#pragma unroll
        for (int n = 0; n < 4; ++n) {
          const int xa = x0 + 2 * n;
          o[n] &= (((xa >= lo) & (xa < hi)) ? 0x0000ffffu : 0u) | (((xa + 1 >= lo) & (xa + 1 < hi)) ? 0xffff0000u : 0u);
        }
      }
      if (dsx[i] >= 0) {
        half_t* dst = rows + (dsx[i] & 0xffff);
        if (!p.x_nchw) {
          *(uint4*)dst = uint4{o[0], o[1], o[2], o[3]};
        } else {
#pragma unroll
          for (int k = 0; k < 8; ++k) ((unsigned short*)dst)[k * cg.C] = (unsigned short)(k & 1 ? o[k >> 1] >> 16 : o[k >> 1] & 0xffffu);
        }
      }
    }
  };
  // This workgroup's tiles: first, first + step, ... below end.  Consecutive workgroup ids land on consecutive XCDs
  // (8, each with an L2 of its own), and neighbouring output rows share R - stride input rows: every XCD takes one
  // contiguous eighth of the tiles, so that the rows its workgroups have in flight are neighbours in one L2.
  int first = blockIdx.x, step = gridDim.x, end = total;
  if ((gridDim.x & 7) == 0 && total >= (int)gridDim.x) {
    const int band = (total + 7) >> 3, xcd = blockIdx.x & 7;
    first = xcd * band + (int)(blockIdx.x >> 3);
    step = gridDim.x >> 3;
    end = (xcd + 1) * band < total ? (xcd + 1) * band : total;
  }
  TileAt cur = locate(first < end ? first : 0);
  if (first < end) fetch(cur);

  // ---- weights and masks: global [K][R][S][C] -> LDS in fragment order ---------------------------------------------
  // Four threads per output channel, each every fourth fragment (r, fr) of it: the 8 halves w[ch][r][8 * fr ..] are
  // contiguous, fetched as the 5 aligned dwords that cover them; halves past the filter row, fragments past the last
  // one and channels past K become zero.  The threads of channel 0 also write the masks.
  {
    const int chl = tid >> 2, sub = tid & 3, ch = n0 + chl;
    const __amdgpu_buffer_rsrc_t wrsrc = make_rsrc(p.W, (unsigned)((int64_t)p.N * p.ldw * 2));
    const int blk = 2 * (chl >> 5) + ((chl >> 2) & 1), row = 4 * ((chl >> 3) & 3) + (chl & 3);
    unsigned wv[T][5];
#pragma unroll
    for (int i = 0; i < T; ++i) {
      const int f = sub + 4 * i, r = fdiv(f, rcp_nf), fr = f - r * NF;
      const int h0 = ch * p.ldw + r * SC + 8 * fr, a = h0 >> 1;
      const bool ok = (f < nfrag) & (ch < p.N);
      const auto q4 = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, ok ? (unsigned)a * 4u : kInvalidOffset, 0, 0);
      wv[i][0] = q4[0]; wv[i][1] = q4[1]; wv[i][2] = q4[2]; wv[i][3] = q4[3];
      wv[i][4] = __builtin_amdgcn_raw_buffer_load_b32(wrsrc, ok ? (unsigned)a * 4u + 16u : kInvalidOffset, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < T; ++i) {
      const int f = sub + 4 * i, r = fdiv(f, rcp_nf), fr = f - r * NF;
      const int h0 = ch * p.ldw + r * SC + 8 * fr;
      const unsigned sh = (unsigned)(h0 & 1) * 16u;
      const int nvalid = f < nfrag ? SC - 8 * fr : 0;  // halves of this fragment inside the filter row
      unsigned o[4], m[4];
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        m[n] = (2 * n < nvalid ? 0x0000ffffu : 0u) | (2 * n + 1 < nvalid ? 0xffff0000u : 0u);
        o[n] = __builtin_amdgcn_alignbit(wv[i][n + 1], wv[i][n], sh) & m[n];
      }
      const int t = f >> 2, grp = f & 3;
      *(uint4*)(wfrag + ((t * 4 + blk) * 64 + grp * 16 + row) * 8) = uint4{o[0], o[1], o[2], o[3]};
      if (chl == 0) *(uint4*)(mtab + f * 8) = uint4{m[0], m[1], m[2], m[3]};
    }
  }
  // (the barrier that publishes the first tile's rows publishes the weights and masks too)

  // this lane's fragment of k-step t: where it starts in the staged rows, relative to the pixel's first half
  int fbase[T];
#pragma unroll
  for (int t = 0; t < T; ++t) {
    const int f = t * 4 + kg, r = fdiv(f, rcp_nf), fr = f - r * NF;
    fbase[t] = f < nfrag ? r * RS + 8 * fr : 0;
  }
  const int qstep = SW * cg.C;  // halves from a pixel to the next

  // this lane's bias: channels n0 + 32 * hb + 8 * kg + [0, 8), hb = 0, 1 (zero beyond K and without a bias)
  half8 bias_h[2];
#pragma unroll
  for (int hb = 0; hb < 2; ++hb) {
    const int n = n0 + 32 * hb + 8 * kg;
    const half8 got = *(const half8*)(p.bias + (n < p.N ? n : 0) * p.bias_on);
    bias_h[hb] = (n < p.N && p.bias_on) ? got : half8{0, 0, 0, 0, 0, 0, 0, 0};
  }

  for (int tile = first; tile < end; tile += step) {
    scatter(cur);
    __syncthreads();
    const int orow = cur.orow, q0 = cur.q0;
    if (tile + step < end) {
      cur = locate(tile + step);
      fetch(cur);
    }

    // ---- k loop ----------------------------------------------------------------------------------------------------
    floatx4 acc[2][4];
#pragma unroll
    for (int pb = 0; pb < 2; ++pb)
#pragma unroll
      for (int b = 0; b < 4; ++b) acc[pb][b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < T; ++t) {
      // (k-steps are kept apart: hoisting all weight reads to the front would need 16 * T registers)
      __builtin_amdgcn_sched_barrier(0);
      half8 wf[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) wf[b] = *(const half8*)(wfrag + ((t * 4 + b) * 64 + lane) * 8);
      const uint4 mk = *(const uint4*)(mtab + (t * 4 + kg) * 8);
#pragma unroll
      for (int pb = 0; pb < 2; ++pb) {
        const half_t* src_h = rows + fbase[t] + (wave * 32 + pb * 16 + l16) * qstep;
        union { unsigned u[4]; half8 h; } xf;
        if constexpr (SW == 2) {
          const unsigned* src = (const unsigned*)src_h;
#pragma unroll
          for (int d = 0; d < 4; ++d) xf.u[d] = src[d];
        } else {
          const unsigned short* src = (const unsigned short*)src_h;
#pragma unroll
          for (int d = 0; d < 4; ++d) xf.u[d] = (unsigned)src[2 * d] | ((unsigned)src[2 * d + 1] << 16);
        }
        xf.u[0] &= mk.x; xf.u[1] &= mk.y; xf.u[2] &= mk.z; xf.u[3] &= mk.w;
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[pb][b] = mfma_16x16x32(wf[b], xf.h, acc[pb][b]);
      }
    }

    // ---- epilogue (Section 3.1, patterns (i)-(iii)): this lane holds channels n0 + 8 * kg + [0, 8) and
    // n0 + 32 + 8 * kg + [0, 8) of its two pixels; one store instruction of the wave writes the first or the second 64
    // bytes of 16 pixels' channel rows
    auto store_tile = [&](auto slow) {
#pragma unroll
      for (int pb = 0; pb < 2; ++pb) {
        const int q = q0 + wave * 32 + pb * 16 + l16;
        if (q >= cg.Q) continue;
        half_t* yrow = p.Y + ((int64_t)orow * cg.Q + q) * p.ldy;
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
          const int n = n0 + 32 * hb + 8 * kg;
          half8 o;
#pragma unroll
          for (int b2 = 0; b2 < 2; ++b2) {
            floatx4 u;
#pragma unroll
            for (int e = 0; e < 4; ++e) u[e] = p.alpha * acc[pb][2 * hb + b2][e] + p.beta * (float)bias_h[hb][4 * b2 + e];
            if constexpr (decltype(slow)::value) {
              u = apply_act_slow4(u, p.act);
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const float r = u[e] > 0.f ? u[e] : 0.f;
                u[e] = p.act == ACT_RELU ? r : u[e];
              }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) o[4 * b2 + e] = (half_t)u[e];
          }
          if (n < p.N) {
            if (!p.y_nchw) {
              __builtin_nontemporal_store(o, (half8*)(yrow + n));
            } else {
              // [N][K][P][Q]: 8 channel planes; the 16 lanes of a pixel block write 16 consecutive pixels of each
              const int img = orow / cg.P, op = orow - img * cg.P;
              half_t* y = p.Y + (((int64_t)img * p.N + n) * cg.P + op) * cg.Q + q;
#pragma unroll
              for (int k = 0; k < 8; ++k) y[(int64_t)k * cg.P * cg.Q] = o[k];
            }
          }
        }
      }
    };
    if (p.act > ACT_RELU) store_tile(std::true_type{});
    else store_tile(std::false_type{});
    __syncthreads();  // every wave has read its fragments: the rows may be overwritten
  }
}

template <int T, int SW>
hipError_t launch_conv_smallc(const FpropParams& p, hipStream_t stream) {
  using Tr = ConvSmallCTraits<T, SW>;
  static LdsOptIn opt_in;
  auto kern = conv_smallc_kernel<T, SW>;
  if (hipError_t e = opt_in.ensure((const void*)kern, Tr::LDS_BYTES); e != hipSuccess) return e;
  const int64_t total = (int64_t)(p.M / p.cg.Q) * ((p.cg.Q + Tr::QT - 1) / Tr::QT);
  constexpr int kComputeUnits = 256, kPerCU = 3;
  dim3 grid((unsigned)(total < kComputeUnits * kPerCU ? total : kComputeUnits * kPerCU), (p.N + Tr::BN - 1) / Tr::BN, 1);
  hipLaunchKernelGGL(kern, grid, dim3(Tr::NT), Tr::LDS_BYTES, stream, p);
  return hipGetLastError();
}

// In the instance table: x mode 4 (few channels, any alignment, NHWC or NCHW input), tile = 128 pixels x 64 channels,
// tile K = the 32 of one matrix instruction, no split-K.
#define BOLT_CONV_SMALLC_INSTANCE(T, SW)                                                                  \
  {                                                                                                       \
    "smallc_t" #T "_sw" #SW, 128, 64, 32, 4, 1, 4, 0, 1, bolt::ConvSmallCTraits<T, SW>::LDS_BYTES,         \
        &bolt::launch_conv_smallc<T, SW>, &bolt::ConvSmallCTraits<T, SW>::supports,                        \
        &bolt::ConvSmallCTraits<T, SW>::lds_bytes, 0, 16, true                                            \
  }

}  // namespace bolt
