// First-layer convolution: few input channels (C <= 4, e.g. the 3 colour planes of an image), read where the model
// keeps them - NHWC with the channels NOT padded, or NCHW - with the layout transformation and the channel padding of
// Section 3.2.3 folded into the kernel's loader instead of running as passes of their own (the paper puts the
// transformation into the generated code of the first layer and pads to alignment 8 because unaligned vector
// accesses are slow; here the unaligned 2-byte accesses touch global memory exactly once per element and everything
// behind them is aligned).
//
// One workgroup (4 waves) computes 128 consecutive output pixels of ONE output row for 64 output channels:
//   * staging: the R input rows that row needs are copied into LDS as R * C "planes", one per (filter row r, channel
//     c): plane[r * C + c][j] = x[img][ih0 + r][iw_lo + j][c], zero outside the image, j over the
//     (128 - 1) * stride_w + 8 columns the tile's windows touch.  Global memory is read in aligned dwords of the
//     contiguous runs either layout offers; the de-interleaving (NHWC) and the 2-byte granularity live in the LDS
//     writes.
//   * the reduction index is ordered (r, c, s) with s padded to 8: k = (r * C + c) * 8 + s.  The B operand of
//     v_mfma_f32_16x16x32_f16 wants 8 consecutive k per lane = 8 consecutive columns of one plane starting at column
//     q * stride_w: an aligned 4-byte read per 2 halves when stride_w is 2, 2-byte reads when it is 1.  Taps s >= S
//     read the neighbours' data; they are masked to zero (their weights are zero as well).
//   * the weights are the A operand (T k-steps x 4 blocks of 16 channels): at kernel start the workgroup scatters
//     w[K][R][S][C] into LDS in fragment order, zero-filled, where they stay; a lane reads its fragments of a k-step
//     with four conflict-free 16-byte reads (holding all of them in registers would leave room for two workgroups per
//     compute unit instead of four).  Row i of block b is output channel 32 * (b / 2) + 8 * (i / 4) + 4 * (b % 2) +
//     i % 4, so that a lane ends up with two runs of 8 consecutive channels of its pixel (two 16-byte stores) and the
//     four lanes of a pixel write 64 contiguous bytes per store instruction.
// Workgroups are persistent over the output rows (grid = four per compute unit), which amortises the weight set-up;
// the global loads of a workgroup's next tile are in flight while it multiplies and stores the current one.
#pragma once
#include "fprop_dma_kernel.hpp"

namespace bolt {

template <int T, int SW>
struct ConvSmallCTraits {
  static constexpr int NT = 256, QT = 128, BN = 64;
  static constexpr int PAIRS = 4 * T;                      // (r, c) planes a k-loop of T steps covers
  static constexpr int COLS = (QT - 1) * SW + 8;           // input columns the windows of a tile touch
  static constexpr int COLS_E = (COLS + 1) & ~1;
  // plane stride: 16 dwords off a multiple of 64, so that the four 16-lane groups of a fragment read (four different
  // planes) fall into four different quarters of the 64 LDS banks
  static constexpr int ROW_HALVES = ((COLS_E / 2 + 47) / 64 * 64 + 16) * 2;
  static constexpr int W_HALVES = T * 4 * 64 * 8;          // weights in fragment order
  static constexpr int IN_HALVES = PAIRS * ROW_HALVES;
  static constexpr int LDS_BYTES = (W_HALVES + IN_HALVES) * 2;
  static_assert(ROW_HALVES >= COLS_E && (ROW_HALVES / 2) % 64 == 16, "plane stride");
  static bool supports(const FpropParams& p) {
    const ConvGeom& g = p.cg;
    return g.C <= 4 && g.R * g.C <= PAIRS && g.S <= 8 && g.stride_w == SW;
  }
  static int lds_bytes(const FpropParams&) { return LDS_BYTES; }
};

// x_nchw (FpropParams::x_nchw): the input is [N][C][H][W] instead of [N][H][W][C]
template <int T, int SW>
__global__ __launch_bounds__(256, 4) void conv_smallc_kernel(const FpropParams p) {
  using Tr = ConvSmallCTraits<T, SW>;
  constexpr int QT = Tr::QT, ROW = Tr::ROW_HALVES, COLS = Tr::COLS;
  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* const wfrag = lds;                   // the weights in fragment order, for the whole kernel
  half_t* const planes = lds + Tr::W_HALVES;   // the staged input rows of the current tile

  const ConvGeom& cg = p.cg;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = lane >> 4, l16 = lane & 15;  // k-group (plane within a k-step) and pixel / channel row of this lane
  const int n0 = blockIdx.y * Tr::BN;
  const int RC = cg.R * cg.C, RSC = RC * cg.S;

  const int tiles_q = (cg.Q + QT - 1) / QT;
  const int total = (p.M / cg.Q) * tiles_q;  // output rows of the whole batch x column tiles

  // ---- staging --------------------------------------------------------------------------------------------------
  // What a tile needs lies in global memory as NSEG contiguous runs of SEGLEN halves: one per input row in NHWC (all
  // columns x channels of the row), one per (input row, channel) in NCHW.  A run starts at any 2-byte boundary, but
  // 2-byte global loads are served at a small fraction of the rate of 4-byte ones, so a work item is one ALIGNED
  // dword of a run (DW of them cover it whatever its start); item w belongs to thread w % 256.  First half (fetch):
  // global memory -> one register per item, all loads together; a dword outside the tensor or of a row outside the
  // image gets an offset beyond the buffer and reads as zero.  Second half (scatter), one tile later, so that the
  // loads of tile i + 1 fly while tile i is multiplied and stored: each of the two halves goes to column j of plane
  // r * C + c with a 2-byte LDS write (zero if its column lies outside the image).
  const int seglen = p.x_nchw ? COLS : COLS * cg.C, nseg = p.x_nchw ? RC : cg.R, dw = seglen / 2 + 1;
  const float rcp_dw = 1.0f / (float)dw;                                       // items < 2^13, dw < 2^10: exact
  const int stride_r = p.x_nchw ? cg.Wi : cg.Wi * cg.C, stride_c = p.x_nchw ? cg.H * cg.Wi : 0;
  const int rcp5_c = cg.C == 1 ? 32 : cg.C == 2 ? 16 : cg.C == 3 ? 11 : 8;     // v / C = (v * rcp5_c) >> 5, v < 32
  const int rcp17_c = cg.C == 1 ? 131072 : cg.C == 2 ? 65536 : cg.C == 3 ? 43691 : 32768;  // ... >> 17, v < 2^15
  constexpr int NI = (Tr::PAIRS * (COLS / 2 + 1) + 255) / 256;  // C * (COLS / 2) + 1 <= C * (COLS / 2 + 1)
  unsigned v[NI];
  // (rounded up to whole dwords: the last element of a tensor with an odd element count shares its dword with two
  // bytes that still lie inside the caller's allocation - x is 16-byte aligned and allocations are multiples of 4)
  const __amdgpu_buffer_rsrc_t xrsrc = make_rsrc(p.X, ((unsigned)((int64_t)(p.M / (cg.P * cg.Q)) * cg.H * cg.Wi * cg.C * 2) + 3u) & ~3u);
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
  // item i of this thread: its run, the first half of the run in the tensor (g0) and the item's dword in the tensor
  struct Item { int seg, r, c, g0, a; };
  auto item = [&](const TileAt& t, int otid, int i) {
    Item it;
    const int w = otid + 256 * i;
    it.seg = (int)(((float)w + 0.5f) * rcp_dw);
    const int m = w - it.seg * dw;
    it.r = p.x_nchw ? (it.seg * rcp5_c) >> 5 : it.seg;
    it.c = p.x_nchw ? it.seg - it.r * cg.C : 0;
    it.g0 = t.base + it.r * stride_r + it.c * stride_c;
    it.a = (it.g0 >> 1) + m;
    return it;
  };
  auto fetch = [&](const TileAt& t) {
    // (everything derived from the thread index alone is the same for every tile; the empty asm keeps the compiler
    // from hoisting those values out of the tile loop into registers of their own)
    int otid = tid;
    asm volatile("" : "+v"(otid));
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const Item it = item(t, otid, i);
      const bool ok = (it.seg < nseg) & ((unsigned)(t.ih0 + it.r) < (unsigned)cg.H) & (it.a >= 0);
      v[i] = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, ok ? (unsigned)it.a * 4u : kInvalidOffset, 0, 0);
    }
  };
  auto scatter = [&](const TileAt& t) {
    int otid = tid;
    asm volatile("" : "+v"(otid));
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const Item it = item(t, otid, i);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int x = 2 * it.a + hh - it.g0;  // position in the run
        const int j = p.x_nchw ? x : (x * rcp17_c) >> 17, c = p.x_nchw ? it.c : x - j * cg.C;
        const bool col_ok = (unsigned)(t.iw_lo + j) < (unsigned)cg.Wi;
        const unsigned short h = col_ok ? (unsigned short)(hh ? v[i] >> 16 : v[i] & 0xffffu) : (unsigned short)0;
        if ((it.seg < nseg) & ((unsigned)x < (unsigned)seglen)) ((unsigned short*)planes)[(it.r * cg.C + c) * ROW + j] = h;
      }
    }
  };
  TileAt cur = locate(blockIdx.x < total ? blockIdx.x : 0);
  if ((int)blockIdx.x < total) fetch(cur);

  // ---- weights: global [K][R][S][C] -> LDS in fragment order, zero-filled -----------------------------------------
  // The 64 channels of this workgroup are one contiguous, 16-byte aligned run of 64 * R * S * C halves: 16-byte loads,
  // all of them first so that their latency is paid once, then every half is scattered to its slot.
  {
    constexpr int NWL = (Tr::BN * Tr::PAIRS * 8 / 8 + 255) / 256;
    const int wtotal = (p.N - n0 < Tr::BN ? p.N - n0 : Tr::BN) * RSC;  // halves of the run; a multiple of 8 (N % 8 == 0)
    const __amdgpu_buffer_rsrc_t wrsrc = make_rsrc(p.W + (int64_t)n0 * p.ldw, (unsigned)wtotal * 2u);
    half8 wv[NWL];
#pragma unroll
    for (int i = 0; i < NWL; ++i) {
      const int f = (tid + 256 * i) * 8;
      const auto raw = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, f < wtotal ? (unsigned)f * 2u : kInvalidOffset, 0, 0);
      __builtin_memcpy(&wv[i], &raw, 16);
    }
    for (int i = tid; i < (Tr::W_HALVES + Tr::IN_HALVES) / 8; i += 256) *(half8*)(lds + i * 8) = half8{0, 0, 0, 0, 0, 0, 0, 0};
    __syncthreads();
    // flat index f -> (channel, r, s, c) with exact float reciprocals (f < 2^14, divisors < 2^8)
    const float rcp_rsc = 1.0f / (float)RSC, rcp_sc = 1.0f / (float)(cg.S * cg.C), rcp_1c = 1.0f / (float)cg.C;
#pragma unroll
    for (int i = 0; i < NWL; ++i) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int f = (tid + 256 * i) * 8 + k;
        const int chl = (int)(((float)f + 0.5f) * rcp_rsc), e = f - chl * RSC;
        const int r = (int)(((float)e + 0.5f) * rcp_sc), rem = e - r * cg.S * cg.C;
        const int s = (int)(((float)rem + 0.5f) * rcp_1c), c = rem - s * cg.C;
        const int pair = r * cg.C + c, t = pair >> 2, grp = pair & 3;
        const int blk = 2 * (chl >> 5) + ((chl >> 2) & 1), row = 4 * ((chl >> 3) & 3) + (chl & 3);
        if (f < wtotal) wfrag[((t * 4 + blk) * 64 + grp * 16 + row) * 8 + s] = wv[i][k];
      }
    }
  }
  // (planes beyond R * C are never written again: they stay zero, as their weights are; the barrier that publishes
  // the first tile's planes publishes the weights too)

  // taps s >= S of a fragment are masked: dword d of the fragment holds taps 2d, 2d + 1
  unsigned tap_mask[4];
#pragma unroll
  for (int d = 0; d < 4; ++d) tap_mask[d] = (2 * d + 1 < cg.S) ? 0xffffffffu : (2 * d < cg.S) ? 0x0000ffffu : 0u;

  // this lane's bias: channels n0 + 32 * hb + 8 * kg + [0, 8), hb = 0, 1 (zero beyond N and without a bias)
  half8 bias_h[2];
#pragma unroll
  for (int hb = 0; hb < 2; ++hb) {
    const int n = n0 + 32 * hb + 8 * kg;
    const half8 got = *(const half8*)(p.bias + (n < p.N ? n : 0) * p.bias_on);
    bias_h[hb] = (n < p.N && p.bias_on) ? got : half8{0, 0, 0, 0, 0, 0, 0, 0};
  }

  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    scatter(cur);
    __syncthreads();
    const int orow = cur.orow, q0 = cur.q0;
    if (tile + (int)gridDim.x < total) {
      cur = locate(tile + gridDim.x);
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
      const half_t* plane = planes + (t * 4 + kg) * ROW;
      half8 wf[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) wf[b] = *(const half8*)(wfrag + ((t * 4 + b) * 64 + lane) * 8);
#pragma unroll
      for (int pb = 0; pb < 2; ++pb) {
        const int ql = wave * 32 + pb * 16 + l16;
        union { unsigned u[4]; half8 h; } xf;
        if constexpr (SW == 2) {
          const unsigned* src = (const unsigned*)(plane + ql * 2);
#pragma unroll
          for (int d = 0; d < 4; ++d) xf.u[d] = src[d] & tap_mask[d];
        } else {
          const unsigned short* src = (const unsigned short*)(plane + ql * SW);
#pragma unroll
          for (int d = 0; d < 4; ++d) xf.u[d] = ((unsigned)src[2 * d] | ((unsigned)src[2 * d + 1] << 16)) & tap_mask[d];
        }
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
          if (n < p.N) __builtin_nontemporal_store(o, (half8*)(yrow + n));
        }
      }
    };
    if (p.act > ACT_RELU) store_tile(std::true_type{});
    else store_tile(std::false_type{});
    __syncthreads();  // every wave has read its fragments: the planes may be overwritten
  }
}

template <int T, int SW>
hipError_t launch_conv_smallc(const FpropParams& p, hipStream_t stream) {
  using Tr = ConvSmallCTraits<T, SW>;
  static LdsOptIn opt_in;
  auto kern = conv_smallc_kernel<T, SW>;
  if (hipError_t e = opt_in.ensure((const void*)kern, Tr::LDS_BYTES); e != hipSuccess) return e;
  const int64_t total = (int64_t)(p.M / p.cg.Q) * ((p.cg.Q + Tr::QT - 1) / Tr::QT);
  constexpr int kComputeUnits = 256, kPerCU = 4;
  dim3 grid((unsigned)(total < kComputeUnits * kPerCU ? total : kComputeUnits * kPerCU), (p.N + Tr::BN - 1) / Tr::BN, 1);
  hipLaunchKernelGGL(kern, grid, dim3(Tr::NT), Tr::LDS_BYTES, stream, p);
  return hipGetLastError();
}

// In the instance table: x mode 4 (few channels, any alignment, NHWC or NCHW input), tile = 128 pixels x 64 channels,
// tile K = the 32 of one matrix instruction, no split-K.
#define BOLT_CONV_SMALLC_INSTANCE(T, SW)                                                                  \
  {                                                                                                       \
    "smallc_t" #T "_sw" #SW, 128, 64, 32, 4, 1, 4, 0, 1, bolt::ConvSmallCTraits<T, SW>::LDS_BYTES,         \
        &bolt::launch_conv_smallc<T, SW>, 0, nullptr, nullptr, &bolt::ConvSmallCTraits<T, SW>::supports,  \
        &bolt::ConvSmallCTraits<T, SW>::lds_bytes, 0, 16, true                                            \
  }

}  // namespace bolt
