// Tiled matrix-core GEMM / implicit-GEMM convolution with the epilogue fused in registers.
//
// Follows the hierarchy of Section 2.2 (Figure 2): workgroup tile BM x BN x BK staged
// global -> LDS, wave tiles read LDS -> registers, MFMA accumulates in registers; the epilogue
// (scale, broadcast bias, activation, FP32 -> FP16: patterns (i)-(iii) of Section 3.1) is applied
// to the accumulators before the single store.  The template parameters are the search space of
// the profiler of Section 3.2.2: workgroup tile, wave grid, K depth.
//
// GEMM view: Y[m][n] = act(alpha * sum_k X[m][k] * Wt[n][k] + beta * bias[n]).
//   XMODE 0: X is a row-major matrix (GEMM A).       XMODE 1: X is the im2col view of an NHWC
//   tensor, never materialised: row m = (img, p, q), column k = (r, s, c), zero outside the image.
//   WMODE 0: weights stored [N][K] (K contiguous: conv KRSC, or a transposed GEMM B).
//   WMODE 1: weights stored [K][N] (row-major GEMM B); 8x8 blocks are transposed in registers on
//   the way to LDS so that both operands sit K-contiguous in LDS.
// The MFMA computes the transposed product (weights as the A operand, activations as the B
// operand), so a lane ends up with 4 consecutive output channels of one output row: a quad for the
// epilogue, and the layout the back-to-back kernels need to reuse accumulators as operands.
#pragma once
#include <type_traits>

#include "bolt_device.hpp"
#include "tile_loaders.hpp"

namespace bolt {

struct FpropParams {
  const half_t* X;
  const half_t* W;
  const half_t* bias;  // [N]; never null inside the kernels: without a bias it addresses 8 zero halves
  int bias_on;         // 1 with a bias, 0 without (multiplies the bias index)
  half_t* Y;           // [M][ldy]
  const half_t* res;   // residual matrix C of Eq. 1, [M][ldr], or nullptr: Y = act(alpha acc + beta bias + gamma res)
  int ldr;
  float gamma;
  float* partial;      // split-K partial sums [split_k][M][N], or nullptr
  int M, N, K;
  int ldx, ldw, ldy;
  float alpha, beta;
  int act;
  int tiles_m, tiles_n, swizzle;
  int split_k, ktiles_per_split;
  ConvGeom cg;  // convolutions only
  int x_nchw;   // x mode 4 only: the input is [N][C][H][W]
  int y_nchw;   // the output is [N][K][P][Q] (first-layer kernels take it as a run-time switch)
};

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int XMODE, int WMODE>
struct FpropTraits {
  static constexpr int NT = 64 * WAVES_M * WAVES_N;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int FM = WTM / 32, FN = WTN / 32;
  static constexpr int LDS_BYTES = 2 * (BM + BN) * BK * 2;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
};

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int XMODE, int WMODE>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void fprop_kernel(const FpropParams p) {
  using T = FpropTraits<BM, BN, BK, WAVES_M, WAVES_N, XMODE, WMODE>;
  constexpr int NT = T::NT, WTM = T::WTM, WTN = T::WTN, FM = T::FM, FN = T::FN;

  extern __shared__ __attribute__((aligned(16))) half_t lds[];
  half_t* Xs = lds;                // [2][BM*BK]
  half_t* Ws = lds + 2 * BM * BK;  // [2][BN*BK]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  int tm, tn;
  tile_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, p.swizzle, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int z = blockIdx.y;
  const int nk_total = (p.K + BK - 1) / BK;
  const int kt_begin = z * p.ktiles_per_split;
  const int kt_end = (kt_begin + p.ktiles_per_split) < nk_total ? (kt_begin + p.ktiles_per_split) : nk_total;

  XTileLoader<BM, BK, NT, XMODE> xl;
  WTileLoader<BN, BK, NT, WMODE> wl;
  xl.init(p.X, p.ldx, p.M, p.K, p.cg, m0, kt_begin, tid);
  wl.init(p.W, p.ldw, p.N, p.K, n0, tid);

  floatx16 acc[FN][FM];
#pragma unroll
  for (int a = 0; a < FN; ++a)
#pragma unroll
    for (int b = 0; b < FM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  auto compute = [&](int buf) {
    const half_t* xs = Xs + buf * BM * BK;
    const half_t* ws = Ws + buf * BN * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      half8 xf[FM], wf[FN];
      const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
      for (int b = 0; b < FM; ++b)
        xf[b] = *(const half8*)(xs + lds_chunk_offset<BK>(wm * WTM + b * 32 + (lane & 31), chunk));
#pragma unroll
      for (int a = 0; a < FN; ++a)
        wf[a] = *(const half8*)(ws + lds_chunk_offset<BK>(wn * WTN + a * 32 + (lane & 31), chunk));
#pragma unroll
      for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b) acc[a][b] = mfma_32x32x16(wf[a], xf[b], acc[a][b]);
    }
  };

  // ---- main loop: register-staged prefetch into a double-buffered LDS tile ----------------
  if (kt_begin < kt_end) {
    xl.load(kt_begin, p.cg);
    wl.load(kt_begin);
    xl.store(Xs);
    wl.store(Ws);
    __syncthreads();
    for (int kt = kt_begin; kt < kt_end; ++kt) {
      const int buf = (kt - kt_begin) & 1;
      const bool more = kt + 1 < kt_end;
      if (more) {
        xl.load(kt + 1, p.cg);
        wl.load(kt + 1);
      }
      compute(buf);
      if (more) {
        xl.store(Xs + (buf ^ 1) * BM * BK);
        wl.store(Ws + (buf ^ 1) * BN * BK);
      }
      __syncthreads();
    }
  }

  // ---- epilogue in registers -----------------------------------------------------------------
  const int mrow = m0 + wm * WTM + (lane & 31);
  const int ncol = n0 + wn * WTN + (lane >> 5) * 4;
  if (p.split_k > 1) {
    float* dst = p.partial + (int64_t)z * p.M * p.N;
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
      for (int b = 0; b < FM; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int m = mrow + b * 32, n = ncol + a * 32 + q * 8;
          if (m < p.M && n < p.N) {
            floatx4 v = {acc[a][b][q * 4], acc[a][b][q * 4 + 1], acc[a][b][q * 4 + 2], acc[a][b][q * 4 + 3]};
            *(floatx4*)(dst + (int64_t)m * p.N + n) = v;
          }
        }
    return;
  }
  // FP16 tile through LDS (over the operand buffers, which the loop's last barrier has retired; 16-byte chunks
  // XOR-swizzled by row, see ctile_swizzle) so that every store instruction writes whole 128-byte row segments
  // instead of one 8-byte quad per lane.  With a residual each lane first reads the quad of C its quad replaces.
  constexpr int CPR = BN / 8, STORE_THREADS = NT / CPR <= BM ? NT : BM * CPR, ROWS_PER_PASS = STORE_THREADS / CPR;
  static_assert(STORE_THREADS % CPR == 0 && BM % ROWS_PER_PASS == 0, "C tile store mapping");
  static_assert(BM * BN * 2 <= T::LDS_BYTES, "the C tile fits over the operand buffers");
  const EpilogueArgs ep{p.bias, p.bias_on, p.N, p.alpha, p.beta, p.act, p.gamma};
  const int g = lane >> 5, l32 = lane & 31;
  auto tile_to_lds = [&](auto slow, auto with_res) {
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nl = wn * WTN + a * 32 + q * 8 + g * 4;  // column inside the tile
#pragma unroll
        for (int b = 0; b < FM; ++b) {
          const int row = wm * WTM + b * 32 + l32;
          half4 o;
          if constexpr (decltype(with_res)::value) {
            const half4 zero = {0, 0, 0, 0};
            const bool ok = n0 + nl < p.N && m0 + row < p.M;
            const half4 r = ok ? *(const half4*)(p.res + (int64_t)(m0 + row) * p.ldr + n0 + nl) : zero;
            o = epilogue_quad_res<decltype(slow)::value>(acc[a][b], q, n0 + nl, ep, r);
          } else {
            o = epilogue_quad<decltype(slow)::value>(acc[a][b], q, n0 + nl, ep);
          }
          *(half4*)(lds + row * BN + (((nl >> 3) ^ ctile_swizzle<CPR>(row)) << 3) + (nl & 4)) = o;
        }
      }
  };
  if (p.res) {
    if (p.act > ACT_RELU) tile_to_lds(std::true_type{}, std::true_type{});
    else tile_to_lds(std::false_type{}, std::true_type{});
  } else {
    if (p.act > ACT_RELU) tile_to_lds(std::true_type{}, std::false_type{});
    else tile_to_lds(std::false_type{}, std::false_type{});
  }
  __syncthreads();
  if (tid < STORE_THREADS) {
    const int chunk = tid % CPR, r0 = tid / CPR;
    const int n = n0 + chunk * 8;
    if (n < p.N) {
#pragma unroll
      for (int i = 0; i < BM / ROWS_PER_PASS; ++i) {
        const int row = r0 + i * ROWS_PER_PASS;
        if (m0 + row < p.M) {
          const half8 v = *(const half8*)(lds + row * BN + ((chunk ^ ctile_swizzle<CPR>(row)) << 3));
          __builtin_nontemporal_store(v, (half8*)(p.Y + (int64_t)(m0 + row) * p.ldy + n));
        }
      }
    }
  }
}

struct FpropInstance {
  const char* name;
  int bm, bn, bk, waves_m, waves_n, xmode, wmode;
  int stages;  // LDS operand buffers in flight
  int lds_bytes;
  hipError_t (*launch)(const FpropParams&, hipStream_t);
  // instances whose legality / LDS need depends on the problem (conv_halo_kernel.hpp); null otherwise
  bool (*dyn_supports)(const FpropParams&);
  int (*dyn_lds_bytes)(const FpropParams&);
  int kgroups;  // k-groups of waves per workgroup (0 or 1: none); threads = 64 * waves_m * waves_n * kgroups
  int mi;       // matrix-core instruction: 0 or 32 = 32 x 32 x 16, 16 = 16 x 16 x 32
  bool no_split_k;  // the kernel has no partial-sum output
  bool nchw_out;    // writes its output as [N][K][P][Q] (and only that)
  bool kn_dma;      // row-major weights fetched through one 32-bit-offset buffer descriptor over the whole matrix
};

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int XMODE, int WMODE>
hipError_t launch_fprop(const FpropParams& p, hipStream_t stream) {
  using T = FpropTraits<BM, BN, BK, WAVES_M, WAVES_N, XMODE, WMODE>;
  auto kern = fprop_kernel<BM, BN, BK, WAVES_M, WAVES_N, XMODE, WMODE>;
  static LdsOptIn opt_in;
  if (hipError_t e = opt_in.ensure((const void*)kern, T::LDS_BYTES); e != hipSuccess) return e;
  dim3 grid(p.tiles_m * p.tiles_n, p.split_k, 1);
  hipLaunchKernelGGL(kern, grid, dim3(T::NT), T::LDS_BYTES, stream, p);
  return hipGetLastError();
}

#define BOLT_FPROP_INSTANCE(BM, BN, BK, WM, WN, XMODE, WMODE)                                          \
  {                                                                                                    \
    #BM "x" #BN "x" #BK "_w" #WM "x" #WN, BM, BN, BK, WM, WN, XMODE, WMODE, 2,                           \
        bolt::FpropTraits<BM, BN, BK, WM, WN, XMODE, WMODE>::LDS_BYTES,                                 \
        &bolt::launch_fprop<BM, BN, BK, WM, WN, XMODE, WMODE>, nullptr, nullptr                        \
  }

}  // namespace bolt
