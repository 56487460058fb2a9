// Multi-stage GEMM / implicit-GEMM convolution kernel: operand tiles go global -> LDS directly
// (buffer_load ... lds, 16 bytes per lane, no staging registers), NS tiles deep, so that the
// latency of the loads for tile k+NS-1 is hidden behind the MFMA work on tiles k .. k+NS-2.
// "Stages" is one of the searched template parameters of Section 3.2.2; everything else follows
// the tiling of Section 2.2 as in fprop_kernel.hpp.  The activations are K-contiguous in memory (NHWC, or a
// row-major A); the weights are K-contiguous too (KRSC, or B stored [N][K]) or, for GEMMs, row-major [K][N]: those
// tiles go to LDS as they lie in memory and are read with the LDS transpose read (WKN, DmaKnTileLoader below).
//
// Out-of-range rows, the K tail and zero-padding taps are not branched on: their lanes are given a
// byte offset beyond the buffer descriptor's range, for which the hardware writes zeros to LDS.
//
// Epilogue (Section 3.1, patterns (i)-(iii)): scale, bias, activation and FP16 conversion on the
// accumulator registers, then the FP16 tile is transposed through LDS so that every store
// instruction writes whole 128-byte row segments.
#pragma once
#include "bolt_device.hpp"
#include "fprop_kernel.hpp"

namespace bolt {

#define BOLT_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

#ifndef BOLT_INTERLEAVE_READS
#define BOLT_INTERLEAVE_READS 1
#endif
#ifndef BOLT_FRAG_DEPTH
#define BOLT_FRAG_DEPTH 4  // MFMAs a register set of fragments should feed
#endif
static constexpr unsigned kInvalidOffset = 0x80000000u;  // beyond any descriptor range we create

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, bytes, 0x00020000);
}

// Workgroup barriers without the full fence of __syncthreads(): that fence would drain every
// outstanding global load, including the prefetches that are meant to stay in flight.  The "memory"
// clobber keeps the compiler from moving LDS accesses or direct-to-LDS loads across the barrier.
//   barrier_after_loads<VM>: this wave's direct-to-LDS loads, except the VM newest, have landed.
//   barrier_after_reads_and_loads<VM>: the same, and this wave's LDS reads have returned.
//   barrier_after_lds_writes: this wave's ds_write instructions have completed.
// The waits go through the s_waitcnt builtin so that the compiler's own wait-count bookkeeping
// sees them (an asm wait would make it wait again, later and for more); the barrier itself is asm
// with a "memory" clobber.  gfx9 s_waitcnt encoding: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8].
__device__ __forceinline__ void raw_barrier() { asm volatile("s_barrier" ::: "memory"); }
template <int VM>
__device__ __forceinline__ void barrier_after_loads() {
  static_assert(VM >= 0 && VM < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((VM & 0xF) | ((VM >> 4) << 14) | 0x0F70);
  raw_barrier();
}
template <int VM>
__device__ __forceinline__ void barrier_after_reads_and_loads() {
  static_assert(VM >= 0 && VM < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((VM & 0xF) | ((VM >> 4) << 14) | 0x0070);
  raw_barrier();
}
__device__ __forceinline__ void barrier_after_lds_writes() {
  __builtin_amdgcn_s_waitcnt(0xC07F);
  raw_barrier();
}

// Swizzle used by the direct-to-LDS tiles.  The LDS of this chip has 64 banks of 4 bytes and serves
// a 128-bit read 16 lanes at a time, so the 16 lanes that read one logical chunk of 16 consecutive
// rows must land in 16 different 16-byte bank groups.  A row is BK*2 bytes, so the bank group of
// (row, chunk) is (row*CH + chunk) mod 16: XOR the chunk with the row bits above the ones that
// already select the bank group.  A lane's 16-byte slot in LDS is fixed by the hardware
// (slot = lane), so the permutation is applied to which global chunk the lane fetches; with an even
// number of waves the XOR term is the same for every row group a lane serves.
template <int BK>
__device__ __forceinline__ int dma_swizzle(int row) {
  return BK == 32 ? ((row >> 2) & 3) : ((row >> 1) & 7);
}
template <int BK>
__device__ __forceinline__ int dma_chunk_offset(int row, int chunk) {
  return row * BK + ((chunk ^ dma_swizzle<BK>(row)) << 3);
}

// One operand tile of ROWS x BK halves moved by NW waves; each load instruction of a wave fills
// 1024 contiguous LDS bytes = RPI whole tile rows.
// KSTRIDE: how many k-tiles the conv cursor advances per issue (k-groups interleave the k-tiles).
template <int ROWS, int BK, int NW, int XMODE, int KSTRIDE = 1>
struct DmaTileLoader {
  static constexpr int CH = BK / 8;
  static constexpr int RPI = 64 / CH;          // tile rows per instruction
  static constexpr int NI = ROWS / RPI / NW;   // instructions per wave per tile
  static_assert(BK == 32 || BK == 64, "BK");
  static_assert(ROWS % (RPI * NW) == 0 && NI >= 1, "tile rows must split evenly over the waves");
  static_assert(NW % 2 == 0, "the swizzle term of a lane must not depend on the row group");

  __amdgpu_buffer_rsrc_t rsrc;
  int xbase[XMODE >= 1 ? NI : 1];
  int xhw[XMODE >= 1 ? NI : 1];
  int cr, cs, cc;
  int ld, rows_valid, K, wave, lrow, lc;

  // GEMM-like source (XMODE 0): `base` points at row 0 of this tile, `bytes` is what remains of the
  // tensor from there.  Conv source (XMODE 1): base/bytes describe the whole NHWC tensor.
  __device__ __forceinline__ void init(const half_t* base, unsigned bytes, int ld_, int rows_valid_, int K_,
                                       const ConvGeom& cg, int m0, int kt_begin, int wave_, int lane) {
    rsrc = make_rsrc(base, bytes);
    ld = ld_;
    rows_valid = rows_valid_;
    K = K_;
    wave = wave_;
    lrow = lane / CH;
    lc = (lane % CH) ^ dma_swizzle<BK>(wave * RPI + lrow);  // same for every j because NW is even
    cr = cs = cc = 0;
    if constexpr (XMODE == 1) {
      const int PQ = cg.P * cg.Q;
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int row = (j * NW + wave) * RPI + lrow;
        if (row < rows_valid) {
          const int m = m0 + row;
          const int img = m / PQ, rem = m - img * PQ;
          const int op = rem / cg.Q, oq = rem - op * cg.Q;
          const int ih0 = op * cg.stride_h - cg.pad_h, iw0 = oq * cg.stride_w - cg.pad_w;
          xbase[j] = ((img * cg.H + ih0) * cg.Wi + iw0) * cg.C;
          xhw[j] = (int)(((unsigned)ih0 << 16) | ((unsigned)iw0 & 0xffffu));
        } else {
          xbase[j] = 0;
          xhw[j] = (int)0x80008000u;
        }
      }
      const int k = kt_begin * BK + lc * 8;
      const int rs = k / cg.C;
      cc = k - rs * cg.C;
      cr = rs / cg.S;
      cs = rs - cr * cg.S;
    }
  }

  // Issue the loads of k-tile kt into the LDS tile at `dst` (conv mode: tiles in increasing order).
  __device__ __forceinline__ void issue(int kt, half_t* dst, const ConvGeom& cg) {
    issue_part<0, NI>(kt, dst, cg);
    advance(cg);
  }
  // Instructions J0 .. J1-1 of k-tile kt only; advance() moves the conv cursor to the next k-tile
  // once all parts of a tile have been issued.
  template <int J0, int J1>
  __device__ __forceinline__ void issue_part(int kt, half_t* dst, const ConvGeom& cg) {
    const int k = kt * BK + lc * 8;
    if constexpr (XMODE == 0) {
#pragma unroll
      for (int j = J0; j < J1; ++j) {
        const int rb = (j * NW + wave) * RPI;
        const int row = rb + lrow;
        const unsigned off = (row < rows_valid && k < K) ? (unsigned)(row * ld + k) * 2u : kInvalidOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, BOLT_LDS_PTR(dst + rb * BK), 16, off, 0, 0, 0);
      }
    } else {
      const int delta = (cr * cg.Wi + cs) * cg.C + cc;
#pragma unroll
      for (int j = J0; j < J1; ++j) {
        const int rb = (j * NW + wave) * RPI;
        const int ih = (xhw[j] >> 16) + cr, iw = (int)(short)(xhw[j] & 0xffff) + cs;
        const bool ok = k < K && (unsigned)ih < (unsigned)cg.H && (unsigned)iw < (unsigned)cg.Wi;
        const unsigned off = ok ? (unsigned)(xbase[j] + delta) * 2u : kInvalidOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, BOLT_LDS_PTR(dst + rb * BK), 16, off, 0, 0, 0);
      }
    }
  }
  __device__ __forceinline__ void advance(const ConvGeom& cg) {
    if constexpr (XMODE == 1) {
      cc += BK * KSTRIDE;
      while (cc >= cg.C) {
        cc -= cg.C;
        if (++cs == cg.S) {
          cs = 0;
          ++cr;
        }
      }
    }
  }
};

// Row-major weights (GEMM, B stored [K][N]): the k-tile is BK rows of BN contiguous halves and goes to LDS as it
// lies in memory, 16 bytes per lane; nothing is transposed on the way.  The matrix core wants, per lane, 8
// consecutive k of ONE column n, which in this tile is a column walk; the LDS transpose read of this chip
// (ds_read_b64_tr_b16) does that walk in hardware: within each group of 16 lanes, lanes 4r .. 4r+3 address the
// four 8-byte quarters of a 16-half row segment r (r = 0..3), and lane i of the group receives element i of each of
// the four segments, that is 4 consecutive k of column i when the segments are 4 consecutive rows of the tile.
// Two such reads make one 8-half operand.
// A half-wave (32 lanes, one pass of an 8-byte read) touches 4 consecutive rows x 64 bytes; the 16-byte chunk of a
// row is XOR-ed with row bits so that those 16 chunks fall into 16 different bank groups whatever the row length.
template <int BN>
__device__ __forceinline__ int kn_swizzle(int k) {
  static_assert(BN == 32 || BN == 64 || BN == 128 || BN == 256, "row-major weight tile width");
  if constexpr (BN == 32) return 0;             // 64-byte rows: 4 consecutive rows already cover 256 bytes
  else if constexpr (BN == 64) return ((k >> 1) & 1) << 2;  // rows k and k+2 share a bank half: flip chunk bit 2
  else return (k & 3) << 2;                     // rows are multiples of 256 bytes: 4 rows take 4 chunk quartets
}
template <int BK, int BN, int NW>
struct DmaKnTileLoader {
  static constexpr int CH = BN / 8;            // 16-byte chunks per tile row
  static constexpr int RPI = 64 / CH;          // tile rows (k) per load instruction
  static constexpr int NI = BK / RPI / NW;     // instructions per wave per tile
  static_assert(CH <= 64 && 64 % CH == 0, "a load instruction fills whole tile rows");
  static_assert(BK % (RPI * NW) == 0 && NI >= 1, "tile rows must split evenly over the waves");

  __amdgpu_buffer_rsrc_t rsrc;
  int ld, cols_valid, K, wave, lrow, lc;

  // `base` points at column n0 of row 0 of the weight matrix, `bytes` is what remains of the matrix from there;
  // cols_valid = N - n0, K = the first k this workgroup must not read.
  __device__ __forceinline__ void init(const half_t* base, unsigned bytes, int ld_, int cols_valid_, int K_, int wave_, int lane) {
    rsrc = make_rsrc(base, bytes);
    ld = ld_;
    cols_valid = cols_valid_;
    K = K_;
    wave = wave_;
    lrow = lane / CH;
    lc = lane % CH;
  }
  template <int J0, int J1>
  __device__ __forceinline__ void issue_part(int kt, half_t* dst, const ConvGeom&) {
#pragma unroll
    for (int j = J0; j < J1; ++j) {
      const int rb = (j * NW + wave) * RPI;
      const int row = rb + lrow, k = kt * BK + row;
      const int c = lc ^ kn_swizzle<BN>(row);  // the chunk of the row this lane's fixed LDS slot holds
      const unsigned off = (k < K && c * 8 < cols_valid) ? (unsigned)(k * ld + c * 8) * 2u : kInvalidOffset;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, BOLT_LDS_PTR(dst + rb * BN), 16, off, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void issue(int kt, half_t* dst, const ConvGeom& cg) { issue_part<0, NI>(kt, dst, cg); }
  __device__ __forceinline__ void advance(const ConvGeom&) {}
};
// This lane's part of the operand for the 32 columns that start at tile column col0, reduction rows row0 .. row0+15 of
// the row-major tile at ws (row0 a multiple of 4): kn_frag_offset is the lane's constant part.  With the defaults the
// lane receives k = row0 + 8 (lane / 32) .. +7 of column col0 + lane % 32, the operand order of the matrix core;
// group_rows = 4 with second = 8 gives rows row0 + 4 (lane / 32) + {0..3, 8..11} (the RF-resident fused kernel's
// permutation of op1's reduction index).
template <int BN>
__device__ __forceinline__ int kn_frag_offset(int col0, int lane, int group_rows = 8) {
  const int r = (lane & 15) >> 2, col = col0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  return ((lane >> 5) * group_rows + r) * BN + (((col >> 3) ^ kn_swizzle<BN>(r)) << 3) + (col & 7);
}
// `ws` is __restrict__ for the sake of the compiler's wait-count pass: an LDS access that carries no alias
// information is given a wait for EVERY direct-to-LDS load in flight (the pass cannot tell the stage being read from
// the stages being filled), which would serialise the pipeline; ordinary loads carry type-based alias information
// and escape that, the transpose-read builtin carries none unless the inlined restrict scope gives it some.  The
// explicit waits in front of the workgroup barriers are what orders these reads after the loads they depend on.
template <int BN>
__device__ __forceinline__ half8 kn_frag_read(const half_t* __restrict__ ws, int lane_off, int row0, int second = 4) {
  typedef short short4v __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) short4v lds_short4;
  const half4 lo = __builtin_bit_cast(half4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(ws + lane_off + row0 * BN)));
  const half4 hi = __builtin_bit_cast(half4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(ws + lane_off + (row0 + second) * BN)));
  return half8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
}
// A whole row-major matrix [rows][cols] (leading dimension ld) into LDS as [rows_padded][BN] with the row swizzle
// above, zero beyond rows / cols: the flat list of 16-byte chunks dealt over the waves, 64 per instruction.  Issues
// the loads only; the caller waits (vmcnt) and synchronises.  The matrix must end below 2 GiB from W (host check).
template <int NT, int BN>
__device__ __forceinline__ void kn_matrix_to_lds(const half_t* W, int ld, int rows, int cols, int rows_padded, half_t* dst, int tid) {
  constexpr int CH = BN / 8;
  const __amdgpu_buffer_rsrc_t rsrc = make_rsrc(W, (unsigned)(((rows - 1) * ld + cols) * 2));
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int ninst = rows_padded * CH / 64;  // (rows_padded and CH are multiples of 32 and 4)
  for (int i = wave; i < ninst; i += NT / 64) {
    const int f = i * 64 + lane, row = f / CH, c = (f - row * CH) ^ kn_swizzle<BN>(row);
    const unsigned off = (row < rows && c * 8 < cols) ? (unsigned)(row * ld + c * 8) * 2u : kInvalidOffset;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, BOLT_LDS_PTR(dst + i * 512), 16, off, 0, 0, 0);
  }
}

// Last step of the tiled single-op kernels: accumulators -> FP16 C tile in LDS ([BM][BN], 16-byte chunks
// XOR-swizzled by row, over whatever the main loop left there) -> 16-byte coalesced non-temporal row stores.
// RES (Eq. 1's C as a full matrix, p.res): the residual tile is first brought into the same LDS locations
// and every lane reads the quad it is about to overwrite.  RES is a compile-time switch: the residual kernels
// are separate instantiations, so the plain kernels keep their register allocation and occupancy.
// `writer`: this wave holds the final accumulators (k-group 0).  Called by every thread of the workgroup.
// `to_lds(slow, ep)` writes this wave's accumulators as FP16 quads into the staged tile (the layout of the quads
// depends on the matrix-core instruction the main loop used).
template <bool RES, int BM, int BN, int STORE_THREADS, int ROWS_PER_PASS, bool NCHW = false, typename ToLds>
__device__ __forceinline__ void fprop_tile_out_with(half_t* lds, const FpropParams& p, int m0, int n0, bool writer, int tid,
                                                    ToLds&& to_lds) {
  constexpr int CPR = BN / 8;
  const int lane = tid & 63;
  const EpilogueArgs ep{p.bias, p.bias_on, p.N, p.alpha, p.beta, p.act, p.gamma};
  barrier_after_lds_writes();  // every wave has finished reading what the tile overwrites
  if constexpr (RES) {
    // direct-to-LDS, 16 bytes per lane: one instruction fills 1024 contiguous LDS bytes = RPI whole tile
    // rows; a lane's slot is fixed, so the row swizzle is applied to which global chunk it fetches.
    // Rows beyond M and columns beyond N are zero-filled.  No registers are held while the loads fly.
    constexpr int RPI = 64 / CPR > 0 ? 64 / CPR : 1, LPR = CPR < 64 ? CPR : 64;
    static_assert(CPR <= 64 && BM % RPI == 0, "residual tile rows per load instruction");
    const int64_t rem = ((int64_t)(p.M - m0 - 1) * p.ldr + p.N) * 2;
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.res + (int64_t)m0 * p.ldr, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff));
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = (int)(blockDim.x >> 6);
    for (int i = wave_all; i < BM / RPI; i += nwaves) {
      const int row = i * RPI + lane / LPR;
      const int c = (lane % LPR) ^ ctile_swizzle<CPR>(row);
      const bool ok = m0 + row < p.M && n0 + c * 8 < p.N;
      const unsigned off = ok ? (unsigned)((row * p.ldr + n0 + c * 8) * 2) : kInvalidOffset;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rr, BOLT_LDS_PTR(lds + i * RPI * BN), 16, off, 0, 0, 0);
    }
    barrier_after_loads<0>();
  }
  if (writer) {
    if (p.act > ACT_RELU) to_lds(std::true_type{}, ep);
    else to_lds(std::false_type{}, ep);
  }
  barrier_after_lds_writes();
  if constexpr (NCHW) {
    // The mirror image of the first layer's loader (Section 3.2.3: the transformation lives in the last layer's
    // kernel): the output is [N][K][P][Q].  A thread takes one 8-channel chunk of one tile row (= output pixel) out of
    // LDS and writes its 8 halves into 8 channel planes; consecutive lanes take consecutive pixels, so that for every
    // channel a wave writes one contiguous run of its plane.
    const int PQ = p.cg.P * p.cg.Q;
    for (int e = tid; e < BM * CPR; e += (int)blockDim.x) {
      const int row = e % BM, chunk = e / BM;
      const int m = m0 + row, n = n0 + chunk * 8;
      if (m < p.M && n < p.N) {
        const half8 v = *(const half8*)(lds + row * BN + ((chunk ^ ctile_swizzle<CPR>(row)) << 3));
        const int img = m / PQ, pq = m - img * PQ;
        half_t* y = p.Y + ((int64_t)img * p.N + n) * PQ + pq;
#pragma unroll
        for (int k = 0; k < 8; ++k) y[(int64_t)k * PQ] = v[k];
      }
    }
    return;
  }
  // LDS -> global: each thread moves 16 bytes, consecutive threads cover consecutive row bytes
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

// The 32 x 32 accumulator layout: lane l of a fragment holds, in registers 4q .. 4q+3, columns 8q + 4(l / 32) .. +3
// of row l % 32.
template <bool RES, int BM, int BN, int WTM, int WTN, int STORE_THREADS, int ROWS_PER_PASS, bool NCHW = false, int FN, int FM>
__device__ __forceinline__ void fprop_tile_out(half_t* lds, const floatx16 (&acc)[FN][FM], const FpropParams& p, int m0,
                                               int n0, int wm, int wn, bool writer, int tid) {
  constexpr int CPR = BN / 8;
  const int lane = tid & 63, g = lane >> 5, l32 = lane & 31;
  fprop_tile_out_with<RES, BM, BN, STORE_THREADS, ROWS_PER_PASS, NCHW>(lds, p, m0, n0, writer, tid, [&](auto slow, const EpilogueArgs& ep) {
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nl = wn * WTN + a * 32 + q * 8 + g * 4;  // column inside the tile
#pragma unroll
        for (int b = 0; b < FM; ++b) {
          const int row = wm * WTM + b * 32 + l32;
          half4* slot = (half4*)(lds + row * BN + (((nl >> 3) ^ ctile_swizzle<CPR>(row)) << 3) + (nl & 4));
          if constexpr (RES) *slot = epilogue_quad_res<decltype(slow)::value>(acc[a][b], q, n0 + nl, ep, *slot);
          else *slot = epilogue_quad<decltype(slow)::value>(acc[a][b], q, n0 + nl, ep);
        }
      }
  });
}

// KG k-groups: KG sets of WAVES_M x WAVES_N waves work on the same output tile, set g on the k-tiles
// g, g+KG, ...; the sets' accumulators are summed through LDS before the epilogue.  This multiplies
// the waves in flight for problems whose tile count cannot fill the chip, without a second kernel.
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int XMODE, int NS, int KG = 1>
struct FpropDmaTraits {
  static constexpr int WPG = WAVES_M * WAVES_N;  // waves per k-group
  static constexpr int NW = WPG * KG;
  static constexpr int NT = 64 * NW;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int FM = WTM / 32, FN = WTN / 32;
  static constexpr int GROUP_HALVES = (BM + BN) * BK;      // one k-tile of both operands
  static constexpr int STAGE_HALVES = KG * GROUP_HALVES;   // one pipeline stage
  static constexpr int PIPE_BYTES = NS * STAGE_HALVES * 2;
  static constexpr int CTILE_BYTES = BM * BN * 2;
  static constexpr int REDUCE_BYTES = (KG - 1) * BM * BN * 4;
  static constexpr int LDS_BYTES = (PIPE_BYTES > CTILE_BYTES ? PIPE_BYTES : CTILE_BYTES) > REDUCE_BYTES
                                       ? (PIPE_BYTES > CTILE_BYTES ? PIPE_BYTES : CTILE_BYTES)
                                       : REDUCE_BYTES;
  static constexpr int CPR = BN / 8;            // 16-byte chunks per C-tile row
  static constexpr int STORE_THREADS = NT / CPR <= BM ? NT : BM * CPR;  // threads that move the C tile out
  static constexpr int ROWS_PER_PASS = STORE_THREADS / CPR;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(NS >= 1 && NS <= 8, "stages (NS == 1: problems of a single k-tile per k-group only)");
  static_assert(KG >= 1 && NT <= 1024, "workgroup size");
  static_assert(STORE_THREADS % CPR == 0 && BM % ROWS_PER_PASS == 0, "C tile store mapping");
};

// NCHW: the output tensor is [N][K][P][Q] (convolutions only; see fprop_tile_out_with)
// WKN: the weights are row-major [K][N] (GEMM only), see DmaKnTileLoader.
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int XMODE, int NS, int KG = 1, bool RES = false, bool NCHW = false,
          bool WKN = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * KG) void fprop_dma_kernel(const FpropParams p) {
  using T = FpropDmaTraits<BM, BN, BK, WAVES_M, WAVES_N, XMODE, NS, KG>;
  constexpr int WPG = T::WPG, WTM = T::WTM, WTN = T::WTN, FM = T::FM, FN = T::FN;
  constexpr int STAGE = T::STAGE_HALVES;
  using XL = DmaTileLoader<BM, BK, WPG, XMODE, KG>;
  using WL = std::conditional_t<WKN, DmaKnTileLoader<BK, BN, WPG>, DmaTileLoader<BN, BK, WPG, 0, KG>>;
  static_assert(!WKN || XMODE == 0, "row-major weights: GEMM only");
  constexpr int L = XL::NI + WL::NI;  // load instructions per wave per k-tile
  static_assert((NS - 1) * L < 64, "vmcnt range");

  extern __shared__ __attribute__((aligned(16))) half_t lds[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = wave_all / WPG, wave = wave_all - kg * WPG;  // k-group, wave inside the group
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int g = lane >> 5, l32 = lane & 31;
  int tm, tn;
  tile_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, p.swizzle, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int z = blockIdx.y;
  const int nk_total = (p.K + BK - 1) / BK;
  const int kt_first = z * p.ktiles_per_split;
  const int kt_end = (kt_first + p.ktiles_per_split) < nk_total ? (kt_first + p.ktiles_per_split) : nk_total;
  // This group's k-tiles are kt_begin, kt_begin + KG, ...; every group runs the same number of
  // pipeline steps (the barriers are shared), tiles at or past kt_end load zeros.
  const int kt_begin = kt_first + kg;
  const int k_limit = kt_end * BK < p.K ? kt_end * BK : p.K;

  XL xl;
  WL wl;
  if constexpr (XMODE == 0) {
    const int64_t rem = ((int64_t)(p.M - m0 - 1) * p.ldx + p.K) * 2;
    xl.init(p.X + (int64_t)m0 * p.ldx, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff), p.ldx, p.M - m0, k_limit, p.cg,
            m0, kt_begin, wave, lane);
  } else {
    const int64_t bytes = (int64_t)p.cg.H * p.cg.Wi * p.cg.C * 2 * (int64_t)(p.M / (p.cg.P * p.cg.Q));
    xl.init(p.X, (unsigned)bytes, 0, p.M - m0, k_limit, p.cg, m0, kt_begin, wave, lane);
  }
  int wfo[WKN ? FN : 1];  // row-major weights: this lane's offset inside the tile, per fragment column
  if constexpr (WKN) {
    const int64_t rem = ((int64_t)(p.K - 1) * p.ldw + (p.N - n0)) * 2;  // (the host keeps the matrix under 2 GiB)
    wl.init(p.W + n0, (unsigned)rem, p.ldw, p.N - n0, k_limit, wave, lane);
#pragma unroll
    for (int a = 0; a < FN; ++a) wfo[a] = kn_frag_offset<BN>(wn * WTN + a * 32, lane);
  } else {
    const int64_t rem = ((int64_t)(p.N - n0 - 1) * p.ldw + p.K) * 2;
    wl.init(p.W + (int64_t)n0 * p.ldw, (unsigned)(rem < 0x7fffffff ? rem : 0x7fffffff), p.ldw, p.N - n0, k_limit, p.cg,
            n0, kt_begin, wave, lane);
  }

  floatx16 acc[FN][FM];
#pragma unroll
  for (int a = 0; a < FN; ++a)
#pragma unroll
    for (int b = 0; b < FM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  half_t* const lds_group = lds + kg * T::GROUP_HALVES;  // this k-group's part of every stage
  auto issue = [&](int kt, int stage) {
    half_t* s = lds_group + stage * STAGE;
    xl.issue(kt, s, p.cg);
    wl.issue(kt, s + BM * BK, p.cg);
  };
  // Fragments are double-buffered in registers in groups of G k-steps: the LDS reads of the next
  // group (or of the first group of the next tile) are in flight while the MFMAs of the current one
  // execute, so the matrix pipe keeps working across the workgroup barrier that separates two
  // k-tiles.  A wave tile with few accumulators issues few MFMAs per k-step, too few to cover an LDS
  // round trip, so it prefetches deeper: G k-steps hold about BOLT_FRAG_DEPTH MFMAs.
  constexpr int KS = BK / 16;
  constexpr int G = FM * FN >= BOLT_FRAG_DEPTH ? 1 : (BOLT_FRAG_DEPTH / (FM * FN) < KS ? BOLT_FRAG_DEPTH / (FM * FN) : KS);
  constexpr int NG = KS / G;  // fragment groups per k-tile
  static_assert(KS % G == 0 && (NG == 1 || NG % 2 == 0), "register sets alternate per group");
  half8 xf[2][G][FM], wf[2][G][FN];
  auto read_group = [&](int stage, int grp, half8 (&x)[G][FM], half8 (&w)[G][FN]) {
    const half_t* xs = lds_group + stage * STAGE;
    const half_t* ws = xs + BM * BK;
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const int chunk = (grp * G + k) * 2 + g;
#pragma unroll
      for (int b = 0; b < FM; ++b)
        x[k][b] = *(const half8*)(xs + dma_chunk_offset<BK>(wm * WTM + b * 32 + l32, chunk));
#pragma unroll
      for (int a = 0; a < FN; ++a) {
        if constexpr (WKN) w[k][a] = kn_frag_read<BN>(ws, wfo[a], (grp * G + k) * 16);
        else w[k][a] = *(const half8*)(ws + dma_chunk_offset<BK>(wn * WTN + a * 32 + l32, chunk));
      }
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

  // ---- NS-deep pipeline: one barrier per k-tile ----------------------------------------------
  const int n_tiles = (kt_end - kt_first + KG - 1) / KG;  // pipeline steps, the same for every k-group
  if (n_tiles > 0) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
      if (s < n_tiles) issue(kt_begin + s * KG, s);
    if (n_tiles >= NS) barrier_after_loads<(NS - 1) * L>();
    else barrier_after_loads<0>();
    read_group(0, 0, xf[0], wf[0]);
    int stage = 0;
    // The L load instructions of a k-tile are issued in SL slices spread over the MFMA groups that
    // follow the barrier which frees their stage: a burst of direct-to-LDS loads stalls in issue while
    // the address path digests it, and a wave issues in order, so everything behind the burst would
    // wait with it.  Slice 0 goes out right after the barrier, the others between the later groups.
    constexpr int SL = NG > 1 ? NG : KS;
    auto issue_slice = [&](int kt, int stg, auto sc) {
      constexpr int S = decltype(sc)::value;
      constexpr int lo = S * L / SL, hi = (S + 1) * L / SL;  // positions in [X instructions | W instructions]
      constexpr int XN = XL::NI;
      constexpr int xlo = lo < XN ? lo : XN, xhi = hi < XN ? hi : XN;
      constexpr int wlo = (lo > XN ? lo : XN) - XN, whi = (hi > XN ? hi : XN) - XN;
      half_t* s = lds_group + stg * STAGE;
      xl.template issue_part<xlo, xhi>(kt, s, p.cg);
      wl.template issue_part<wlo, whi>(kt, s + BM * BK, p.cg);
      if (S == SL - 1) {
        xl.advance(p.cg);
        wl.advance(p.cg);
      }
    };
    auto read_step = [&](int stg, int ks, half8 (&x)[FM], half8 (&w)[FN]) {
      const half_t* xs = lds_group + stg * STAGE;
      const half_t* ws = xs + BM * BK;
      const int chunk = ks * 2 + g;
#pragma unroll
      for (int b = 0; b < FM; ++b) x[b] = *(const half8*)(xs + dma_chunk_offset<BK>(wm * WTM + b * 32 + l32, chunk));
#pragma unroll
      for (int a = 0; a < FN; ++a) {
        if constexpr (WKN) w[a] = kn_frag_read<BN>(ws, wfo[a], ks * 16);
        else w[a] = *(const half8*)(ws + dma_chunk_offset<BK>(wn * WTN + a * 32 + l32, chunk));
      }
    };
    int fill_stage = 0;  // stage that the tile in flight of issue (tile it-1+NS) goes to
    // One k-tile; `par` = register set that holds its first fragment group.
    auto tile_body = [&](int it, auto par) {
      constexpr int P = decltype(par)::value;
      if constexpr (NG > 1) {
        // Large wave tiles: one LDS read between consecutive MFMAs instead of a burst of FM + FN reads in front
        // of them (a burst is FM + FN issue slots during which this wave feeds the matrix pipe nothing).
        constexpr bool IL = BOLT_INTERLEAVE_READS && G == 1 && FM * FN > FM + FN;
        auto group = [&](auto jc) {
          constexpr int j = decltype(jc)::value;
          constexpr int cur = (P + j) & 1, nxt = cur ^ 1;
          // Fences keep the order "loads, the next group's reads, this group's MFMAs": left alone, the
          // scheduler sinks each read to just before its first use and the MFMAs wait on LDS.
          __builtin_amdgcn_sched_barrier(0);
          if (j + 1 < NG) {
            // slice j+1 of the tile whose slice 0 went out at the barrier that ended tile it-1
            if (it >= 1 && it - 1 + NS < n_tiles)
              issue_slice(kt_begin + (it - 1 + NS) * KG, fill_stage, std::integral_constant<int, (j + 1 < NG ? j + 1 : 0)>{});
            if constexpr (IL) __builtin_amdgcn_sched_barrier(0);
            read_group(stage, j + 1, xf[nxt], wf[nxt]);
          } else {
            // end of tile `it`: this wave's reads of the tile are complete (lgkmcnt 0) and tile it+1 has
            // landed (vmcnt); after the barrier that holds for every wave, so the stage just read
            // can be refilled with tile it+NS while the last MFMAs of tile `it` are still to issue.
            // After the last tile this runs once more unconditionally (the fragments it reads are
            // never used): a branch here would make the compiler wait for the new reads before
            // the MFMAs below.
            if (NS >= 2 && n_tiles - 2 - it >= NS - 2) barrier_after_reads_and_loads<(NS >= 2 ? NS - 2 : 0) * L>();
            else barrier_after_reads_and_loads<0>();
            if (it + NS < n_tiles) issue_slice(kt_begin + (it + NS) * KG, stage, std::integral_constant<int, 0>{});
            fill_stage = stage;
            stage = stage + 1 == NS ? 0 : stage + 1;
            if constexpr (IL) __builtin_amdgcn_sched_barrier(0);
            read_group(stage, 0, xf[nxt], wf[nxt]);
          }
          if constexpr (!IL) __builtin_amdgcn_sched_barrier(0);
          mfma_group(xf[cur], wf[cur]);
          if constexpr (IL) {
#pragma unroll
            for (int i = 0; i < FM + FN; ++i) {
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
              __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
            }
            __builtin_amdgcn_sched_group_barrier(0x008, FM * FN - (FM + FN), 0);
            __builtin_amdgcn_sched_barrier(0);
          }
        };
        group(std::integral_constant<int, 0>{});
        group(std::integral_constant<int, 1>{});
        if constexpr (NG > 2) {
          group(std::integral_constant<int, 2>{});
          group(std::integral_constant<int, 3>{});
        }
        static_assert(NG == 2 || NG == 4 || NG == 1, "fragment groups per k-tile");
      } else {
        // One fragment group per tile (small wave tiles): the same interleave per k-step.
        constexpr int cur = P, nxt = P ^ 1;
        __builtin_amdgcn_sched_barrier(0);
        if (NS >= 2 && n_tiles - 2 - it >= NS - 2) barrier_after_reads_and_loads<(NS >= 2 ? NS - 2 : 0) * L>();
        else barrier_after_reads_and_loads<0>();
        const int nstage = stage + 1 == NS ? 0 : stage + 1;
        const bool more = it + NS < n_tiles;
        auto step = [&](auto kc) {
          constexpr int ks = decltype(kc)::value;
          if (more) issue_slice(kt_begin + (it + NS) * KG, stage, kc);
          read_step(nstage, ks, xf[nxt][ks], wf[nxt][ks]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int a = 0; a < FN; ++a)
#pragma unroll
            for (int b = 0; b < FM; ++b) acc[a][b] = mfma_32x32x16(wf[cur][ks][a], xf[cur][ks][b], acc[a][b]);
          __builtin_amdgcn_sched_barrier(0);
        };
        step(std::integral_constant<int, 0>{});
        if constexpr (KS > 1) step(std::integral_constant<int, 1>{});
        if constexpr (KS > 2) step(std::integral_constant<int, 2>{});
        if constexpr (KS > 3) step(std::integral_constant<int, 3>{});
        stage = nstage;
      }
    };
    if constexpr (NG % 2 == 0) {
      for (int it = 0; it < n_tiles; ++it) tile_body(it, std::integral_constant<int, 0>{});
    } else {  // one group per tile: the register sets swap roles every tile
      int it = 0;
      for (; it + 1 < n_tiles; it += 2) {
        tile_body(it, std::integral_constant<int, 0>{});
        tile_body(it + 1, std::integral_constant<int, 1>{});
      }
      if (it < n_tiles) tile_body(it, std::integral_constant<int, 0>{});
    }
  }

  // ---- k-groups: sum the accumulators through LDS, group 0 carries on ------------------------------
  if constexpr (KG > 1) {
    float* red = reinterpret_cast<float*>(lds);  // [KG-1][WPG][FN*FM*16][64 lanes]
    barrier_after_lds_writes();                  // every wave has finished reading the operand stages
    if (kg > 0) {
      float* mine = red + ((kg - 1) * WPG + wave) * (FN * FM * 16 * 64) + lane;
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
        const float* theirs = red + (o * WPG + wave) * (FN * FM * 16 * 64) + lane;
#pragma unroll
        for (int a = 0; a < FN; ++a)
#pragma unroll
          for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] += theirs[((a * FM + b) * 16 + r) * 64];
      }
    }
  }

  // ---- epilogue ---------------------------------------------------------------------------------
  const int mrow = m0 + wm * WTM + l32;
  const int ncol = n0 + wn * WTN + g * 4;
  if (p.split_k > 1) {
    if (kg > 0) return;  // (no barrier follows on this path)
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

  fprop_tile_out<RES, BM, BN, WTM, WTN, T::STORE_THREADS, T::ROWS_PER_PASS, NCHW>(lds, acc, p, m0, n0, wm, wn, kg == 0, tid);
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int XMODE, int NS, int KG = 1, bool WKN = false>
hipError_t launch_fprop_dma(const FpropParams& p, hipStream_t stream) {
  using T = FpropDmaTraits<BM, BN, BK, WAVES_M, WAVES_N, XMODE, NS, KG>;
  // the residual epilogue is a kernel of its own (see fprop_tile_out)
  auto kern = p.res ? fprop_dma_kernel<BM, BN, BK, WAVES_M, WAVES_N, XMODE, NS, KG, true, false, WKN>
                    : fprop_dma_kernel<BM, BN, BK, WAVES_M, WAVES_N, XMODE, NS, KG, false, false, WKN>;
  static LdsOptIn opt_in[2];
  if (hipError_t e = opt_in[p.res ? 1 : 0].ensure((const void*)kern, T::LDS_BYTES); e != hipSuccess) return e;
  dim3 grid(p.tiles_m * p.tiles_n, p.split_k, 1);
  hipLaunchKernelGGL(kern, grid, dim3(T::NT), T::LDS_BYTES, stream, p);
  return hipGetLastError();
}

// The instances whose output is NCHW: no residual form, no split-K (the reduction kernel writes NHWC).
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int XMODE, int NS>
hipError_t launch_fprop_dma_nchw(const FpropParams& p, hipStream_t stream) {
  using T = FpropDmaTraits<BM, BN, BK, WAVES_M, WAVES_N, XMODE, NS, 1>;
  auto kern = fprop_dma_kernel<BM, BN, BK, WAVES_M, WAVES_N, XMODE, NS, 1, false, true>;
  static LdsOptIn opt_in;
  if (hipError_t e = opt_in.ensure((const void*)kern, T::LDS_BYTES); e != hipSuccess) return e;
  dim3 grid(p.tiles_m * p.tiles_n, 1, 1);
  hipLaunchKernelGGL(kern, grid, dim3(T::NT), T::LDS_BYTES, stream, p);
  return hipGetLastError();
}
#define BOLT_FPROP_DMA_NCHW_INSTANCE(BM, BN, BK, WM, WN, NS, XMODE)                                     \
  {                                                                                                     \
    "dma_nchw_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS, BM, BN, BK, WM, WN, XMODE, 0, NS,          \
        bolt::FpropDmaTraits<BM, BN, BK, WM, WN, XMODE, NS>::LDS_BYTES,                                  \
        &bolt::launch_fprop_dma_nchw<BM, BN, BK, WM, WN, XMODE, NS>, nullptr, nullptr, 0, 0, true, true  \
  }

#define BOLT_FPROP_DMA_INSTANCE(BM, BN, BK, WM, WN, NS, XMODE)                                          \
  {                                                                                                     \
    "dma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS, BM, BN, BK, WM, WN, XMODE, 0, NS,               \
        bolt::FpropDmaTraits<BM, BN, BK, WM, WN, XMODE, NS>::LDS_BYTES,                                  \
        &bolt::launch_fprop_dma<BM, BN, BK, WM, WN, XMODE, NS>, nullptr, nullptr                        \
  }

// GEMM with row-major weights [K][N] (wmode 1): X(BM, BN, BK, WM, WN, NS, KG).
#define BOLT_FPROP_DMA_KN_INSTANCE(BM, BN, BK, WM, WN, NS, KG)                                          \
  {                                                                                                     \
    "dmakn_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS "_kg" #KG, BM, BN, BK, WM, WN, 0, 1, NS,       \
        bolt::FpropDmaTraits<BM, BN, BK, WM, WN, 0, NS, KG>::LDS_BYTES,                                  \
        &bolt::launch_fprop_dma<BM, BN, BK, WM, WN, 0, NS, KG, true>, nullptr, nullptr, KG, 0, false,  \
        false, true                                                                                     \
  }

// The same kernel with KG k-groups (64 * WM * WN * KG threads).
#define BOLT_FPROP_DMA_KG_INSTANCE(BM, BN, BK, WM, WN, NS, XMODE, KG)                                   \
  {                                                                                                     \
    "dma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS "_kg" #KG, BM, BN, BK, WM, WN, XMODE, 0, NS,     \
        bolt::FpropDmaTraits<BM, BN, BK, WM, WN, XMODE, NS, KG>::LDS_BYTES,                              \
        &bolt::launch_fprop_dma<BM, BN, BK, WM, WN, XMODE, NS, KG>, nullptr, nullptr, KG                 \
  }

}  // namespace bolt
