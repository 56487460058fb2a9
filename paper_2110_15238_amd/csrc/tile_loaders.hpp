// Global -> register -> LDS tile movers used by all kernel templates.
//
// Every operand tile lands in LDS as [rows][BK] halves with K contiguous and the 16-byte chunk
// swizzle of lds_chunk_offset<BK>.  Global accesses are 128-bit (8 halves), which is why channel
// counts and leading dimensions must be multiples of 8 ("alignment 8" of Section 3.2.3, Kernel
// padding); the alignment-2 modes fetch the same chunks as four 32-bit pairs and only need even
// channel counts: they are the slow "unpadded" kernels that padding is measured against (Table 3).
// A tile is fetched into registers first (load) and written to LDS later (store) so the fetch of
// tile k+1 overlaps the MFMA work on tile k.
#pragma once
#include "bolt_device.hpp"

namespace bolt {

struct ConvGeom {
  int H, Wi, C, R, S, P, Q, stride_h, stride_w, pad_h, pad_w;
};

// Activation-side tile: ROWS output rows x BK reduction columns.
//   XMODE 0: rows of a row-major matrix with leading dimension ld.
//   XMODE 1: implicit im2col of an NHWC tensor: row m = (img, p, q), column k = (r, s, c); taps
//            outside the image read as zero.  Needs C % 8 == 0 so a chunk never straddles a tap.
//   XMODE 2: the same view for C % 2 == 0 (alignment 2): every pair of halves has its own tap,
//            bounds test and 32-bit load.
template <int ROWS, int BK, int NT, int XMODE>
struct XTileLoader {
  static constexpr int CH = BK / 8;
  static constexpr int RP = NT / CH;
  static constexpr int PASSES = ROWS / RP;
  static_assert(ROWS % RP == 0 && PASSES >= 1, "tile rows must be a multiple of the rows one pass covers");

  half8 r[PASSES];
  int xbase[XMODE != 0 ? PASSES : 1];
  int xhw[XMODE != 0 ? PASSES : 1];
  int cr, cs, cc;
  const half_t* g;
  int ld, rows_valid, K, lc, lr;

  __device__ __forceinline__ void init(const half_t* X, int ldx, int M, int K_, const ConvGeom& cg, int m0,
                                       int kt_begin, int tid) {
    lc = tid % CH;
    lr = tid / CH;
    K = K_;
    ld = ldx;
    rows_valid = M - m0;
    cr = cs = cc = 0;
    if constexpr (XMODE == 0) {
      g = X + (int64_t)m0 * ldx;
    } else {
      g = X;
      const int PQ = cg.P * cg.Q;
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        const int m = m0 + lr + i * RP;
        if (m < M) {
          const int img = m / PQ, rem = m - img * PQ;
          const int op = rem / cg.Q, oq = rem - op * cg.Q;
          const int ih0 = op * cg.stride_h - cg.pad_h, iw0 = oq * cg.stride_w - cg.pad_w;
          xbase[i] = ((img * cg.H + ih0) * cg.Wi + iw0) * cg.C;
          xhw[i] = (int)(((unsigned)ih0 << 16) | ((unsigned)iw0 & 0xffffu));
        } else {
          xbase[i] = 0;
          xhw[i] = (int)0x80008000u;  // far outside the image: every tap fails the bounds test
        }
      }
      const int k = kt_begin * BK + lc * 8;
      const int rs = k / cg.C;
      cc = k - rs * cg.C;
      cr = rs / cg.S;
      cs = rs - cr * cg.S;
    }
  }

  // Fetch k-tile kt.  In conv mode tiles must be requested in increasing order, one by one,
  // starting at the kt_begin given to init (the (r, s, c) cursor advances incrementally).
  __device__ __forceinline__ void load(int kt, const ConvGeom& cg) {
    const half8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    const int k = kt * BK + lc * 8;
    if constexpr (XMODE == 0) {
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        const int row = lr + i * RP;
        r[i] = (row < rows_valid && k < K) ? *(const half8*)(g + (int64_t)row * ld + k) : zero8;
      }
    } else {
      if constexpr (XMODE == 1) {
        const int delta = (cr * cg.Wi + cs) * cg.C + cc;
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
          const int ih = (xhw[i] >> 16) + cr, iw = (int)(short)(xhw[i] & 0xffff) + cs;
          const bool ok = k < K && (unsigned)ih < (unsigned)cg.H && (unsigned)iw < (unsigned)cg.Wi;
          r[i] = ok ? *(const half8*)(g + (xbase[i] + delta)) : zero8;
        }
      } else {
        uintx4 v[PASSES];
        int pr = cr, ps = cs, pc = cc;  // tap of the current pair
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int delta = (pr * cg.Wi + ps) * cg.C + pc;
          const bool k_ok = k + 2 * j < K;
#pragma unroll
          for (int i = 0; i < PASSES; ++i) {
            const int ih = (xhw[i] >> 16) + pr, iw = (int)(short)(xhw[i] & 0xffff) + ps;
            const bool ok = k_ok && (unsigned)ih < (unsigned)cg.H && (unsigned)iw < (unsigned)cg.Wi;
            v[i][j] = ok ? *(const unsigned*)(g + (xbase[i] + delta)) : 0u;
          }
          pc += 2;
          if (pc >= cg.C) {  // C is even: a pair never straddles a tap
            pc = 0;
            if (++ps == cg.S) {
              ps = 0;
              ++pr;
            }
          }
        }
#pragma unroll
        for (int i = 0; i < PASSES; ++i) r[i] = __builtin_bit_cast(half8, v[i]);
      }
      cc += BK;
      while (cc >= cg.C) {
        cc -= cg.C;
        if (++cs == cg.S) {
          cs = 0;
          ++cr;
        }
      }
    }
  }

  __device__ __forceinline__ void store(half_t* dst) const {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) *(half8*)(dst + lds_chunk_offset<BK>(lr + i * RP, lc)) = r[i];
  }
};

// Weight-side tile: ROWS output channels x BK reduction columns.
//   WMODE 0: source is [N][K] with leading dimension ld (K contiguous).
//   WMODE 1: source is [K][N] with leading dimension ld (N contiguous): each thread fetches an
//            8(k) x 8(n) block as 8 row chunks and writes its transpose as 8 column chunks.
//   WMODE 2: as WMODE 0 with an even (not 8-divisible) ld and K: four 32-bit loads per chunk.
template <int ROWS, int BK, int NT, int WMODE>
struct WTileLoader {
  static constexpr int CH = BK / 8;
  static constexpr int RP = NT / CH;
  static constexpr int PASSES = (ROWS + RP - 1) / RP;       // WMODE 0, 2
  static constexpr int NB = (BK / 8) * (ROWS / 8);          // WMODE 1: 8x8 blocks in the tile
  static constexpr int KP = (NB + NT - 1) / NT;
  static constexpr bool RAGGED0 = (ROWS % RP) != 0;
  static constexpr bool RAGGED1 = (NB % NT) != 0;

  half8 r[WMODE != 1 ? PASSES : KP * 8];
  const half_t* g;
  int ld, rows_valid, K, tid;

  __device__ __forceinline__ void init(const half_t* W, int ldw, int N, int K_, int n0, int tid_) {
    tid = tid_;
    K = K_;
    ld = ldw;
    rows_valid = N - n0;
    g = (WMODE != 1) ? W + (int64_t)n0 * ldw : W + n0;
  }

  __device__ __forceinline__ void load(int kt) {
    const half8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (WMODE == 0) {
      const int lc = tid % CH, lr = tid / CH;
      const int k = kt * BK + lc * 8;
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        const int row = lr + i * RP;
        const bool ok = (!RAGGED0 || row < ROWS) && row < rows_valid && k < K;
        r[i] = ok ? *(const half8*)(g + (int64_t)row * ld + k) : zero8;
      }
    } else if constexpr (WMODE == 2) {
      const int lc = tid % CH, lr = tid / CH;
      const int k = kt * BK + lc * 8;
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        const int row = lr + i * RP;
        const bool ok = (!RAGGED0 || row < ROWS) && row < rows_valid;
        uintx4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          v[j] = (ok && k + 2 * j < K) ? *(const unsigned*)(g + (int64_t)row * ld + k + 2 * j) : 0u;
        r[i] = __builtin_bit_cast(half8, v);
      }
    } else {
#pragma unroll
      for (int j = 0; j < KP; ++j) {
        const int blk = tid + j * NT;
        const int nb = blk % (ROWS / 8), kb = blk / (ROWS / 8);
        const bool in_tile = !RAGGED1 || blk < NB;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
          const int k = kt * BK + kb * 8 + jj;
          r[j * 8 + jj] = (in_tile && k < K && nb * 8 < rows_valid) ? *(const half8*)(g + (int64_t)k * ld + nb * 8) : zero8;
        }
      }
    }
  }

  __device__ __forceinline__ void store(half_t* dst) const {
    if constexpr (WMODE != 1) {
      const int lc = tid % CH, lr = tid / CH;
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        const int row = lr + i * RP;
        if (!RAGGED0 || row < ROWS) *(half8*)(dst + lds_chunk_offset<BK>(row, lc)) = r[i];
      }
    } else {
#pragma unroll
      for (int j = 0; j < KP; ++j) {
        const int blk = tid + j * NT;
        const int nb = blk % (ROWS / 8), kb = blk / (ROWS / 8);
        if (!RAGGED1 || blk < NB) {
#pragma unroll
          for (int nn = 0; nn < 8; ++nn) {
            half8 t;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) t[jj] = r[j * 8 + jj][nn];
            *(half8*)(dst + lds_chunk_offset<BK>(nb * 8 + nn, kb)) = t;
          }
        }
      }
    }
  }
};

}  // namespace bolt
