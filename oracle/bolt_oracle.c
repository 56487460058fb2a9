/*
 * CPU oracle for the Bolt hot path (arxiv 2110.15238).  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct definitions of what the GPU library computes.  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may call this; the product path never does.
 * Shares no code with the HIP library.
 *
 * All tensors are IEEE binary16 stored as uint16_t.  Every sum is accumulated in double, in index
 * order, and rounded once to binary16 (round-to-nearest-even) at the end.  The only
 * parallelism is an OpenMP "parallel for" over output rows, which does not touch the arithmetic
 * order inside an output element.
 *
 * What follows the paper:
 *   - ref_gemm:        D = act(alpha * A.B + beta * bias), bias broadcast along rows
 *                      (Eq. 1 of Section 3.1.1 with C0 a bias; epilogue patterns (i)-(iii) of
 *                      Section 3.1 "Prerequisite: Epilogue fusion").
 *   - ref_conv2d_nhwc: direct NHWC cross-correlation with zero padding, (kernel, stride, padding)
 *                      attributes as in Section 4.1.1 / Table 2, + BiasAdd + activation.
 *   - ref_b2b_*:       Eq. 1 then Eq. 2 as two explicit calls, the intermediate D0 materialised
 *                      in binary16 (the second op consumes FP16 operands).
 *   - ref_pad_channels: "Kernel padding" of Section 3.2.3: copy and zero the tail channels.
 *   - ref_im2col:      only used to pin the convolution against ref_gemm.
 *
 * Pins (tests/test_oracle_*.py): exhaustive binary16 round trip and RNE midpoints, numpy's own
 * double->half conversion, float64 library matmul / conv on small shapes, unit-impulse closed form,
 * identity 1x1, im2col.gemm equality, zero-padding invariance, integer-exact brute force.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_ACT_NONE = 0, REF_ACT_RELU = 1, REF_ACT_GELU = 2, REF_ACT_HARDSWISH = 3, REF_ACT_SOFTPLUS = 4 };

/* ---- binary16 <-> double, by bit manipulation ------------------------------------------- */

double bolt_ref_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1f;
  int f = h & 0x3ff;
  double v;
  if (e == 0) {
    v = ldexp((double)f, -24); /* subnormal or zero: f * 2^-24 */
  } else if (e == 31) {
    v = f ? NAN : INFINITY;
  } else {
    v = ldexp((double)(f | 0x400), e - 25); /* (1024+f) * 2^(e-15-10) */
  }
  return sign ? -v : v;
}

/* Round a double to the nearest binary16, ties to even; overflow goes to infinity. */
uint16_t bolt_ref_double_to_half(double v) {
  uint64_t bits;
  memcpy(&bits, &v, sizeof bits);
  uint16_t sign = (uint16_t)((bits >> 48) & 0x8000u);
  int e = (int)((bits >> 52) & 0x7ff);
  uint64_t m = bits & 0xFFFFFFFFFFFFFull;
  if (e == 0x7ff) return (uint16_t)(sign | 0x7c00u | (m ? 0x200u : 0)); /* inf / nan */
  if (e == 0) return sign;                 /* double zero or subnormal: far below half's range */
  int ue = e - 1023;                       /* unbiased exponent; value = 1.m * 2^ue */
  uint64_t sig = m | (1ull << 52);         /* 53-bit significand */
  int shift;                               /* number of low bits of sig to drop */
  int he;                                  /* resulting biased half exponent (0 for subnormal) */
  if (ue >= -14) { he = ue + 15; shift = 42; }       /* normal half: keep 11 bits */
  else { he = 0; shift = 42 + (-14 - ue); }          /* subnormal half: unit is 2^-24 */
  if (shift > 63) return sign;             /* below half of the smallest subnormal */
  uint64_t kept = sig >> shift;
  uint64_t rem = sig & ((1ull << shift) - 1);
  uint64_t halfway = 1ull << (shift - 1);
  if (rem > halfway || (rem == halfway && (kept & 1))) kept++;
  uint32_t out;
  if (he == 0) out = (uint32_t)kept;       /* kept == 0x400 becomes the smallest normal */
  else out = ((uint32_t)he << 10) + (uint32_t)(kept - 0x400); /* kept == 0x800 carries into he */
  if (out >= 0x7c00u) out = 0x7c00u;       /* overflow to infinity */
  return (uint16_t)(sign | out);
}

static double apply_act(double v, int act) {
  switch (act) {
    case REF_ACT_RELU: return v > 0.0 ? v : 0.0;
    case REF_ACT_GELU: return 0.5 * v * (1.0 + erf(v * 0.70710678118654752440));
    case REF_ACT_HARDSWISH: {
      double t = v + 3.0;
      t = t < 0.0 ? 0.0 : (t > 6.0 ? 6.0 : t);
      return v * t / 6.0;
    }
    case REF_ACT_SOFTPLUS: return v > 0.0 ? v + log1p(exp(-v)) : log1p(exp(v));
    default: return v;
  }
}

static double epilogue(double s, float alpha, float beta, const uint16_t *bias, int n, int act) {
  double v = (double)alpha * s;
  if (bias) v += (double)beta * bolt_ref_half_to_double(bias[n]);
  return apply_act(v, act);
}

/* ---- stand-alone epilogue: out[m,n] = act(alpha * in[m,n] + beta * bias[n]) ----------------
 * The un-fused baseline of the epilogue-fusion experiment (Section 4.1.1): the GEMM writes its
 * FP16 result, a second pass reads it back, applies bias and activation, and rounds again. */
void bolt_ref_bias_act(int64_t M, int64_t N, const uint16_t *in, int64_t ldi, const uint16_t *bias, float alpha,
                       float beta, int act, uint16_t *out, int64_t ldo) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n)
      out[m * ldo + n] = bolt_ref_double_to_half(
          epilogue(bolt_ref_half_to_double(in[m * ldi + n]), alpha, beta, bias, (int)n, act));
}

/* ---- GEMM: D[m,n] = act(alpha * sum_k A[m,k] B[k,n] + beta * bias[n]) -------------------- */

static double gemm_dot(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, int64_t m, int64_t n,
                       int64_t K) {
  double s = 0.0;
  for (int64_t k = 0; k < K; ++k)
    s += bolt_ref_half_to_double(A[m * lda + k]) * bolt_ref_half_to_double(B[k * ldb + n]);
  return s;
}

void bolt_ref_gemm(int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B,
                   int64_t ldb, const uint16_t *bias, float alpha, float beta, int act, uint16_t *D,
                   int64_t ldd) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n)
      D[m * ldd + n] = bolt_ref_double_to_half(epilogue(gemm_dot(A, lda, B, ldb, m, n, K), alpha, beta, bias, (int)n, act));
}

/* Selected outputs only: idx[i] = m * N + n. */
void bolt_ref_gemm_at(int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B,
                      int64_t ldb, const uint16_t *bias, float alpha, float beta, int act, int64_t count,
                      const int64_t *idx, uint16_t *out) {
  (void)M;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    int64_t m = idx[i] / N, n = idx[i] % N;
    out[i] = bolt_ref_double_to_half(epilogue(gemm_dot(A, lda, B, ldb, m, n, K), alpha, beta, bias, (int)n, act));
  }
}

/* ---- direct NHWC convolution (cross-correlation), weights [K][R][S][C] ------------------- */

typedef struct {
  int64_t N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w;
} conv_dims;

static int64_t out_extent(int64_t in, int64_t pad, int64_t filt, int64_t stride) {
  return (in + 2 * pad - filt) / stride + 1;
}

static double conv_dot(const conv_dims *d, const uint16_t *x, const uint16_t *w, int64_t n, int64_t p, int64_t q,
                       int64_t k) {
  double s = 0.0;
  for (int64_t r = 0; r < d->R; ++r) {
    int64_t ih = p * d->stride_h - d->pad_h + r;
    for (int64_t ss = 0; ss < d->S; ++ss) {
      int64_t iw = q * d->stride_w - d->pad_w + ss;
      if (ih < 0 || ih >= d->H || iw < 0 || iw >= d->W) continue; /* zero padding */
      const uint16_t *xp = x + ((n * d->H + ih) * d->W + iw) * d->C;
      const uint16_t *wp = w + ((k * d->R + r) * d->S + ss) * d->C;
      for (int64_t c = 0; c < d->C; ++c) s += bolt_ref_half_to_double(xp[c]) * bolt_ref_half_to_double(wp[c]);
    }
  }
  return s;
}

void bolt_ref_conv2d_nhwc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                          int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, const uint16_t *x,
                          const uint16_t *w, const uint16_t *bias, float alpha, float beta, int act,
                          uint16_t *y) {
  conv_dims d = {N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w};
  int64_t P = out_extent(H, pad_h, R, stride_h), Q = out_extent(W, pad_w, S, stride_w);
#pragma omp parallel for schedule(static)
  for (int64_t row = 0; row < N * P * Q; ++row) {
    int64_t n = row / (P * Q), p = (row / Q) % P, q = row % Q;
    for (int64_t k = 0; k < K; ++k)
      y[row * K + k] = bolt_ref_double_to_half(epilogue(conv_dot(&d, x, w, n, p, q, k), alpha, beta, bias, (int)k, act));
  }
}

/* Selected outputs only: idx[i] = ((n*P + p)*Q + q)*K + k. */
void bolt_ref_conv2d_nhwc_at(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                             int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, const uint16_t *x,
                             const uint16_t *w, const uint16_t *bias, float alpha, float beta, int act,
                             int64_t count, const int64_t *idx, uint16_t *out) {
  conv_dims d = {N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w};
  int64_t P = out_extent(H, pad_h, R, stride_h), Q = out_extent(W, pad_w, S, stride_w);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    int64_t row = idx[i] / K, k = idx[i] % K;
    int64_t n = row / (P * Q), p = (row / Q) % P, q = row % Q;
    out[i] = bolt_ref_double_to_half(epilogue(conv_dot(&d, x, w, n, p, q, k), alpha, beta, bias, (int)k, act));
  }
}

/* ---- Eq. 1 with C a full pre-existing matrix (the skip connection of a residual block) ------------
 * D[m,n] = act(alpha * sum_k A[m,k] B[k,n] + beta * bias[n] + gamma * C[m,n]); C is FP16, ldc elements
 * per row.  The convolution form takes C in the output's NHWC layout. */
static double epilogue_residual(double s, float alpha, float beta, const uint16_t *bias, int n, float gamma,
                                uint16_t c, int act) {
  double v = (double)alpha * s;
  if (bias) v += (double)beta * bolt_ref_half_to_double(bias[n]);
  v += (double)gamma * bolt_ref_half_to_double(c);
  return apply_act(v, act);
}

void bolt_ref_gemm_residual(int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B,
                            int64_t ldb, const uint16_t *bias, const uint16_t *C, int64_t ldc, float alpha,
                            float beta, float gamma, int act, uint16_t *D, int64_t ldd) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n)
      D[m * ldd + n] = bolt_ref_double_to_half(
          epilogue_residual(gemm_dot(A, lda, B, ldb, m, n, K), alpha, beta, bias, (int)n, gamma, C[m * ldc + n], act));
}

void bolt_ref_conv2d_nhwc_residual(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                                   int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                   const uint16_t *x, const uint16_t *w, const uint16_t *bias, const uint16_t *res,
                                   float alpha, float beta, float gamma, int act, uint16_t *y) {
  conv_dims d = {N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w};
  int64_t P = out_extent(H, pad_h, R, stride_h), Q = out_extent(W, pad_w, S, stride_w);
#pragma omp parallel for schedule(static)
  for (int64_t row = 0; row < N * P * Q; ++row) {
    int64_t n = row / (P * Q), p = (row / Q) % P, q = row % Q;
    for (int64_t k = 0; k < K; ++k)
      y[row * K + k] = bolt_ref_double_to_half(
          epilogue_residual(conv_dot(&d, x, w, n, p, q, k), alpha, beta, bias, (int)k, gamma, res[row * K + k], act));
  }
}

/* ---- back-to-back chains: two explicit ops, D0 stored as binary16 ------------------------ */

void bolt_ref_b2b_gemm(int64_t M, int64_t N0, int64_t K0, int64_t N1, const uint16_t *A0, int64_t lda,
                       const uint16_t *W0, int64_t ldw0, const uint16_t *b0, float alpha0, float beta0,
                       int act0, const uint16_t *W1, int64_t ldw1, const uint16_t *b1, float alpha1,
                       float beta1, int act1, uint16_t *D1, int64_t ldd) {
  uint16_t *D0 = (uint16_t *)malloc((size_t)(M * N0 > 0 ? M * N0 : 1) * sizeof(uint16_t));
  bolt_ref_gemm(M, N0, K0, A0, lda, W0, ldw0, b0, alpha0, beta0, act0, D0, N0);
  bolt_ref_gemm(M, N1, N0, D0, N0, W1, ldw1, b1, alpha1, beta1, act1, D1, ldd);
  free(D0);
}

/* conv0 is general; conv1 is 1x1, stride 1, no padding, C1 = K0. */
void bolt_ref_b2b_conv(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K0, int64_t R, int64_t S,
                       int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, int64_t K1,
                       const uint16_t *x, const uint16_t *w0, const uint16_t *b0, float alpha0, float beta0,
                       int act0, const uint16_t *w1, const uint16_t *b1, float alpha1, float beta1, int act1,
                       uint16_t *y) {
  int64_t P = out_extent(H, pad_h, R, stride_h), Q = out_extent(W, pad_w, S, stride_w);
  int64_t rows = N * P * Q;
  uint16_t *y0 = (uint16_t *)malloc((size_t)(rows * K0 > 0 ? rows * K0 : 1) * sizeof(uint16_t));
  bolt_ref_conv2d_nhwc(N, H, W, C, K0, R, S, stride_h, stride_w, pad_h, pad_w, x, w0, b0, alpha0, beta0, act0, y0);
  bolt_ref_conv2d_nhwc(N, P, Q, K0, K1, 1, 1, 1, 1, 0, 0, y0, w1, b1, alpha1, beta1, act1, y);
  free(y0);
}

/* Selected rows of a b2b conv: rows[i] = (n*P + p)*Q + q; out gets K1 values per row. */
void bolt_ref_b2b_conv_rows(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K0, int64_t R, int64_t S,
                            int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, int64_t K1,
                            const uint16_t *x, const uint16_t *w0, const uint16_t *b0, float alpha0,
                            float beta0, int act0, const uint16_t *w1, const uint16_t *b1, float alpha1,
                            float beta1, int act1, int64_t count, const int64_t *rows, uint16_t *out) {
  conv_dims d = {N, H, W, C, K0, R, S, stride_h, stride_w, pad_h, pad_w};
  int64_t P = out_extent(H, pad_h, R, stride_h), Q = out_extent(W, pad_w, S, stride_w);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    int64_t row = rows[i];
    int64_t n = row / (P * Q), p = (row / Q) % P, q = row % Q;
    uint16_t *d0 = (uint16_t *)malloc((size_t)K0 * sizeof(uint16_t));
    for (int64_t k = 0; k < K0; ++k)
      d0[k] = bolt_ref_double_to_half(epilogue(conv_dot(&d, x, w0, n, p, q, k), alpha0, beta0, b0, (int)k, act0));
    for (int64_t k1 = 0; k1 < K1; ++k1) {
      double s = 0.0;
      for (int64_t c = 0; c < K0; ++c) s += bolt_ref_half_to_double(d0[c]) * bolt_ref_half_to_double(w1[k1 * K0 + c]);
      out[i * K1 + k1] = bolt_ref_double_to_half(epilogue(s, alpha1, beta1, b1, (int)k1, act1));
    }
    free(d0);
  }
}

/* ---- helpers ------------------------------------------------------------------------------ */

/* dst[pix, 0:C] = src[pix, 0:C]; dst[pix, C:C8] = 0 */
void bolt_ref_pad_channels(const uint16_t *src, uint16_t *dst, int64_t pixels, int64_t C, int64_t C8) {
  for (int64_t p = 0; p < pixels; ++p) {
    for (int64_t c = 0; c < C; ++c) dst[p * C8 + c] = src[p * C + c];
    for (int64_t c = C; c < C8; ++c) dst[p * C8 + c] = 0;
  }
}

/* Layout transformation (Section 3.2.3): dst[n, h, w, c] = src[n, c, h, w] for c < C, 0 for C <= c < C8. */
void bolt_ref_nchw_to_nhwc(const uint16_t *src, uint16_t *dst, int64_t N, int64_t C, int64_t H, int64_t W, int64_t C8) {
  for (int64_t n = 0; n < N; ++n)
    for (int64_t h = 0; h < H; ++h)
      for (int64_t w = 0; w < W; ++w)
        for (int64_t c = 0; c < C8; ++c)
          dst[((n * H + h) * W + w) * C8 + c] = c < C ? src[((n * C + c) * H + h) * W + w] : 0;
}

/* ... and back: dst[n, c, h, w] = src[n, h, w, c] for c < C; src holds Cs >= C channels per pixel. */
void bolt_ref_nhwc_to_nchw(const uint16_t *src, uint16_t *dst, int64_t N, int64_t C, int64_t H, int64_t W, int64_t Cs) {
  for (int64_t n = 0; n < N; ++n)
    for (int64_t c = 0; c < C; ++c)
      for (int64_t h = 0; h < H; ++h)
        for (int64_t w = 0; w < W; ++w) dst[((n * C + c) * H + h) * W + w] = src[((n * H + h) * W + w) * Cs + c];
}

/* col[(n,p,q), (r,s,c)] = x[n, p*sh-ph+r, q*sw-pw+s, c] or 0 outside the image. */
void bolt_ref_im2col(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S, int64_t stride_h,
                     int64_t stride_w, int64_t pad_h, int64_t pad_w, const uint16_t *x, uint16_t *col) {
  int64_t P = out_extent(H, pad_h, R, stride_h), Q = out_extent(W, pad_w, S, stride_w);
  int64_t Kg = R * S * C;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t p = 0; p < P; ++p)
      for (int64_t q = 0; q < Q; ++q) {
        uint16_t *row = col + ((n * P + p) * Q + q) * Kg;
        for (int64_t r = 0; r < R; ++r)
          for (int64_t s = 0; s < S; ++s) {
            int64_t ih = p * stride_h - pad_h + r, iw = q * stride_w - pad_w + s;
            for (int64_t c = 0; c < C; ++c) {
              uint16_t v = 0;
              if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = x[((n * H + ih) * W + iw) * C + c];
              row[(r * S + s) * C + c] = v;
            }
          }
      }
}

int bolt_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
