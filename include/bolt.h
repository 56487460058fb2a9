/*
 * bolt.h -- C ABI of the MI355X (gfx950) implementation of Bolt's hardware-native kernel family
 * (arxiv 2110.15238): FP16 GEMM and implicit-GEMM NHWC conv2d with fused bias + activation
 * epilogues, persistent back-to-back (b2b) GEMM / conv fusion, channel padding, and the
 * light-weight profiler that picks template parameters per shape.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers to IEEE binary16 data unless stated otherwise.
 *     They are borrowed: the library never allocates, frees or keeps them.  Base pointers must be
 *     16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls enqueue work and
 *     return; they do not synchronise (bolt_tune does, it has to read timers).
 *   - `workspace` is a device buffer of at least bolt_workspace_bytes(...) bytes (may be NULL when
 *     that is 0).
 *   - The return value is the only error channel.  Descriptors are validated before anything is
 *     launched, so every error except BOLT_ERR_LAUNCH can be produced without a GPU.
 *   - Accumulation is FP32 on the matrix cores; the epilogue runs in FP32 and converts once to
 *     FP16 with round-to-nearest-even.
 *   - Alignment (Section 3.2.3, "Kernel padding"): 128-bit accesses need every channel count,
 *     reduction length and leading dimension to be a multiple of 8, else BOLT_ERR_ALIGNMENT;
 *     pad with bolt_pad_channels_nhwc first.  The one exception is the input channel count of
 *     bolt_conv2d_fprop_nhwc: an even C that is not a multiple of 8 is accepted and runs on slow
 *     alignment-2 kernels (32-bit accesses), the "unpadded" case that Table 3 measures padding
 *     against.  An odd C is BOLT_ERR_ALIGNMENT.
 */
#ifndef BOLT_H_
#define BOLT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BOLT_OK = 0,
  BOLT_ERR_INVALID_ARG = 1,     /* null pointer, non-positive size, unknown enum value        */
  BOLT_ERR_UNSUPPORTED = 2,     /* no compiled template instance can run this problem          */
  BOLT_ERR_ALIGNMENT = 3,       /* a size / leading dimension / pointer breaks the 8-half rule */
  BOLT_ERR_WORKSPACE = 4,       /* workspace missing or too small                              */
  BOLT_ERR_LAUNCH = 5,          /* the HIP runtime reported an error                           */
  BOLT_ERR_ILLEGAL_FUSION = 6   /* the two ops cannot be fused (Section 3.1.1 preconditions)   */
} bolt_status;

/* Epilogue activations (Section 3.1 pattern (i); Section 3.3 lists ReLU, GELU, Hardswish, Softplus). */
typedef enum {
  BOLT_ACT_NONE = 0,
  BOLT_ACT_RELU = 1,
  BOLT_ACT_GELU = 2,       /* 0.5 v (1 + erf(v / sqrt 2)) */
  BOLT_ACT_HARDSWISH = 3,  /* v * clamp(v + 3, 0, 6) / 6   */
  BOLT_ACT_SOFTPLUS = 4    /* log(1 + exp v)               */
} bolt_act;

typedef enum {
  BOLT_OP_GEMM = 0,
  BOLT_OP_CONV2D = 1,
  BOLT_OP_B2B_GEMM = 2,
  BOLT_OP_B2B_CONV = 3,
  BOLT_OP_GEMM_CHAIN3 = 4, /* three GEMMs fused (the *_chain entry points)                    */
  BOLT_OP_CONV_CHAIN3 = 5, /* a convolution and two 1x1 convolutions fused                    */
  BOLT_OP_B2B_GEMM_RES = 6, /* bolt_b2b_gemm_residual: the instances of BOLT_OP_B2B_GEMM, those  */
  BOLT_OP_B2B_CONV_RES = 7  /* without the residual epilogue unsupported; same for _CONV         */
} bolt_op;

/* Storage of a GEMM's second operand. */
typedef enum {
  BOLT_LAYOUT_KN = 0, /* B[k][n] at B[k*ldb + n]: row-major K x N                      */
  BOLT_LAYOUT_NK = 1  /* B[k][n] at B[n*ldb + k]: N x K, reduction index contiguous     */
} bolt_layout;

/* How a b2b kernel keeps the first op's output tile on chip (Section 3.1.1). */
typedef enum {
  BOLT_B2B_RF = 0,  /* register-file resident: each wave owns whole rows of D0            */
  BOLT_B2B_LDS = 1  /* LDS resident: D0 tile staged through LDS and shared between waves   */
} bolt_b2b_mode;

/*
 * The searched template parameters (Section 3.2.2: threadblock / warp / instruction shapes,
 * swizzling functor, stages, ...).  kernel_id selects a compiled instance of the op's table
 * (0 <= kernel_id < bolt_num_instances(op)); kernel_id = -1 (or a NULL config) lets the library
 * choose by a built-in rule.  swizzle and split_k are run-time knobs and are honoured as given
 * (0 is read as "off"; with a NULL config the rule also chooses the tile order, never split-K);
 * the remaining fields describe the instance and are filled in by bolt_tune /
 * bolt_instance_config, ignored on input.
 */
typedef struct {
  int32_t kernel_id;
  int32_t tile_m, tile_n, tile_k; /* workgroup tile                                              */
  int32_t waves_m, waves_n;       /* wave grid inside the workgroup (64-lane wavefronts)          */
  int32_t mfma_shape;             /* 32 = v_mfma_f32_32x32x16_f16, 16 = v_mfma_f32_16x16x32_f16    */
  int32_t stages;                 /* LDS buffers in the operand pipeline                          */
  int32_t swizzle;                /* 0: n-tile fastest; g>0: XCD-aware remap, bands of g m-tiles  */
  int32_t split_k;                /* >1: K split over workgroups, FP32 partials in the workspace  */
  int32_t b2b_mode;               /* bolt_b2b_mode, b2b ops only                                  */
} bolt_config;

/* D[M x N] = act(alpha * A[M x K] . B[K x N] + beta * bias[N])   (Eq. 1 with C0 = broadcast bias) */
typedef struct {
  int32_t M, N, K;
  int32_t lda, ldb, ldd; /* in elements; A and D are row-major                                   */
  float alpha, beta;
  int32_t act;           /* bolt_act                                                              */
  int32_t b_layout;      /* bolt_layout                                                           */
} bolt_gemm_desc;

/* Layout of a convolution's input or output tensor in memory (Section 3.2.3, Layout transformation:
 * done inside the first and the last layer's kernel instead of as passes of their own). */
typedef enum {
  BOLT_TENSOR_NHWC = 0, /* [N][H][W][C], channels contiguous: what every kernel computes in          */
  BOLT_TENSOR_NCHW = 1  /* [N][C][H][W].  As x_layout: the input of a first layer (C <= 4), whose   */
                        /* loader reads it in place - no bolt_nchw_to_nhwc pass, no padded copy.     */
                        /* As y_layout: the output [N][K][P][Q] of a last layer, written by the     */
                        /* kernel's own store - no bolt_nhwc_to_nchw pass.                           */
} bolt_tensor_layout;

/* y[N,P,Q,K] = act(alpha * conv(x[N,H,W,C], w[K,R,S,C]) + beta * bias[K]); cross-correlation,
 * zero padding, P = (H + 2 pad_h - R) / stride_h + 1 (floor), Q likewise; dilation 1, groups 1.
 * x_layout, y_layout: bolt_tensor_layout of x and y (0 = NHWC; a zero-initialised descriptor keeps the
 * defaults).  The weights are always [K][R][S][C].  y_layout = NCHW runs on a few general instances
 * (and on the first-layer kernels); it has no residual form, no split-K, and fused pairs / chains do
 * not take it (BOLT_ERR_UNSUPPORTED). */
typedef struct {
  int32_t N, H, W, C;
  int32_t K, R, S;
  int32_t stride_h, stride_w, pad_h, pad_w;
  float alpha, beta;
  int32_t act;      /* bolt_act */
  int32_t x_layout; /* bolt_tensor_layout */
  int32_t y_layout; /* bolt_tensor_layout */
} bolt_conv_desc;

/* GEMM + fused epilogue (Section 2.2 tiling; Section 3.1 epilogue fusion patterns (i)-(iii)).
 * A: M x K (lda), B per desc->b_layout (ldb), bias: N halves or NULL (beta term skipped),
 * D: M x N (ldd).  Requires K, N, lda, ldb, ldd multiples of 8. */
bolt_status bolt_gemm_epilogue(const bolt_gemm_desc* desc, const void* A, const void* B, const void* bias, void* D,
                               const bolt_config* config, void* workspace, size_t workspace_bytes, void* stream);

/* Implicit-GEMM NHWC forward convolution + fused epilogue (Section 3.2.3: NHWC only; workloads of
 * Section 4.1.1).  x: N*H*W*C, w: K*R*S*C, bias: K halves or NULL, y: N*P*Q*K.  Requires K a
 * multiple of 8.  C a multiple of 8: the fast (128-bit) kernels; another even C: the alignment-2
 * kernels (Table 3's "unpadded" side); C <= 4 of either parity, e.g. the 3 colour planes of a first
 * layer: the first-layer kernels, which read x without channel padding and, with
 * desc->x_layout = BOLT_TENSOR_NCHW, in NCHW (they need R * C <= 24, S <= 8, stride_w <= 2, else
 * BOLT_ERR_UNSUPPORTED; an odd C > 4 is BOLT_ERR_ALIGNMENT: pad it with bolt_pad_channels_nhwc). */
bolt_status bolt_conv2d_fprop_nhwc(const bolt_conv_desc* desc, const void* x, const void* w, const void* bias,
                                   void* y, const bolt_config* config, void* workspace, size_t workspace_bytes,
                                   void* stream);

/* bolt_gemm_epilogue for callers that cannot allocate device memory and have no workspace to hand over (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the FP32 partial sums of a
 * split-K config go to a fixed array of BOLT_NOALLOC_SCRATCH_BYTES that lives in the library's device image, one
 * copy per GPU, held until the process ends.  The call itself allocates and frees nothing.
 * Arguments, layouts, alignment rules and results are those of bolt_gemm_epilogue (all pointers device, FP16,
 * borrowed); a config with split_k <= 1 needs no scratch at all.
 * Errors: as bolt_gemm_epilogue; BOLT_ERR_WORKSPACE if split_k * M * N * 4 exceeds BOLT_NOALLOC_SCRATCH_BYTES
 * (nothing is launched); BOLT_ERR_LAUNCH if the array's address cannot be obtained on the current device.
 * The partial sums are fully overwritten before they are read, so nothing has to be cleared between calls; all
 * calls on one GPU share the one array, so two calls that overlap in time on the same GPU (different streams)
 * race on it: keep them on one stream or order them yourself. */
#define BOLT_NOALLOC_SCRATCH_BYTES (16u << 20)
bolt_status bolt_gemm_epilogue_noalloc(const bolt_gemm_desc* desc, const void* A, const void* B, const void* bias,
                                       void* D, const bolt_config* config, void* stream);

/* Persistent back-to-back GEMM (Eq. 1-2, Section 3.1.1): D0 = act0(alpha0 A0.W0 + beta0 b0) is
 * rounded to FP16 and stays on chip; D1 = act1(alpha1 D0.W1 + beta1 b1) is the only output.
 * Legal only if g1->M == g0->M and g1->K == g0->N (else BOLT_ERR_ILLEGAL_FUSION).  Threadblock
 * residence: the workgroup tile spans all of N0 and N1, so N0 <= 128, N1 <= 256 and W1 must fit
 * in LDS next to the streaming tiles (else BOLT_ERR_UNSUPPORTED); W0 may be of any depth K0.
 * Row-major weights (BOLT_LAYOUT_KN) are addressed with 32-bit byte offsets from their first element: a matrix with
 * rows * ldb * 2 >= 2^31 bytes is BOLT_ERR_UNSUPPORTED here and in the chain calls (bolt_gemm_epilogue has a slower
 * kernel for it).
 * g0->ldd and g1->lda are ignored (D0 is never stored). */
bolt_status bolt_b2b_gemm(const bolt_gemm_desc* g0, const bolt_gemm_desc* g1, const void* A0, const void* W0,
                          const void* b0, const void* W1, const void* b1, void* D1, const bolt_config* config,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Persistent back-to-back convolution: c0 is any supported conv, c1 must be 1x1, stride 1, no
 * padding, with c1->C == c0->K and c1's input extent equal to c0's output extent
 * (N, P0, Q0) (else BOLT_ERR_ILLEGAL_FUSION).  Same residence limits as bolt_b2b_gemm with
 * N0 = c0->K, N1 = c1->K. */
bolt_status bolt_b2b_conv(const bolt_conv_desc* c0, const bolt_conv_desc* c1, const void* x, const void* w0,
                          const void* b0, const void* w1, const void* b1, void* y, const bolt_config* config,
                          void* workspace, size_t workspace_bytes, void* stream);

/* The same two ops with Eq. 1's C as a full pre-existing matrix next to the broadcast bias (the skip
 * connection of a residual block, added before the activation):
 *   D[m, n] = act(alpha * (A . B)[m, n] + beta * bias[n] + gamma * C[m, n]).
 * C: device, FP16, M x N with row stride ldc (GEMM; ldc >= N, ldc % 8 == 0), or in the output's NHWC
 * layout N*P*Q*K (convolution).  C may be the output buffer itself (each element is read before it is
 * written, by the workgroup that owns it) unless split_k > 1.  Everything else as in the calls above;
 * a config tuned for the plain op is valid here unless it names one of the persistent weights-resident
 * instances (BOLT_ERR_UNSUPPORTED). */
bolt_status bolt_gemm_epilogue_residual(const bolt_gemm_desc* desc, const void* A, const void* B, const void* bias,
                                        const void* C, int32_t ldc, float gamma, void* D, const bolt_config* config,
                                        void* workspace, size_t workspace_bytes, void* stream);
bolt_status bolt_conv2d_fprop_nhwc_residual(const bolt_conv_desc* desc, const void* x, const void* w, const void* bias,
                                            const void* residual, float gamma, void* y, const bolt_config* config,
                                            void* workspace, size_t workspace_bytes, void* stream);

/* The fused pair with the same full-matrix C in the epilogue of its second op (Section 3.1.1's C1):
 *   D1 = act1(alpha1 * D0 . W1 + beta1 * b1 + gamma * C),  D0 as in bolt_b2b_gemm / bolt_b2b_conv.
 * With bolt_conv2d_fprop_nhwc for the first 1x1 this runs a residual bottleneck block (1x1, then
 * 3x3 -> 1x1 + skip connection + activation) in two launches.  C: M x N1 with row stride ldc (GEMM;
 * ldc >= N1, ldc % 8 == 0) or the output's NHWC layout (convolution); it may be the output buffer.
 * Only part of the fused instances have this epilogue: kernel_id indexes the BOLT_OP_B2B_GEMM /
 * BOLT_OP_B2B_CONV tables, an instance without it returns BOLT_ERR_UNSUPPORTED, and bolt_tune,
 * bolt_check, bolt_instance_supports take BOLT_OP_B2B_GEMM_RES / BOLT_OP_B2B_CONV_RES to restrict
 * themselves to the ones that have it (bolt_tune: ptrs = {x, w0, b0, w1, b1, y, C}, C dense). */
bolt_status bolt_b2b_gemm_residual(const bolt_gemm_desc* g0, const bolt_gemm_desc* g1, const void* A0, const void* W0,
                                   const void* b0, const void* W1, const void* b1, const void* C, int32_t ldc,
                                   float gamma, void* D1, const bolt_config* config, void* workspace,
                                   size_t workspace_bytes, void* stream);
bolt_status bolt_b2b_conv_residual(const bolt_conv_desc* c0, const bolt_conv_desc* c1, const void* x, const void* w0,
                                   const void* b0, const void* w1, const void* b1, const void* residual, float gamma,
                                   void* y, const bolt_config* config, void* workspace, size_t workspace_bytes,
                                   void* stream);

/* Persistent fusion of more than two ops (Section 3.1.1: the scheme extends to longer chains by
 * duplicating the pipeline; Section 3.3 deepens models with extra 1x1 convolutions that fuse this way).
 * n_ops = 3 is compiled; any other positive n_ops is BOLT_ERR_UNSUPPORTED.
 *   D_i = act_i(alpha_i * D_{i-1} . W_i + beta_i * bias_i),  D_{-1} = A0 (or the input image),
 * every D_i but the last stays in registers, rounded to FP16 between ops as if it had been stored.
 * descs: host array of n_ops descriptor pointers.  Legality is that of bolt_b2b_gemm / bolt_b2b_conv
 * applied to each consecutive pair (else BOLT_ERR_ILLEGAL_FUSION): same M, K_i = N_{i-1}; for
 * convolutions every op after the first is 1x1, stride 1, no padding, on the previous op's output
 * extent.  The weight matrices of a GEMM chain share one layout (either one).  Each N_i must fit a
 * compiled bound (N_0, N_1 <= 128, N_2 <= 256), else BOLT_ERR_UNSUPPORTED.
 * weights, biases: host arrays of n_ops device pointers (biases, or single entries of it, may be NULL).
 * config->kernel_id indexes the instances of BOLT_OP_GEMM_CHAIN3 / BOLT_OP_CONV_CHAIN3. */
bolt_status bolt_b2b_gemm_chain(int32_t n_ops, const bolt_gemm_desc* const* descs, const void* A0,
                                const void* const* weights, const void* const* biases, void* D,
                                const bolt_config* config, void* stream);
bolt_status bolt_b2b_conv_chain(int32_t n_ops, const bolt_conv_desc* const* descs, const void* x,
                                const void* const* weights, const void* const* biases, void* y,
                                const bolt_config* config, void* stream);
/* The chain with Eq. 1's full-matrix C in the epilogue of its last op (Section 3.1.1, Eq. 1-2 with C a matrix,
 * taken by the op whose output is stored; Section 3.3's deepened blocks end in a skip connection):
 *   D_2 = act_2(alpha_2 * D_1 . W_2 + beta_2 * bias_2 + gamma * C),  D_0, D_1 as in the plain chain.
 * C: M x N_2 with row stride ldc (GEMM; ldc >= N_2 else BOLT_ERR_INVALID_ARG, ldc % 8 == 0 and C 16-byte
 * aligned else BOLT_ERR_ALIGNMENT) or the output's NHWC layout (convolution); device memory, read only, it
 * may be the output buffer.  Every chain instance has this epilogue: config, bolt_tune_chain, bolt_check_chain
 * and bolt_chain_instance_supports are those of the plain chain.  All other arguments and errors as above. */
bolt_status bolt_b2b_gemm_chain_residual(int32_t n_ops, const bolt_gemm_desc* const* descs, const void* A0,
                                         const void* const* weights, const void* const* biases, const void* C,
                                         int32_t ldc, float gamma, void* D, const bolt_config* config, void* stream);
bolt_status bolt_b2b_conv_chain_residual(int32_t n_ops, const bolt_conv_desc* const* descs, const void* x,
                                         const void* const* weights, const void* const* biases, const void* residual,
                                         float gamma, void* y, const bolt_config* config, void* stream);
/* bolt_tune for a chain: op is BOLT_OP_GEMM_CHAIN3 or BOLT_OP_CONV_CHAIN3, ptrs = {x, w0, b0, w1, b1,
 * w2, b2, y} (biases may be NULL).  Synchronises the stream; y is overwritten; nothing is cached. */
bolt_status bolt_tune_chain(bolt_op op, int32_t n_ops, const void* const* descs, const void* const* ptrs, void* stream,
                            bolt_config* best, float* best_ms, int32_t* n_tried);
/* Validation only (no GPU needed), and whether instance kernel_id can run the chain (1) or not (0). */
bolt_status bolt_check_chain(bolt_op op, int32_t n_ops, const void* const* descs, const bolt_config* config);
int32_t bolt_chain_instance_supports(bolt_op op, int32_t kernel_id, int32_t n_ops, const void* const* descs);

/* Light-weight profiler (Section 3.2.2): runs every compiled instance that is legal for the given
 * problem (and a few split-K / swizzle settings) on the caller's real buffers, times them with
 * HIP events and returns the fastest.  ptrs holds the device pointers of the op call in call order:
 *   GEMM  {A, B, bias, D}            CONV     {x, w, bias, y}
 *   B2B_GEMM {A0, W0, b0, W1, b1, D1}  B2B_CONV {x, w0, b0, w1, b1, y}
 * desc1 is NULL for single ops.  The output buffer is overwritten.  Synchronises the stream.
 * best_ms (may be NULL) receives the mean time per launch of the winner, n_tried (may be NULL) the
 * number of candidates timed.  Results are cached per (op, shape) for the life of the process.
 * With BOLT_TUNE_LOG=1 in the environment every candidate's time goes to stderr (and, for calls that
 * pass no config, every candidate's estimate under the built-in rule with the instance it picks). */
bolt_status bolt_tune(bolt_op op, const void* desc0, const void* desc1, const void* const* ptrs, void* workspace,
                      size_t workspace_bytes, void* stream, bolt_config* best, float* best_ms, int32_t* n_tried);

/* dst[p, 0:C] = src[p, 0:C], dst[p, C:C_padded] = 0 for p < pixels (Section 3.2.3, Kernel
 * padding).  C_padded >= C, C_padded % 8 == 0, pixels * C_padded < 2^34 (else BOLT_ERR_UNSUPPORTED).
 * src and dst must not overlap. */
bolt_status bolt_pad_channels_nhwc(const void* src, void* dst, int64_t pixels, int32_t C, int32_t C_padded,
                                   void* stream);

/* Layout transformation (Section 3.2.3: the kernels are NHWC only, frameworks hand over NCHW) into and out
 * of buffers the caller has pre-allocated, as the paper keeps them with the model's parameters.
 *   bolt_nchw_to_nhwc: dst[n, h, w, c] = src[n, c, h, w] for c < C, 0 for C <= c < C_padded: the transform
 *     of a network's first layer and its channel padding in one pass.  C_padded >= C, C_padded % 8 == 0.
 *   bolt_nhwc_to_nchw: dst[n, c, h, w] = src[n, h, w, c] for c < C, where src holds C_src >= C channels per
 *     pixel (C_src % 8 == 0): the transform of the last layer, dropping any padding.
 * FP16, device pointers, the NHWC side 16-byte aligned; src and dst must not overlap.  N <= 65535. */
bolt_status bolt_nchw_to_nhwc(const void* src, void* dst, int32_t N, int32_t C, int32_t H, int32_t W, int32_t C_padded,
                              void* stream);
bolt_status bolt_nhwc_to_nchw(const void* src, void* dst, int32_t N, int32_t C, int32_t H, int32_t W, int32_t C_src,
                              void* stream);

/* Stand-alone epilogue, in place: D[m, n] = act(alpha * D[m, n] + beta * bias[n]) for m < M, n < N,
 * FP16 in and out, arithmetic in FP32.  This is the separate element-wise pass that epilogue fusion
 * removes (Section 3.1; Section 4.1.1 measures the fused GEMM against GEMM followed by this pass);
 * it exists so that the comparison can be made.  D: device, row-major, row stride ldd >= N;
 * bias: device, N halves, or NULL (no bias term).  M == 0 is a no-op.  N % 8 == 0, ldd % 8 == 0, 16-byte aligned pointers. */
bolt_status bolt_bias_act(void* D, const void* bias, int64_t M, int32_t N, int32_t ldd, float alpha, float beta,
                          bolt_act act, void* stream);

/* Workspace bytes the op needs with this config (0 unless split_k > 1).  With config NULL: an
 * upper bound over everything bolt_tune may try for this problem. */
size_t bolt_workspace_bytes(bolt_op op, const void* desc0, const void* desc1, const bolt_config* config);

/* Validation only: the status the op call would return before launching anything (no GPU needed). */
bolt_status bolt_check(bolt_op op, const void* desc0, const void* desc1, const bolt_config* config);

const char* bolt_status_string(bolt_status s);

/* Number of compiled template instances of an op, and the description of instance kernel_id. */
int32_t bolt_num_instances(bolt_op op);
bolt_status bolt_instance_config(bolt_op op, int32_t kernel_id, bolt_config* out);
/* Whether instance kernel_id can run the described problem (1) or not (0). */
int32_t bolt_instance_supports(bolt_op op, int32_t kernel_id, const void* desc0, const void* desc1);

/* Measured roofline denominators: runs an MFMA-only loop of v_mfma_f32_16x16x32_f16 on pseudo-random FP16
 * operands, `iterations` x 16 instructions per wave, 8 waves per compute unit (returns the sustained FP16 TFLOP/s
 * under the chip's power limit), or a streaming copy of `bytes` bytes between two halves of `buffer` (returns
 * GB/s, read + write).  Neither allocates. */
bolt_status bolt_probe_mfma_peak(int32_t iterations, void* stream, float* tflops);
bolt_status bolt_probe_copy_bandwidth(void* buffer, size_t bytes, int32_t repeats, void* stream, float* gbps);

#ifdef __cplusplus
}
#endif
#endif /* BOLT_H_ */
