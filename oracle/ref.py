"""ctypes front end of the CPU oracle (oracle/bolt_oracle.c).  TEST INFRASTRUCTURE ONLY.

Argument marshalling only: numpy float16 arrays in, numpy float16 arrays out.  Nothing here is
imported by the product package; nothing here imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bolt_oracle.c")
_LIB = os.path.join(_HERE, "libbolt_oracle.so")

ACT = {"none": 0, "relu": 1, "gelu": 2, "hardswish": 3, "softplus": 4}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None
_i64, _f32, _int, _p = C.c_int64, C.c_float, C.c_int, C.c_void_p


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.bolt_ref_half_to_double.restype = C.c_double
        L.bolt_ref_half_to_double.argtypes = [C.c_uint16]
        L.bolt_ref_double_to_half.restype = C.c_uint16
        L.bolt_ref_double_to_half.argtypes = [C.c_double]
        L.bolt_ref_bias_act.restype = None
        L.bolt_ref_bias_act.argtypes = [_i64, _i64, _p, _i64, _p, _f32, _f32, _int, _p, _i64]
        L.bolt_ref_nchw_to_nhwc.restype = None
        L.bolt_ref_nchw_to_nhwc.argtypes = [_p, _p, _i64, _i64, _i64, _i64, _i64]
        L.bolt_ref_nhwc_to_nchw.restype = None
        L.bolt_ref_nhwc_to_nchw.argtypes = [_p, _p, _i64, _i64, _i64, _i64, _i64]
        L.bolt_ref_gemm_residual.restype = None
        L.bolt_ref_gemm_residual.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _p, _p, _i64, _f32, _f32, _f32, _int,
                                             _p, _i64]
        L.bolt_ref_conv2d_nhwc_residual.restype = None
        L.bolt_ref_conv2d_nhwc_residual.argtypes = [_i64] * 11 + [_p, _p, _p, _p, _f32, _f32, _f32, _int, _p]
        L.bolt_ref_gemm.restype = None
        L.bolt_ref_gemm.argtypes = [_i64] * 3 + [_p, _i64, _p, _i64, _p, _f32, _f32, _int, _p, _i64]
        L.bolt_ref_gemm_at.restype = None
        L.bolt_ref_gemm_at.argtypes = [_i64] * 3 + [_p, _i64, _p, _i64, _p, _f32, _f32, _int, _i64, _p, _p]
        L.bolt_ref_conv2d_nhwc.restype = None
        L.bolt_ref_conv2d_nhwc.argtypes = [_i64] * 11 + [_p, _p, _p, _f32, _f32, _int, _p]
        L.bolt_ref_conv2d_nhwc_at.restype = None
        L.bolt_ref_conv2d_nhwc_at.argtypes = [_i64] * 11 + [_p, _p, _p, _f32, _f32, _int, _i64, _p, _p]
        L.bolt_ref_b2b_gemm.restype = None
        L.bolt_ref_b2b_gemm.argtypes = ([_i64] * 4 + [_p, _i64, _p, _i64, _p, _f32, _f32, _int,
                                                      _p, _i64, _p, _f32, _f32, _int, _p, _i64])
        L.bolt_ref_b2b_conv.restype = None
        L.bolt_ref_b2b_conv.argtypes = ([_i64] * 12 + [_p, _p, _p, _f32, _f32, _int, _p, _p, _f32, _f32, _int, _p])
        L.bolt_ref_b2b_conv_rows.restype = None
        L.bolt_ref_b2b_conv_rows.argtypes = ([_i64] * 12 + [_p, _p, _p, _f32, _f32, _int, _p, _p, _f32, _f32, _int,
                                                            _i64, _p, _p])
        L.bolt_ref_pad_channels.restype = None
        L.bolt_ref_pad_channels.argtypes = [_p, _p, _i64, _i64, _i64]
        L.bolt_ref_im2col.restype = None
        L.bolt_ref_im2col.argtypes = [_i64] * 10 + [_p, _p]
        L.bolt_ref_num_threads.restype = _int
    return _lib


def num_threads() -> int:
    return int(lib().bolt_ref_num_threads())


def _h(a: np.ndarray) -> np.ndarray:
    assert a.dtype == np.float16, a.dtype
    return np.ascontiguousarray(a)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def half_to_double(bits: int) -> float:
    return float(lib().bolt_ref_half_to_double(int(bits)))


def double_to_half(v: float) -> int:
    return int(lib().bolt_ref_double_to_half(float(v)))


def out_hw(H, W, R, S, stride, pad):
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    return (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1, sh, sw, ph, pw


def bias_act(X, bias=None, alpha=1.0, beta=1.0, act="relu"):
    """Stand-alone epilogue on an FP16 matrix: act(alpha * X + beta * bias) -> float16 (Section 4.1.1's un-fused baseline)."""
    X = _h(X)
    M, N = X.shape
    bias = None if bias is None else _h(bias)
    out = np.empty((M, N), np.float16)
    lib().bolt_ref_bias_act(M, N, _ptr(X), N, _ptr(bias), alpha, beta, ACT[act], _ptr(out), N)
    return out


def gemm(A, B, bias=None, alpha=1.0, beta=1.0, act="relu"):
    """A[M,K] . B[K,N] (both row-major) -> D[M,N] float16."""
    A, B = _h(A), _h(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    bias = None if bias is None else _h(bias)
    D = np.empty((M, N), np.float16)
    lib().bolt_ref_gemm(M, N, K, _ptr(A), K, _ptr(B), N, _ptr(bias), alpha, beta, ACT[act], _ptr(D), N)
    return D


def gemm_at(A, B, idx, bias=None, alpha=1.0, beta=1.0, act="relu"):
    A, B = _h(A), _h(B)
    M, K = A.shape
    _, N = B.shape
    bias = None if bias is None else _h(bias)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, np.float16)
    lib().bolt_ref_gemm_at(M, N, K, _ptr(A), K, _ptr(B), N, _ptr(bias), alpha, beta, ACT[act], idx.size,
                           _ptr(idx), _ptr(out))
    return out


def conv2d_nhwc(x, w, bias=None, stride=1, pad=0, alpha=1.0, beta=1.0, act="relu"):
    """x[N,H,W,C], w[K,R,S,C] -> y[N,P,Q,K] float16."""
    x, w = _h(x), _h(w)
    N, H, W, Cc = x.shape
    K, R, S, C2 = w.shape
    assert Cc == C2
    P, Q, sh, sw, ph, pw = out_hw(H, W, R, S, stride, pad)
    bias = None if bias is None else _h(bias)
    y = np.empty((N, P, Q, K), np.float16)
    lib().bolt_ref_conv2d_nhwc(N, H, W, Cc, K, R, S, sh, sw, ph, pw, _ptr(x), _ptr(w), _ptr(bias), alpha, beta,
                               ACT[act], _ptr(y))
    return y


def conv2d_nhwc_at(x, w, idx, bias=None, stride=1, pad=0, alpha=1.0, beta=1.0, act="relu"):
    """Outputs at flat positions idx (into y[N,P,Q,K]) only."""
    x, w = _h(x), _h(w)
    N, H, W, Cc = x.shape
    K, R, S, _ = w.shape
    P, Q, sh, sw, ph, pw = out_hw(H, W, R, S, stride, pad)
    bias = None if bias is None else _h(bias)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, np.float16)
    lib().bolt_ref_conv2d_nhwc_at(N, H, W, Cc, K, R, S, sh, sw, ph, pw, _ptr(x), _ptr(w), _ptr(bias), alpha, beta,
                                  ACT[act], idx.size, _ptr(idx), _ptr(out))
    return out


def b2b_gemm(A, W0, b0, W1, b1, alpha0=1.0, beta0=1.0, act0="relu", alpha1=1.0, beta1=1.0, act1="relu"):
    A, W0, W1 = _h(A), _h(W0), _h(W1)
    M, K0 = A.shape
    _, N0 = W0.shape
    _, N1 = W1.shape
    assert W0.shape[0] == K0 and W1.shape[0] == N0
    b0 = None if b0 is None else _h(b0)
    b1 = None if b1 is None else _h(b1)
    D1 = np.empty((M, N1), np.float16)
    lib().bolt_ref_b2b_gemm(M, N0, K0, N1, _ptr(A), K0, _ptr(W0), N0, _ptr(b0), alpha0, beta0, ACT[act0],
                            _ptr(W1), N1, _ptr(b1), alpha1, beta1, ACT[act1], _ptr(D1), N1)
    return D1


def b2b_conv(x, w0, b0, w1, b1, stride=1, pad=0, alpha0=1.0, beta0=1.0, act0="relu", alpha1=1.0, beta1=1.0,
             act1="relu"):
    x, w0, w1 = _h(x), _h(w0), _h(w1)
    N, H, W, Cc = x.shape
    K0, R, S, _ = w0.shape
    K1 = w1.shape[0]
    assert w1.shape[1:] == (1, 1, K0)
    P, Q, sh, sw, ph, pw = out_hw(H, W, R, S, stride, pad)
    b0 = None if b0 is None else _h(b0)
    b1 = None if b1 is None else _h(b1)
    y = np.empty((N, P, Q, K1), np.float16)
    lib().bolt_ref_b2b_conv(N, H, W, Cc, K0, R, S, sh, sw, ph, pw, K1, _ptr(x), _ptr(w0), _ptr(b0), alpha0, beta0,
                            ACT[act0], _ptr(w1), _ptr(b1), alpha1, beta1, ACT[act1], _ptr(y))
    return y


def b2b_conv_rows(x, w0, b0, w1, b1, rows, stride=1, pad=0, alpha0=1.0, beta0=1.0, act0="relu", alpha1=1.0,
                  beta1=1.0, act1="relu"):
    """Full K1-wide output rows at flat pixel indices `rows` (into [N*P*Q])."""
    x, w0, w1 = _h(x), _h(w0), _h(w1)
    N, H, W, Cc = x.shape
    K0, R, S, _ = w0.shape
    K1 = w1.shape[0]
    P, Q, sh, sw, ph, pw = out_hw(H, W, R, S, stride, pad)
    b0 = None if b0 is None else _h(b0)
    b1 = None if b1 is None else _h(b1)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    out = np.empty((rows.size, K1), np.float16)
    lib().bolt_ref_b2b_conv_rows(N, H, W, Cc, K0, R, S, sh, sw, ph, pw, K1, _ptr(x), _ptr(w0), _ptr(b0), alpha0,
                                 beta0, ACT[act0], _ptr(w1), _ptr(b1), alpha1, beta1, ACT[act1], rows.size,
                                 _ptr(rows), _ptr(out))
    return out


def gemm_residual(A, B, bias, C, alpha=1.0, beta=1.0, gamma=1.0, act="relu"):
    """act(alpha * A @ B + beta * bias + gamma * C) -> float16; Eq. 1 with a full matrix C (B is [K][N])."""
    A, B, C = _h(A), _h(B), _h(C)
    M, K = A.shape
    N = B.shape[1]
    assert B.shape[0] == K and C.shape == (M, N)
    bias = None if bias is None else _h(bias)
    D = np.empty((M, N), np.float16)
    lib().bolt_ref_gemm_residual(M, N, K, _ptr(A), K, _ptr(B), N, _ptr(bias), _ptr(C), N, alpha, beta, gamma, ACT[act],
                                 _ptr(D), N)
    return D


def conv2d_nhwc_residual(x, w, bias, res, stride=1, pad=0, alpha=1.0, beta=1.0, gamma=1.0, act="relu"):
    """act(alpha * conv(x, w) + beta * bias + gamma * res), res in the output's NHWC layout."""
    x, w, res = _h(x), _h(w), _h(res)
    N, H, W, Cc = x.shape
    K, R, S, _ = w.shape
    P, Q, sh, sw, ph, pw = out_hw(H, W, R, S, stride, pad)
    assert res.shape == (N, P, Q, K)
    bias = None if bias is None else _h(bias)
    y = np.empty((N, P, Q, K), np.float16)
    lib().bolt_ref_conv2d_nhwc_residual(N, H, W, Cc, K, R, S, sh, sw, ph, pw, _ptr(x), _ptr(w), _ptr(bias), _ptr(res),
                                        alpha, beta, gamma, ACT[act], _ptr(y))
    return y


def b2b_gemm_residual(A, W0, b0, W1, b1, C, gamma=1.0, act0="relu", act1="relu"):
    """Eq. 1-2 with Eq. 2's C1 a full matrix: D0 = act0(A W0 + b0) rounded to FP16 as if stored, then
    D1 = act1(D0 W1 + b1 + gamma C).  W0 is [K0][N0], W1 is [N0][N1], C is [M][N1]."""
    return gemm_residual(gemm(A, W0, b0, act=act0), W1, b1, C, gamma=gamma, act=act1)


def b2b_conv_residual(x, w0, b0, w1, b1, res, stride=1, pad=0, gamma=1.0, act0="relu", act1="relu"):
    """The convolution pair of Section 3.1.1 (any conv, then 1x1 / stride 1 / unpadded) with a full residual
    tensor in the second epilogue: the tail of a bottleneck block (3x3, 1x1, + skip connection, activation)."""
    assert w1.shape[1:3] == (1, 1)
    y0 = conv2d_nhwc(x, w0, b0, stride=stride, pad=pad, act=act0)
    return conv2d_nhwc_residual(y0, w1, b1, res, stride=1, pad=0, gamma=gamma, act=act1)


def gemm_chain(A, Ws, bs, acts, alphas=None, betas=None):
    """Eq. 1-2 carried on to more ops (Section 3.1.1): D_i = act_i(alpha_i D_{i-1} W_i + beta_i b_i), every D_i
    rounded to FP16 before the next op reads it, as if it had been stored.  Ws[i] is [K_i][N_i]."""
    D = _h(A)
    for i, (W, b) in enumerate(zip(Ws, bs)):
        D = gemm(D, W, b, 1.0 if alphas is None else alphas[i], 1.0 if betas is None else betas[i], acts[i])
    return D


def conv_chain(x, ws, bs, acts, stride=1, pad=0):
    """A convolution followed by 1x1 / stride 1 / unpadded convolutions, FP16 between ops.  ws[i] is KRSC."""
    y = conv2d_nhwc(x, ws[0], bs[0], stride=stride, pad=pad, act=acts[0])
    for w, b, act in zip(ws[1:], bs[1:], acts[1:]):
        assert w.shape[1:3] == (1, 1)
        y = conv2d_nhwc(y, w, b, stride=1, pad=0, act=act)
    return y


def gemm_chain_residual(A, Ws, bs, acts, C, gamma=1.0):
    """The chain of gemm_chain with Eq. 1's full-matrix C in the epilogue of its LAST op only (Section 3.1.1: the
    pipeline of fused ops extended, Eq. 2's C1 taken by the op that produces the stored output):
    D_last = act_last(D_{last-1} W_last + b_last + gamma C); every earlier D_i is rounded to FP16 as if stored."""
    D = gemm_chain(A, Ws[:-1], bs[:-1], acts[:-1])
    return gemm_residual(D, Ws[-1], bs[-1], C, gamma=gamma, act=acts[-1])


def conv_chain_residual(x, ws, bs, acts, res, stride=1, pad=0, gamma=1.0):
    """conv_chain with a full residual tensor (the NHWC layout of the output) added in the last op's epilogue: a
    bottleneck block written as one chain (1x1 or 3x3, then 1x1s, + skip connection, activation; Section 3.3)."""
    y = conv_chain(x, ws[:-1], bs[:-1], acts[:-1], stride=stride, pad=pad)
    assert ws[-1].shape[1:3] == (1, 1)
    return conv2d_nhwc_residual(y, ws[-1], bs[-1], res, stride=1, pad=0, gamma=gamma, act=acts[-1])


def nchw_to_nhwc(src, C8=None):
    """[N][C][H][W] -> [N][H][W][C8], channels C..C8-1 zero (Section 3.2.3, layout transformation + padding)."""
    src = _h(src)
    N, Cc, H, W = src.shape
    C8 = Cc if C8 is None else C8
    dst = np.empty((N, H, W, C8), np.float16)
    lib().bolt_ref_nchw_to_nhwc(_ptr(src), _ptr(dst), N, Cc, H, W, C8)
    return dst


def nhwc_to_nchw(src, C=None):
    """[N][H][W][Cs] -> [N][C][H][W], keeping the first C channels."""
    src = _h(src)
    N, H, W, Cs = src.shape
    C = Cs if C is None else C
    dst = np.empty((N, C, H, W), np.float16)
    lib().bolt_ref_nhwc_to_nchw(_ptr(src), _ptr(dst), N, C, H, W, Cs)
    return dst


def pad_channels(src, C8):
    src = _h(src)
    Cc = src.shape[-1]
    pixels = src.size // Cc if Cc else 0
    dst = np.empty(src.shape[:-1] + (C8,), np.float16)
    lib().bolt_ref_pad_channels(_ptr(src), _ptr(dst), pixels, Cc, C8)
    return dst


def im2col(x, R, S, stride=1, pad=0):
    x = _h(x)
    N, H, W, Cc = x.shape
    P, Q, sh, sw, ph, pw = out_hw(H, W, R, S, stride, pad)
    col = np.empty((N * P * Q, R * S * Cc), np.float16)
    lib().bolt_ref_im2col(N, H, W, Cc, R, S, sh, sw, ph, pw, _ptr(x), _ptr(col))
    return col
