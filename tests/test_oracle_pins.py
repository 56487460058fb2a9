"""Pins of the CPU oracle against things other than itself (CPU only).

Each test is chosen so that a plausible mistake in oracle/bolt_oracle.c (dropped term, wrong sign
or index, transposed operand, filter flip, wrong rounding) fails at least one of them.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------------------------
# binary16 conversion
# --------------------------------------------------------------------------------------------
def test_half_to_double_all_values_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([ref.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_double_to_half_round_trip_exhaustive():
    for b in range(65536):
        v = np.uint16(b).view(np.float16).astype(np.float64)
        if math.isnan(v):
            continue
        assert ref.double_to_half(float(v)) == b, hex(b)


def test_double_to_half_midpoints_tie_to_even():
    # every pair of adjacent non-negative finite halves: the exact midpoint goes to the even one,
    # a hair either side goes to the nearer one
    for b in range(0, 0x7bff):
        lo = float(np.uint16(b).view(np.float16))
        hi = float(np.uint16(b + 1).view(np.float16))
        mid = (lo + hi) / 2.0  # exact in double
        even = b if b % 2 == 0 else b + 1
        assert ref.double_to_half(mid) == even, hex(b)
        assert ref.double_to_half(-mid) == (even | 0x8000), hex(b)
        assert ref.double_to_half(math.nextafter(mid, math.inf)) == b + 1
        assert ref.double_to_half(math.nextafter(mid, -math.inf)) == b


def test_double_to_half_range_edges():
    assert ref.double_to_half(65504.0) == 0x7bff
    assert ref.double_to_half(65519.999) == 0x7bff
    assert ref.double_to_half(65520.0) == 0x7c00          # tie rounds to "even" = infinity
    assert ref.double_to_half(1e30) == 0x7c00
    assert ref.double_to_half(-1e30) == 0xfc00
    assert ref.double_to_half(2.0 ** -24) == 1             # smallest subnormal
    assert ref.double_to_half(2.0 ** -25) == 0             # tie to even (zero)
    assert ref.double_to_half(math.nextafter(2.0 ** -25, 1.0)) == 1
    assert ref.double_to_half(2.0 ** -14) == 0x0400        # smallest normal
    assert ref.double_to_half(1e-300) == 0
    assert ref.double_to_half(-0.0) == 0x8000
    assert ref.double_to_half(float("inf")) == 0x7c00


def test_double_to_half_random_against_numpy():
    rng = np.random.default_rng(7)
    v = np.concatenate([rng.uniform(-70000, 70000, 20000), rng.normal(0, 1, 20000),
                        rng.normal(0, 1e-5, 20000), rng.normal(0, 1e-7, 5000)])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = np.array([ref.double_to_half(float(t)) for t in v], dtype=np.uint16)
    assert np.array_equal(got, want)


# --------------------------------------------------------------------------------------------
# GEMM
# --------------------------------------------------------------------------------------------
def _np_epilogue(s, bias, alpha, beta, act):
    v = alpha * s
    if bias is not None:
        v = v + beta * bias.astype(np.float64)
    if act == "relu":
        v = np.maximum(v, 0.0)
    return v


@pytest.mark.parametrize("M,N,K", [(5, 7, 3), (16, 8, 24), (33, 17, 40), (1, 1, 1)])
@pytest.mark.parametrize("act", ["none", "relu"])
def test_gemm_integer_inputs_exact_vs_numpy_float64(M, N, K, act):
    A = wl.integer_fp16(11, 0, (M, K), -3, 3)
    B = wl.integer_fp16(11, 1, (K, N), -3, 3)
    bias = wl.integer_fp16(11, 2, (N,), -3, 3)
    want = _np_epilogue(A.astype(np.float64) @ B.astype(np.float64), bias, 1.0, 1.0, act).astype(np.float16)
    got = ref.gemm(A, B, bias, act=act)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_gemm_uniform_inputs_vs_numpy_float64_with_alpha_beta():
    M, N, K = 37, 29, 53
    A = wl.uniform_fp16(12, 0, (M, K), -1, 1)
    B = wl.uniform_fp16(12, 1, (K, N), -1, 1)
    bias = wl.uniform_fp16(12, 2, (N,), -1, 1)
    for alpha, beta, act in [(1.0, 1.0, "relu"), (0.5, 2.0, "none"), (-1.25, 0.0, "relu")]:
        exact = _np_epilogue(A.astype(np.float64) @ B.astype(np.float64), bias, alpha, beta, act)
        got = ref.gemm(A, B, bias, alpha=alpha, beta=beta, act=act).astype(np.float64)
        # the oracle's double sum and numpy's differ by ~1e-15; after one FP16 rounding the two can
        # differ by at most one FP16 ulp, and only on values that sit on a rounding boundary
        ulp = np.spacing(np.abs(exact).astype(np.float16)).astype(np.float64)
        assert np.all(np.abs(got - exact) <= 0.5 * ulp * (1 + 1e-9) + 1e-300)


def test_gemm_no_bias_pointer_skips_beta_term():
    A = wl.integer_fp16(13, 0, (6, 8), -2, 2)
    B = wl.integer_fp16(13, 1, (8, 5), -2, 2)
    got = ref.gemm(A, B, None, beta=5.0, act="none").astype(np.float64)
    assert np.array_equal(got, A.astype(np.float64) @ B.astype(np.float64))


def test_gemm_brute_force_fractions():
    """Exact rational arithmetic in a different loop order on a tiny case."""
    M, N, K = 3, 4, 5
    A = wl.uniform_fp16(14, 0, (M, K), -1, 1)
    B = wl.uniform_fp16(14, 1, (K, N), -1, 1)
    bias = wl.uniform_fp16(14, 2, (N,), -1, 1)
    got = ref.gemm(A, B, bias, act="relu")
    for n in range(N):
        for m in range(M):
            s = Fraction(float(bias[n]))
            for k in reversed(range(K)):
                s += Fraction(float(A[m, k])) * Fraction(float(B[k, n]))
            s = max(s, Fraction(0))
            assert float(got[m, n]) == float(np.float16(float(s))), (m, n)


def test_gemm_at_matches_full():
    A = wl.uniform_fp16(15, 0, (19, 24), -1, 1)
    B = wl.uniform_fp16(15, 1, (24, 13), -1, 1)
    bias = wl.uniform_fp16(15, 2, (13,), -1, 1)
    full = ref.gemm(A, B, bias)
    idx = np.array([0, 5, 13, 100, 19 * 13 - 1])
    assert np.array_equal(ref.gemm_at(A, B, idx, bias), full.reshape(-1)[idx])


# --------------------------------------------------------------------------------------------
# convolution
# --------------------------------------------------------------------------------------------
def _torch_conv(x, w, bias, stride, pad, act, alpha=1.0, beta=1.0):
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)
    y = torch.nn.functional.conv2d(xt, wt, None, stride=stride, padding=pad) * alpha
    if bias is not None:
        y = y + beta * torch.from_numpy(bias.astype(np.float64)).view(1, -1, 1, 1)
    if act == "relu":
        y = torch.relu(y)
    return y.permute(0, 2, 3, 1).contiguous().numpy()


def test_conv_hand_computed_golden():
    x = np.arange(1, 10, dtype=np.float16).reshape(1, 3, 3, 1)
    w = np.array([1, 2, 3, 4], dtype=np.float16).reshape(1, 2, 2, 1)
    n_cases = 0
    for line in open(os.path.join(GOLDEN, "hand_conv_3x3_k2x2.txt")):
        if line.startswith("#") or "->" not in line:
            continue
        head, vals = line.split("->")
        _, stride, pad = head.split()
        want = np.array([float(v) for v in vals.split()])
        got = ref.conv2d_nhwc(x, w, None, stride=int(stride), pad=int(pad), act="none")
        assert np.array_equal(got.reshape(-1).astype(np.float64), want), head
        n_cases += 1
    assert n_cases == 3


CONV_CASES = [
    # N H W C K R S stride pad
    (2, 5, 5, 3, 4, 3, 3, 1, 1),
    (1, 7, 6, 2, 3, 3, 3, 2, 1),
    (2, 9, 9, 3, 2, 7, 7, 2, 3),
    (1, 6, 8, 4, 5, 1, 1, 1, 0),
    (1, 6, 8, 4, 5, 1, 1, 2, 0),
    (1, 8, 7, 2, 3, 5, 3, (1, 2), (2, 0)),   # non-square filter, asymmetric stride and padding
    (1, 4, 4, 1, 1, 4, 4, 1, 0),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_integer_inputs_exact_vs_torch_float64(case):
    N, H, W, Cc, K, R, S, stride, pad = case
    x = wl.integer_fp16(21, 0, (N, H, W, Cc), -2, 2)
    w = wl.integer_fp16(21, 1, (K, R, S, Cc), -2, 2)
    bias = wl.integer_fp16(21, 2, (K,), -2, 2)
    for act in ("none", "relu"):
        want = _torch_conv(x, w, bias, stride, pad, act).astype(np.float16)
        got = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad, act=act)
        assert got.shape == want.shape
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("case", CONV_CASES[:4])
def test_conv_uniform_inputs_vs_torch_float64(case):
    N, H, W, Cc, K, R, S, stride, pad = case
    x = wl.uniform_fp16(22, 0, (N, H, W, Cc), -1, 1)
    w = wl.uniform_fp16(22, 1, (K, R, S, Cc), -1, 1)
    bias = wl.uniform_fp16(22, 2, (K,), -1, 1)
    exact = _torch_conv(x, w, bias, stride, pad, "relu", alpha=0.75, beta=1.5)
    got = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad, alpha=0.75, beta=1.5, act="relu").astype(np.float64)
    ulp = np.spacing(np.abs(exact).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(got - exact) <= 0.5 * ulp * (1 + 1e-9) + 1e-300)


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (2, 3), (1, 0)])
def test_conv_unit_impulse_closed_form(stride, pad):
    """x = delta at (n0,h0,w0,c0)  =>  y[n0,p,q,k] = w[k, h0-p*s+pad, w0-q*s+pad, c0] where in range."""
    N, H, W, Cc, K, R, S = 2, 7, 8, 3, 4, 3, 5
    if pad == 3:
        R, S = 7, 7
    w = wl.uniform_fp16(23, 1, (K, R, S, Cc), -1, 1)
    n0, h0, w0, c0 = 1, 2, 5, 1
    x = np.zeros((N, H, W, Cc), np.float16)
    x[n0, h0, w0, c0] = 1.0
    y = ref.conv2d_nhwc(x, w, None, stride=stride, pad=pad, act="none")
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    assert y.shape == (N, P, Q, K)
    want = np.zeros_like(y)
    for p, q, k in itertools.product(range(P), range(Q), range(K)):
        r, s = h0 - p * stride + pad, w0 - q * stride + pad
        if 0 <= r < R and 0 <= s < S:
            want[n0, p, q, k] = w[k, r, s, c0]
    assert np.array_equal(y, want)


def test_conv_identity_1x1_returns_input():
    x = wl.uniform_fp16(24, 0, (2, 5, 6, 8), -1, 1)
    w = np.zeros((8, 1, 1, 8), np.float16)
    for k in range(8):
        w[k, 0, 0, k] = 1.0
    y = ref.conv2d_nhwc(x, w, None, act="none")
    assert np.array_equal(y.view(np.uint16), x.view(np.uint16))


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_equals_im2col_times_gemm_bitwise(case):
    N, H, W, Cc, K, R, S, stride, pad = case
    x = wl.uniform_fp16(25, 0, (N, H, W, Cc), -1, 1)
    w = wl.uniform_fp16(25, 1, (K, R, S, Cc), -1, 1)
    bias = wl.uniform_fp16(25, 2, (K,), -1, 1)
    y = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad, act="relu")
    col = ref.im2col(x, R, S, stride=stride, pad=pad)
    B = np.ascontiguousarray(w.reshape(K, -1).T)
    g = ref.gemm(col, B, bias, act="relu")
    assert np.array_equal(g.view(np.uint16).reshape(-1), y.view(np.uint16).reshape(-1))


def test_im2col_against_numpy_gather():
    N, H, W, Cc, R, S, stride, pad = 1, 5, 4, 2, 3, 3, 2, 1
    x = wl.uniform_fp16(26, 0, (N, H, W, Cc), -1, 1)
    col = ref.im2col(x, R, S, stride=stride, pad=pad)
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    rows = [xp[0, p * stride:p * stride + R, q * stride:q * stride + S, :].reshape(-1)
            for p in range(P) for q in range(Q)]
    assert np.array_equal(col, np.stack(rows))


def test_conv_1x1_equals_gemm_on_flattened_pixels():
    x = wl.uniform_fp16(27, 0, (2, 4, 5, 16), -1, 1)
    w = wl.uniform_fp16(27, 1, (24, 1, 1, 16), -1, 1)
    bias = wl.uniform_fp16(27, 2, (24,), -1, 1)
    y = ref.conv2d_nhwc(x, w, bias, act="relu")
    g = ref.gemm(x.reshape(-1, 16), np.ascontiguousarray(w.reshape(24, 16).T), bias, act="relu")
    assert np.array_equal(y.reshape(-1, 24), g)


def test_zero_padded_channels_change_nothing():
    x = wl.uniform_fp16(28, 0, (2, 6, 6, 3), -1, 1)
    w = wl.uniform_fp16(28, 1, (5, 3, 3, 3), -1, 1)
    bias = wl.uniform_fp16(28, 2, (5,), -1, 1)
    y = ref.conv2d_nhwc(x, w, bias, stride=2, pad=1)
    xp, wp = ref.pad_channels(x, 8), ref.pad_channels(w, 8)
    assert xp.shape == (2, 6, 6, 8) and np.array_equal(xp[..., :3], x) and not xp[..., 3:].any()
    yp = ref.conv2d_nhwc(xp, wp, bias, stride=2, pad=1)
    assert np.array_equal(y.view(np.uint16), yp.view(np.uint16))


def test_conv_bias_only_and_linearity():
    x = wl.integer_fp16(29, 0, (1, 5, 5, 4), -2, 2)
    x2 = wl.integer_fp16(29, 3, (1, 5, 5, 4), -2, 2)
    w = wl.integer_fp16(29, 1, (3, 3, 3, 4), -2, 2)
    bias = wl.uniform_fp16(29, 2, (3,), -1, 1)
    y0 = ref.conv2d_nhwc(x, np.zeros_like(w), bias, pad=1, act="relu")
    assert np.array_equal(y0, np.broadcast_to(np.maximum(bias, 0), y0.shape))
    ya = ref.conv2d_nhwc(x, w, None, pad=1, act="none").astype(np.float64)
    yb = ref.conv2d_nhwc(x2, w, None, pad=1, act="none").astype(np.float64)
    yab = ref.conv2d_nhwc((x + x2).astype(np.float16), w, None, pad=1, act="none").astype(np.float64)
    assert np.array_equal(ya + yb, yab)


def test_conv_brute_force_fractions_other_loop_order():
    N, H, W, Cc, K, R, S, stride, pad = 1, 4, 5, 3, 2, 3, 3, 2, 1
    x = wl.uniform_fp16(30, 0, (N, H, W, Cc), -1, 1)
    w = wl.uniform_fp16(30, 1, (K, R, S, Cc), -1, 1)
    bias = wl.uniform_fp16(30, 2, (K,), -1, 1)
    y = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad, act="relu")
    P, Q = y.shape[1:3]
    for k, q, p in itertools.product(range(K), range(Q), range(P)):
        s = Fraction(float(bias[k]))
        for c, sx, r in itertools.product(range(Cc), range(S), range(R)):
            ih, iw = p * stride - pad + r, q * stride - pad + sx
            if 0 <= ih < H and 0 <= iw < W:
                s += Fraction(float(x[0, ih, iw, c])) * Fraction(float(w[k, r, sx, c]))
        s = max(s, Fraction(0))
        assert float(y[0, p, q, k]) == float(np.float16(float(s)))


def test_conv_at_matches_full():
    x = wl.uniform_fp16(31, 0, (2, 6, 7, 4), -1, 1)
    w = wl.uniform_fp16(31, 1, (5, 3, 3, 4), -1, 1)
    bias = wl.uniform_fp16(31, 2, (5,), -1, 1)
    y = ref.conv2d_nhwc(x, w, bias, stride=2, pad=1)
    idx = np.array([0, 7, 33, y.size - 1, y.size // 2])
    assert np.array_equal(ref.conv2d_nhwc_at(x, w, idx, bias, stride=2, pad=1), y.reshape(-1)[idx])


# --------------------------------------------------------------------------------------------
# back-to-back chains
# --------------------------------------------------------------------------------------------
def test_b2b_gemm_is_two_gemms_with_fp16_intermediate():
    M, K0, N0, N1 = 21, 40, 16, 24
    A = wl.uniform_fp16(41, 0, (M, K0), -1, 1)
    W0 = wl.uniform_fp16(41, 1, (K0, N0), -1, 1)
    b0 = wl.uniform_fp16(41, 2, (N0,), -1, 1)
    W1 = wl.uniform_fp16(41, 3, (N0, N1), -1, 1)
    b1 = wl.uniform_fp16(41, 4, (N1,), -1, 1)
    got = ref.b2b_gemm(A, W0, b0, W1, b1).astype(np.float64)
    # independent float64 model of the chain with the intermediate rounded by numpy
    d0 = np.maximum(A.astype(np.float64) @ W0.astype(np.float64) + b0.astype(np.float64), 0).astype(np.float16)
    exact = np.maximum(d0.astype(np.float64) @ W1.astype(np.float64) + b1.astype(np.float64), 0)
    ulp = np.spacing(np.abs(exact).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(got - exact) <= 0.5 * ulp * (1 + 1e-9) + 1e-300)
    # and the rounding of D0 is really there: an unrounded chain differs somewhere
    unrounded = np.maximum(np.maximum(A.astype(np.float64) @ W0.astype(np.float64) + b0.astype(np.float64), 0)
                           @ W1.astype(np.float64) + b1.astype(np.float64), 0).astype(np.float16)
    assert not np.array_equal(unrounded, got.astype(np.float16))


def test_b2b_conv_is_two_convs_and_matches_b2b_gemm_on_im2col():
    N, H, W, Cc, K0, K1 = 2, 6, 6, 8, 16, 24
    x = wl.uniform_fp16(42, 0, (N, H, W, Cc), -1, 1)
    w0 = wl.normal_fp16(42, 1, (K0, 3, 3, Cc), 0.2)
    b0 = wl.uniform_fp16(42, 2, (K0,), -1, 1)
    w1 = wl.normal_fp16(42, 3, (K1, 1, 1, K0), 0.3)
    b1 = wl.uniform_fp16(42, 4, (K1,), -1, 1)
    y = ref.b2b_conv(x, w0, b0, w1, b1, stride=1, pad=1)
    y0 = ref.conv2d_nhwc(x, w0, b0, stride=1, pad=1)
    y1 = ref.conv2d_nhwc(y0, w1, b1)
    assert np.array_equal(y, y1)
    col = ref.im2col(x, 3, 3, stride=1, pad=1)
    g = ref.b2b_gemm(col, np.ascontiguousarray(w0.reshape(K0, -1).T), b0,
                     np.ascontiguousarray(w1.reshape(K1, K0).T), b1)
    assert np.array_equal(g, y.reshape(-1, K1))
    rows = np.array([0, 5, 17, N * H * W - 1])
    assert np.array_equal(ref.b2b_conv_rows(x, w0, b0, w1, b1, rows, stride=1, pad=1), y.reshape(-1, K1)[rows])


def test_b2b_conv_stride2_first_op():
    N, H, W, Cc, K0, K1 = 1, 9, 8, 4, 8, 8
    x = wl.integer_fp16(43, 0, (N, H, W, Cc), -2, 2)
    w0 = wl.integer_fp16(43, 1, (K0, 3, 3, Cc), -1, 1)
    b0 = wl.integer_fp16(43, 2, (K0,), -2, 2)
    w1 = wl.integer_fp16(43, 3, (K1, 1, 1, K0), -1, 1)
    b1 = wl.integer_fp16(43, 4, (K1,), -2, 2)
    y = ref.b2b_conv(x, w0, b0, w1, b1, stride=2, pad=1)
    t0 = _torch_conv(x, w0, b0, 2, 1, "relu").astype(np.float16)
    t1 = _torch_conv(t0, w1, b1, 1, 0, "relu").astype(np.float16)
    assert np.array_equal(y, t1)


def test_layout_transforms_against_numpy_transpose():
    x = wl.uniform_fp16(61, 0, (3, 5, 7, 6), -1, 1)  # N C H W, all extents different
    y = ref.nchw_to_nhwc(x, 8)
    assert y.shape == (3, 7, 6, 8)
    assert np.array_equal(y[..., :5], np.transpose(x, (0, 2, 3, 1))) and not y[..., 5:].any()
    assert np.array_equal(ref.nchw_to_nhwc(x), np.transpose(x, (0, 2, 3, 1)))
    assert np.array_equal(ref.nhwc_to_nchw(y, 5), x)                      # round trip drops the padding
    assert np.array_equal(ref.nhwc_to_nchw(y), np.transpose(y, (0, 3, 1, 2)))
    assert np.array_equal(ref.pad_channels(np.transpose(x, (0, 2, 3, 1)), 8), y)  # transform + pad == transpose, then pad


def test_residual_epilogue_full_matrix_c():
    # Eq. 1 with C a full matrix: against numpy float64 (exact on integers, half-ulp on fractions), the
    # gamma = 0 and C = 0 cases reduce to the plain ops, and conv == im2col GEMM with the same residual
    A = wl.integer_fp16(51, 0, (33, 24), -3, 3)
    B = wl.integer_fp16(51, 1, (24, 16), -3, 3)
    bias = wl.integer_fp16(51, 2, (16,), -4, 4)
    Cm = wl.integer_fp16(51, 3, (33, 16), -9, 9)
    f = lambda a: a.astype(np.float64)
    got = ref.gemm_residual(A, B, bias, Cm, 1.0, 1.0, -2.0, "relu")
    assert np.array_equal(f(got), np.maximum(f(A) @ f(B) + f(bias) - 2.0 * f(Cm), 0))
    assert np.array_equal(ref.gemm_residual(A, B, bias, Cm, gamma=0.0), ref.gemm(A, B, bias))
    assert np.array_equal(ref.gemm_residual(A, B, bias, np.zeros_like(Cm)), ref.gemm(A, B, bias))
    # a transposed or row-shifted C would break this: C varies along both axes
    Au, Bu, Cu = wl.uniform_fp16(52, 0, (20, 40), -1, 1), wl.uniform_fp16(52, 1, (40, 24), -1, 1), wl.uniform_fp16(52, 2, (20, 24), -4, 4)
    got = f(ref.gemm_residual(Au, Bu, None, Cu, 0.5, 1.0, 0.25, "none"))
    want = 0.5 * (f(Au) @ f(Bu)) + 0.25 * f(Cu)
    ulp = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(got - want) <= 0.5 * ulp * (1 + 1e-6) + 1e-300)
    x = wl.integer_fp16(53, 0, (2, 6, 5, 8), -2, 2)
    w = wl.integer_fp16(53, 1, (16, 3, 3, 8), -1, 1)
    b = wl.integer_fp16(53, 2, (16,), -2, 2)
    res = wl.integer_fp16(53, 3, (2, 3, 3, 16), -5, 5)
    y = ref.conv2d_nhwc_residual(x, w, b, res, stride=2, pad=1)
    col = ref.im2col(x, 3, 3, 2, 1)
    assert np.array_equal(y.reshape(-1, 16), ref.gemm_residual(col, w.reshape(16, -1).T, b, res.reshape(-1, 16)))
    assert not np.array_equal(y, ref.conv2d_nhwc(x, w, b, stride=2, pad=1))


def test_fused_pair_with_residual_in_the_second_epilogue():
    # Eq. 1-2 with C1 a full matrix, on integers small enough that D0 and every sum are exact: against numpy
    # float64 written out here; gamma = 0 reduces to the plain pair; the conv pair equals the GEMM pair on im2col
    A = wl.integer_fp16(54, 0, (21, 16), -2, 2)
    W0 = wl.integer_fp16(54, 1, (16, 8), -1, 1)
    b0 = wl.integer_fp16(54, 2, (8,), -2, 2)
    W1 = wl.integer_fp16(54, 3, (8, 24), -1, 1)
    b1 = wl.integer_fp16(54, 4, (24,), -2, 2)
    Cm = wl.integer_fp16(54, 5, (21, 24), -9, 9)
    f = lambda a: a.astype(np.float64)
    d0 = np.maximum(f(A) @ f(W0) + f(b0), 0)
    want = np.maximum(d0 @ f(W1) + f(b1) - 3.0 * f(Cm), 0)
    got = ref.b2b_gemm_residual(A, W0, b0, W1, b1, Cm, gamma=-3.0)
    assert np.array_equal(f(got), want) and np.abs(want).max() < 2048 and want.any()
    assert np.array_equal(ref.b2b_gemm_residual(A, W0, b0, W1, b1, Cm, gamma=0.0), ref.b2b_gemm(A, W0, b0, W1, b1))
    # the residual enters after op1 only: adding it to op0's output instead gives something else
    assert not np.array_equal(f(got), np.maximum(np.maximum(d0 - 3.0 * f(Cm)[:, :8], 0) @ f(W1) + f(b1), 0))
    x = wl.integer_fp16(55, 0, (2, 6, 5, 8), -2, 2)
    w0 = wl.integer_fp16(55, 1, (8, 3, 3, 8), -1, 1)
    w1 = wl.integer_fp16(55, 2, (16, 1, 1, 8), -1, 1)
    res = wl.integer_fp16(55, 3, (2, 3, 3, 16), -5, 5)
    y = ref.b2b_conv_residual(x, w0, b0, w1, b1[:16], res, stride=2, pad=1, gamma=2.0)
    col = ref.im2col(x, 3, 3, 2, 1)
    want = ref.b2b_gemm_residual(col, w0.reshape(8, -1).T, b0, w1.reshape(16, 8).T, b1[:16], res.reshape(-1, 16), gamma=2.0)
    assert np.array_equal(y.reshape(-1, 16), want)
    assert not np.array_equal(y, ref.b2b_conv(x, w0, b0, w1, b1[:16], stride=2, pad=1))


def test_chain_of_three_ops_rounds_between_ops_and_extends_b2b():
    # integers small enough that every intermediate is exactly representable: the chain must equal float64
    # matrix products with ReLUs, and the first two ops of it must be the b2b oracle bit for bit
    A = wl.integer_fp16(41, 0, (37, 24), -2, 2)
    Ws = [wl.integer_fp16(41, 1, (24, 16), -1, 1), wl.integer_fp16(41, 2, (16, 8), -1, 1), wl.integer_fp16(41, 3, (8, 24), -1, 1)]
    bs = [wl.integer_fp16(41, 4, (16,), -2, 2), None, wl.integer_fp16(41, 5, (24,), -2, 2)]
    got = ref.gemm_chain(A, Ws, bs, ["relu", "relu", "none"])
    f = lambda a: a.astype(np.float64)
    d0 = np.maximum(f(A) @ f(Ws[0]) + f(bs[0]), 0)
    d1 = np.maximum(d0 @ f(Ws[1]), 0)
    want = d1 @ f(Ws[2]) + f(bs[2])
    assert np.abs(want).max() < 2048 and np.array_equal(f(got), want)
    two = ref.b2b_gemm(A, Ws[0], bs[0], Ws[1], bs[1])
    assert np.array_equal(ref.gemm_chain(A, Ws[:2], bs[:2], ["relu", "relu"]), two)
    # with fractions the FP16 rounding between ops is visible: an unrounded chain differs somewhere
    A = wl.uniform_fp16(42, 0, (64, 32), -1, 1)
    Ws = [wl.uniform_fp16(42, 1 + i, s, -1, 1) for i, s in enumerate([(32, 32), (32, 32), (32, 16)])]
    got = ref.gemm_chain(A, Ws, [None] * 3, ["relu"] * 3)
    stepwise = f(A)
    for W in Ws:
        stepwise = f(np.maximum(stepwise @ f(W), 0).astype(np.float16))
    unrounded = f(A)
    for W in Ws:
        unrounded = np.maximum(unrounded @ f(W), 0)
    assert np.array_equal(f(got), stepwise) and not np.array_equal(f(got), unrounded.astype(np.float16).astype(np.float64))
    # convolution chain == GEMM chain on the im2col of the first op
    x = wl.integer_fp16(43, 0, (2, 6, 5, 8), -2, 2)
    ws = [wl.integer_fp16(43, 1, (16, 3, 3, 8), -1, 1), wl.integer_fp16(43, 2, (8, 1, 1, 16), -1, 1), wl.integer_fp16(43, 3, (24, 1, 1, 8), -1, 1)]
    cb = [wl.integer_fp16(43, 4, (16,), -2, 2), wl.integer_fp16(43, 5, (8,), -2, 2), None]
    y = ref.conv_chain(x, ws, cb, ["relu", "relu", "relu"], stride=2, pad=1)
    col = ref.im2col(x, 3, 3, 2, 1)
    gw = [w.reshape(w.shape[0], -1).T for w in ws]
    assert np.array_equal(y.reshape(-1, 24), ref.gemm_chain(col, gw, cb, ["relu"] * 3))


def test_chain_with_a_residual_adds_gamma_c_before_the_last_activation_only():
    # small integers: every intermediate and the result are exact in FP16, so the chain must equal the float64
    # expression relu(relu(relu(A W0 + b0) W1) W2 + b2 + gamma C) - the residual inside the LAST activation, scaled
    # by gamma, and nowhere else
    A = wl.integer_fp16(51, 0, (29, 16), -2, 2)
    Ws = [wl.integer_fp16(51, 1, (16, 8), -1, 1), wl.integer_fp16(51, 2, (8, 8), -1, 1), wl.integer_fp16(51, 3, (8, 24), -1, 1)]
    bs = [wl.integer_fp16(51, 4, (8,), -2, 2), None, wl.integer_fp16(51, 5, (24,), -2, 2)]
    C = wl.integer_fp16(51, 6, (29, 24), -40, 40)
    f = lambda a: a.astype(np.float64)
    d0 = np.maximum(f(A) @ f(Ws[0]) + f(bs[0]), 0)
    d1 = np.maximum(d0 @ f(Ws[1]), 0)
    pre = d1 @ f(Ws[2]) + f(bs[2])
    got = ref.gemm_chain_residual(A, Ws, bs, ["relu", "relu", "relu"], C, gamma=-3.0)
    want = np.maximum(pre - 3.0 * f(C), 0)
    assert np.abs(pre).max() + 120 < 2048 and np.array_equal(f(got), want)
    # the residual matters, sits inside the activation (adding it after the ReLU differs), and gamma = 0 removes it
    plain = ref.gemm_chain(A, Ws, bs, ["relu", "relu", "relu"])
    assert not np.array_equal(got, plain)
    assert not np.array_equal(f(got), np.maximum(pre, 0) - 3.0 * f(C))
    assert np.array_equal(ref.gemm_chain_residual(A, Ws, bs, ["relu", "relu", "relu"], C, gamma=0.0), plain)
    # a chain of two with a residual is the fused pair with a residual
    assert np.array_equal(ref.gemm_chain_residual(A, Ws[:2], bs[:2], ["relu", "relu"], C[:, :8], gamma=2.0),
                          ref.b2b_gemm_residual(A, Ws[0], bs[0], Ws[1], bs[1], C[:, :8], gamma=2.0))
    # convolution chain with a residual == GEMM chain with a residual on the im2col of the first op
    x = wl.integer_fp16(52, 0, (2, 6, 5, 8), -2, 2)
    ws = [wl.integer_fp16(52, 1, (16, 3, 3, 8), -1, 1), wl.integer_fp16(52, 2, (8, 1, 1, 16), -1, 1), wl.integer_fp16(52, 3, (24, 1, 1, 8), -1, 1)]
    cb = [wl.integer_fp16(52, 4, (16,), -2, 2), wl.integer_fp16(52, 5, (8,), -2, 2), None]
    res = wl.integer_fp16(52, 6, (2, 3, 3, 24), -30, 30)
    y = ref.conv_chain_residual(x, ws, cb, ["relu", "relu", "relu"], res, stride=2, pad=1, gamma=1.0)
    col = ref.im2col(x, 3, 3, 2, 1)
    gw = [w.reshape(w.shape[0], -1).T for w in ws]
    assert y.shape == (2, 3, 3, 24)
    assert np.array_equal(y.reshape(-1, 24), ref.gemm_chain_residual(col, gw, cb, ["relu"] * 3, res.reshape(-1, 24), gamma=1.0))
    assert not np.array_equal(y, ref.conv_chain(x, ws, cb, ["relu"] * 3, stride=2, pad=1))


# --------------------------------------------------------------------------------------------
# epilogue activations (closed forms)
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("act", ["gelu", "hardswish", "softplus"])
def test_activation_closed_forms(act):
    # GEMM with K=1, B=[1]: D = act(A + bias)
    v = np.linspace(-8, 8, 129).astype(np.float16)
    A = v.reshape(-1, 1)
    B = np.ones((1, 1), np.float16)
    got = ref.gemm(A, B, None, act=act).reshape(-1).astype(np.float64)
    t = v.astype(np.float64)
    if act == "gelu":
        want = np.array([0.5 * a * (1 + math.erf(a / math.sqrt(2))) for a in t])
    elif act == "hardswish":
        want = t * np.clip(t + 3, 0, 6) / 6
    else:
        want = np.log1p(np.exp(t))
    ulp = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(got - want) <= 0.5 * ulp * (1 + 1e-6) + 1e-300)


def _oracle_act(act, v16):
    """act(v) for a vector of halves through the oracle: a K = 1 GEMM against B = [1]."""
    return ref.gemm(v16.reshape(-1, 1), np.ones((1, 1), np.float16), None, act=act).reshape(-1).astype(np.float64)


def _half_ulp_ok(got, want):
    ulp = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
    return np.all(np.abs(got - want) <= 0.5 * ulp * (1 + 1e-6) + 1e-300)


@pytest.mark.parametrize("act", ["gelu", "hardswish", "softplus"])
def test_activation_values_from_an_independent_implementation(act):
    # Values that do not come from the formula the oracle evaluates: PyTorch's own float64 activation kernels
    # (Section 3.2.3 lists these three next to ReLU) over every finite half in [-10, 10] (a wrong constant,
    # a tanh approximation in place of the exact GELU, a shifted Hardswish knee all fail here).
    import torch
    import torch.nn.functional as F
    allh = np.arange(0x10000, dtype=np.uint32).astype(np.uint16).view(np.float16)
    v = allh[np.isfinite(allh) & (np.abs(allh.astype(np.float64)) <= 10)]
    t = torch.from_numpy(v.astype(np.float64))
    want = {"gelu": lambda: F.gelu(t, approximate="none"), "hardswish": lambda: F.hardswish(t),
            "softplus": lambda: F.softplus(t, beta=1.0, threshold=1e9)}[act]().numpy()
    assert _half_ulp_ok(_oracle_act(act, v), want)


def test_gelu_is_v_times_the_gaussian_cdf_by_quadrature_and_table_values():
    # GELU(v) = v * Phi(v) with Phi the integral of the standard normal density: the integral is evaluated by
    # adaptive quadrature (no erf anywhere), plus the table values Phi(1) = 0.8413447461, Phi(2) = 0.9772498681.
    from scipy import integrate
    pts = np.array([-6, -3.5, -2, -1, -0.5, -0.125, 0, 0.125, 0.5, 1, 2, 3.5, 6], dtype=np.float16)
    dens = lambda u: math.exp(-0.5 * u * u) / math.sqrt(2 * math.pi)
    phi = np.array([integrate.quad(dens, -np.inf, float(a), epsabs=1e-14, epsrel=1e-13)[0] for a in pts])
    assert _half_ulp_ok(_oracle_act("gelu", pts), pts.astype(np.float64) * phi)
    table = {1.0: 0.8413447461, 2.0: 1.9544997361, -1.0: -0.1586552539, 0.0: 0.0}
    got = _oracle_act("gelu", np.array(list(table), dtype=np.float16))
    assert _half_ulp_ok(got, np.array(list(table.values())))


def test_hardswish_knees_and_table_values():
    # v * relu6(v + 3) / 6: zero up to -3, the identity from +3, exact rationals in between
    v = np.array([-8, -3, -1.5, -1, 0, 1, 1.5, 3, 8], dtype=np.float16)
    want = np.array([0, 0, -0.375, -1.0 / 3, 0, 2.0 / 3, 1.125, 3, 8])
    assert _half_ulp_ok(_oracle_act("hardswish", v), want)


@pytest.mark.parametrize("act", ["none", "relu", "gelu", "hardswish", "softplus"])
def test_bias_act_closed_forms_with_alpha_beta(act):
    # the stand-alone epilogue pass (Section 4.1.1's un-fused baseline): every finite-range half in a
    # column strip, per-column bias, alpha/beta exactly representable so the affine part is exact in fp64
    M, N = 96, 16
    x = wl.uniform_fp16(31, 0, (M, N), -6, 6)
    b = wl.uniform_fp16(31, 1, (N,), -2, 2)
    alpha, beta = 0.75, -1.5
    got = ref.bias_act(x, b, alpha, beta, act).astype(np.float64)
    t = alpha * x.astype(np.float64) + beta * b.astype(np.float64)[None, :]
    want = {"none": t, "relu": np.maximum(t, 0), "gelu": 0.5 * t * (1 + np.vectorize(math.erf)(t / math.sqrt(2))),
            "hardswish": t * np.clip(t + 3, 0, 6) / 6, "softplus": np.logaddexp(0, t)}[act]
    ulp = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(got - want) <= 0.5 * ulp * (1 + 1e-6) + 1e-300)
    # no bias pointer: the beta term vanishes; a transposed bias index would break the per-column check above
    nb = ref.bias_act(x, None, alpha, 123.0, "none").astype(np.float64)
    assert np.array_equal(nb, (alpha * x.astype(np.float64)).astype(np.float16).astype(np.float64))


def test_unfused_epilogue_equals_fused_on_integer_inputs():
    # with small integers nothing rounds, so GEMM(act none, no bias) followed by the stand-alone pass must
    # reproduce the fused GEMM bit for bit
    A = wl.integer_fp16(32, 0, (40, 24), -3, 3)
    B = wl.integer_fp16(32, 1, (24, 16), -3, 3)
    bias = wl.integer_fp16(32, 2, (16,), -4, 4)
    fused = ref.gemm(A, B, bias, 1.0, 1.0, "relu")
    plain = ref.gemm(A, B, None, 1.0, 1.0, "none")
    assert np.array_equal(ref.bias_act(plain, bias, 1.0, 1.0, "relu"), fused)
    assert np.array_equal(fused.astype(np.float64),
                          np.maximum(A.astype(np.float64) @ B.astype(np.float64) + bias.astype(np.float64), 0))


# --------------------------------------------------------------------------------------------
# workload tables
# --------------------------------------------------------------------------------------------
def test_resnet50_table_totals():
    layers = wl.resnet50_layers(32)
    flops = sum(s.flops * c for s, c in layers)
    byts = sum(s.bytes * c for s, c in layers)
    assert abs(flops / 1e9 - 261.6) < 0.5
    assert abs(byts / 1e6 - 1389) < 15
    s2 = wl.CONFIG2_SHAPE
    assert s2.gemm_m == 100352 and s2.gemm_k == 576 and s2.flops == 2 * 100352 * 64 * 576


def test_generators_are_deterministic_and_in_range():
    a = wl.uniform_fp16(5, 0, (1000,), -1, 1)
    b = wl.uniform_fp16(5, 0, (1000,), -1, 1)
    c = wl.uniform_fp16(5, 1, (1000,), -1, 1)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert a.min() >= -1 and a.max() <= 1 and abs(float(a.astype(np.float64).mean())) < 0.1
    n = wl.normal_fp16(5, 2, (20000,), 0.5).astype(np.float64)
    assert abs(n.std() - 0.5) < 0.02 and abs(n.mean()) < 0.02
    i = wl.integer_fp16(5, 3, (1000,), -2, 2)
    assert set(np.unique(i)) == {-2.0, -1.0, 0.0, 1.0, 2.0}
