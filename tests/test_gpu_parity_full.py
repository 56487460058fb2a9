"""GPU parity, second part: whole-tensor compares at the full configuration sizes, bit-exact integer cases for the
fused and re-use kernels, the activations over every finite half, and sampled parity at the sizes bench.py times.

Same rules as test_gpu_parity.py: the HIP library through its C ABI against the CPU oracle on the same seeded
inputs; |gpu - oracle| <= 1e-2 * (1 + |oracle|) for floating point, identical bits for integer-valued cases.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import ref
from util import assert_bit_equal, assert_close, dev, host

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def bolt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2110_15238_amd as b
    return b


def _say(msg):
    print(msg, flush=True)


def _nan16(*shape):
    return torch.full(shape, float("nan"), dtype=torch.float16, device="cuda")


def _sample(total, count, seed):
    rng = np.random.default_rng(seed)
    return np.unique(np.concatenate([rng.integers(0, total, size=count), np.array([0, total - 1])]))


def _pad8(v):
    return (v + 7) // 8 * 8


def _padc(a, c8):
    """Zero-pad the last axis to c8 (Section 3.2.3, kernel padding) on the host; the oracle sees the unpadded tensor."""
    out = np.zeros(a.shape[:-1] + (c8,), a.dtype)
    out[..., :a.shape[-1]] = a
    return out


# ---------------------------------------------------------------------------------------------
# activations: every finite half through the fused epilogue, within one FP16 ulp of the oracle
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("act", ["relu", "gelu", "hardswish", "softplus"])
def test_activation_of_every_finite_half_within_one_ulp(bolt, act):
    # D = act(A . B) with K = 8 and B = e0 e0^T: column 0 of D is act(v) for the v in column 0 of A, the other
    # columns are act(0).  The device evaluates GELU / Softplus with its own FP32 forms on the hardware exp2 / log2 /
    # rcp units: their error has to stay far below half an ulp for the rounded result to be at most one ulp off.
    allh = np.arange(0x10000, dtype=np.uint32).astype(np.uint16).view(np.float16)
    v = allh[np.isfinite(allh)]
    assert v.size == 63488
    A = np.zeros((v.size, 8), np.float16)
    A[:, 0] = v
    B = np.zeros((8, 8), np.float16)
    B[0, 0] = 1
    want = ref.gemm(A, B, None, act=act).astype(np.float64)
    d = bolt.gemm_desc(v.size, 8, 8, act=act)
    D = _nan16(v.size, 8)
    bolt.bolt_gemm_epilogue(d, dev(A), dev(B), None, D)
    torch.cuda.synchronize()
    got = host(D).astype(np.float64)
    assert np.all(np.isfinite(got) | ~np.isfinite(want))
    with np.errstate(over="ignore"):  # the spacing above the largest finite half is infinite; such entries are not compared
        ulp = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
    fin = np.isfinite(want) & np.isfinite(ulp)
    worst = np.max(np.abs(got[fin] - want[fin]) / ulp[fin])
    _say("%s: worst deviation %.2f ulp over %d halves" % (act, worst, v.size))
    assert worst <= 1.0
    assert np.array_equal(got[~fin], want[~fin])  # overflow to infinity where the oracle overflows


# ---------------------------------------------------------------------------------------------
# configs 2 and 4 at batch 32: every output element
# ---------------------------------------------------------------------------------------------
def test_config2_full_size_every_element(bolt):
    t, s = wl.config2(), wl.CONFIG2_SHAPE
    d = bolt.conv_desc(s.N, s.H, s.W, s.C, s.K, s.R, s.S, s.stride, s.pad)
    x, w, b = dev(t["x"]), dev(t["w"]), dev(t["bias"])
    y = _nan16(s.N, s.P, s.Q, s.K)
    ws = torch.empty(max(bolt.bolt_workspace_bytes(bolt.OP_CONV2D, d), 16) // 4, dtype=torch.float32, device="cuda")
    cfg = bolt.bolt_tune(bolt.OP_CONV2D, d, None, [x, w, b, y], ws).config
    y.fill_(float("nan"))
    bolt.bolt_conv2d_fprop_nhwc(d, x, w, b, y, cfg, ws)
    torch.cuda.synchronize()
    _say("config 2 tuned %s; oracle over all %d outputs" % (cfg.as_dict(), y.numel()))
    assert_close(host(y), ref.conv2d_nhwc(t["x"], t["w"], t["bias"], stride=1, pad=1), "config 2, batch 32, every element")


def test_config4_full_size_every_element(bolt):
    t = wl.config4()
    c0 = bolt.conv_desc(32, 56, 56, 64, 64, 3, 3, 1, 1)
    c1 = bolt.conv_desc(32, 56, 56, 64, 256, 1, 1, 1, 0)
    x, w0, b0, w1, b1 = (dev(t[k]) for k in ("x", "w0", "b0", "w1", "b1"))
    y = _nan16(32, 56, 56, 256)
    cfg = bolt.bolt_tune(bolt.OP_B2B_CONV, c0, c1, [x, w0, b0, w1, b1, y]).config
    y.fill_(float("nan"))
    bolt.bolt_b2b_conv(c0, c1, x, w0, b0, w1, b1, y, cfg)
    torch.cuda.synchronize()
    _say("config 4 tuned %s; oracle over all %d outputs" % (cfg.as_dict(), y.numel()))
    want = ref.b2b_conv(t["x"], t["w0"], t["b0"], t["w1"], t["b1"], stride=1, pad=1)
    assert_close(host(y), want, "config 4, batch 32, every element")


# ---------------------------------------------------------------------------------------------
# integer inputs: identical bits from the fused, halo re-use and k-group kernels
# ---------------------------------------------------------------------------------------------
def _sparse(w):
    """Keep one weight in four (those with row % 4 == col % 4 over the first and last axis): the intermediates of a
    chain stay small enough to be exact in FP16."""
    k, c = w.shape[0], w.shape[-1]
    keep = (np.arange(k)[:, None] % 4) == (np.arange(c)[None, :] % 4)
    w = w.copy()
    w[np.broadcast_to(~keep.reshape((k,) + (1,) * (w.ndim - 2) + (c,)), w.shape)] = 0
    return w


B2B_CONV_INT = [  # N H W C K0 stride K1: stride-1 "same" shapes (halo family), stride 2, thin and ragged widths
    (2, 12, 12, 64, 64, 1, 256), (2, 12, 12, 64, 64, 2, 64), (1, 15, 17, 48, 48, 1, 48), (2, 20, 20, 8, 48, 2, 48),
    (3, 9, 11, 128, 64, 1, 128), (1, 11, 11, 24, 128, 1, 128), (1, 10, 12, 64, 64, 1, 200), (2, 9, 10, 64, 40, 1, 136),
]


@pytest.mark.parametrize("shape", B2B_CONV_INT)
def test_b2b_conv_integer_bit_exact_every_instance(bolt, shape):
    N, H, W, Cc, K0, stride, K1 = shape
    x = wl.integer_fp16(601, 0, (N, H, W, Cc), -1, 1)
    w0 = wl.integer_fp16(601, 1, (K0, 3, 3, Cc), -1, 1)
    b0 = wl.integer_fp16(601, 2, (K0,), -3, 3)
    w1 = _sparse(wl.integer_fp16(601, 3, (K1, 1, 1, K0), -1, 1))
    b1 = wl.integer_fp16(601, 4, (K1,), -3, 3)
    # |D0| <= 9 C + 3 <= 1155: exact in FP16; |D1| <= K0 / 4 * 1155 + 3 < 2^24: exact in FP32, so both sides round the
    # same integer to FP16
    want = ref.b2b_conv(x, w0, b0, w1, b1, stride=stride, pad=1)
    assert np.all(np.isfinite(want))
    c0 = bolt.conv_desc(N, H, W, Cc, K0, 3, 3, stride, 1)
    P, Q = bolt.conv_out_hw(c0)
    c1 = bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0)
    xd, w0d, b0d, w1d, b1d = dev(x), dev(w0), dev(b0), dev(w1), dev(b1)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_CONV)):
        if not bolt.bolt_instance_supports(bolt.OP_B2B_CONV, kid, c0, c1):
            continue
        _say("integer b2b conv %s instance %d" % (shape, kid))
        y = _nan16(N, P, Q, K1)
        bolt.bolt_b2b_conv(c0, c1, xd, w0d, b0d, w1d, b1d, y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_bit_equal(host(y), want, "integer b2b conv %s instance %d" % (shape, kid))
        ran += 1
    assert ran >= 1


@pytest.mark.parametrize("shape", [(2, 12, 12, 64, 64, 3, 3, 1, 1, 64, 64), (1, 17, 13, 24, 48, 3, 3, 2, 1, 48, 48),
                                   (2, 23, 23, 8, 64, 7, 7, 2, 3, 64, 256), (3, 9, 11, 64, 64, 1, 1, 1, 0, 256, 64),
                                   (2, 9, 10, 128, 64, 3, 3, 1, 1, 64, 256), (1, 11, 9, 192, 128, 5, 3, 1, (2, 1), 120, 128),
                                   (3, 30, 30, 64, 64, 3, 3, 1, 1, 64, 128), (2, 10, 10, 64, 64, 3, 3, 1, 1, 128, 128),
                                   (1, 9, 12, 128, 128, 3, 3, 1, 1, 64, 64)])
def test_conv_chain3_integer_bit_exact_every_instance(bolt, shape):
    N, H, W, Cc, K0, R, S, stride, pad, K1, K2 = shape
    x = wl.integer_fp16(602, 0, (N, H, W, Cc), -1, 1)
    ws = [_sparse(wl.integer_fp16(602, 1, (K0, R, S, Cc), -1, 1)), _sparse(wl.integer_fp16(602, 2, (K1, 1, 1, K0), -1, 1)),
          _sparse(wl.integer_fp16(602, 3, (K2, 1, 1, K1), -1, 1))]
    bs = [wl.integer_fp16(602, 4, (K0,), -2, 2), wl.integer_fp16(602, 5, (K1,), -2, 2), wl.integer_fp16(602, 6, (K2,), -2, 2)]
    acts = ["relu", "relu", "none"]
    want = ref.conv_chain(x, ws, bs, acts, stride=stride, pad=pad)
    # every partial sum is an integer below 2^24, exact in FP32 and in double, so both sides round the same exact
    # values to FP16 between the ops and at the end
    assert np.all(np.isfinite(want))
    d0 = bolt.conv_desc(N, H, W, Cc, K0, R, S, stride, pad, act=acts[0])
    P, Q = bolt.conv_out_hw(d0)
    descs = [d0, bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0, act=acts[1]), bolt.conv_desc(N, P, Q, K1, K2, 1, 1, 1, 0, act=acts[2])]
    wd, bd, xd = [dev(w) for w in ws], [dev(b) for b in bs], dev(x)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_CONV_CHAIN3)):
        if not bolt.bolt_chain_instance_supports(bolt.OP_CONV_CHAIN3, kid, descs):
            continue
        _say("integer conv chain %s instance %d" % (shape, kid))
        y = _nan16(N, P, Q, K2)
        bolt.bolt_b2b_conv_chain(descs, xd, wd, bd, y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_bit_equal(host(y), want, "integer conv chain %s instance %d" % (shape, kid))
        ran += 1
    assert ran >= 1


@pytest.mark.parametrize("case", [(2, 12, 12, 64, 72, 3, 3, 1, 1), (2, 9, 10, 256, 72, 3, 3, 1, 1), (1, 9, 11, 128, 40, 3, 3, 1, 1),
                                  (2, 7, 9, 192, 136, 5, 3, 1, (2, 1)), (1, 17, 13, 128, 136, 3, 3, 2, 1), (2, 7, 7, 512, 64, 1, 1, 1, 0)])
def test_conv_integer_bit_exact_halo_and_k_group_instances(bolt, case):
    # shapes every kernel family accepts: stride-1 "same" filters with C % 64 == 0 (halo re-use, 1 to 4 channel
    # chunks), deep reductions (k-groups of 2 and 4 share one tile and sum through LDS in a fixed order)
    N, H, W, Cc, K, R, S, stride, pad = case
    x = wl.integer_fp16(603, 0, (N, H, W, Cc), -2, 2)
    w = wl.integer_fp16(603, 1, (K, R, S, Cc), -1, 1)
    bias = wl.integer_fp16(603, 2, (K,), -3, 3)
    want = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad)
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_CONV2D)):
        if not bolt.bolt_instance_supports(bolt.OP_CONV2D, kid, d):
            continue
        _say("integer conv %s instance %d" % (case, kid))
        y = _nan16(*want.shape)
        bolt.bolt_conv2d_fprop_nhwc(d, dev(x), dev(w), dev(bias), y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_bit_equal(host(y), want, "integer conv %s instance %d" % (case, kid))
        ran += 1
    assert ran >= 5


# ---------------------------------------------------------------------------------------------
# the sizes bench.py times, tuned as bench.py tunes them, sampled against the oracle
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("row", list(range(len(wl.TABLE1_B2B_GEMM))))
def test_table1_b2b_gemm_full_size_sampled_rows(bolt, row):
    # Table 1 (Section 4.1.2) at its own M; extents that are not multiples of 8 are zero-padded first (Section
    # 3.2.3), the oracle works on the unpadded problem
    M, N0, K0, N1 = wl.TABLE1_B2B_GEMM[row]
    A = wl.uniform_fp16(611 + row, 0, (M, K0), -0.5, 0.5)
    W0 = wl.uniform_fp16(611 + row, 1, (K0, N0), -0.5, 0.5)
    b0 = wl.uniform_fp16(611 + row, 2, (N0,), -0.5, 0.5)
    W1 = wl.uniform_fp16(611 + row, 3, (N0, N1), -0.5, 0.5)
    b1 = wl.uniform_fp16(611 + row, 4, (N1,), -0.5, 0.5)
    n0, k0, n1 = _pad8(N0), _pad8(K0), _pad8(N1)
    Ap, W0p, b0p = _padc(A, k0), _padc(_padc(W0.T, k0).T, n0), _padc(b0, n0)   # W0: [k0][n0]
    W1p, b1p = _padc(_padc(W1.T, n0).T, n1), _padc(b1, n1)                      # W1: [n0][n1]
    g0, g1 = bolt.gemm_desc(M, n0, k0), bolt.gemm_desc(M, n1, n0)
    W0d, W1d = dev(W0p), dev(W1p)
    if bolt.bolt_check(bolt.OP_B2B_GEMM, g0, g1) != 0:
        # row-major weights of this size do not fit the weights-resident kernels: reduction-contiguous instead
        g0 = bolt.gemm_desc(M, n0, k0, b_layout=bolt.LAYOUT_NK)
        g1 = bolt.gemm_desc(M, n1, n0, b_layout=bolt.LAYOUT_NK)
        W0d, W1d = dev(np.ascontiguousarray(W0p.T)), dev(np.ascontiguousarray(W1p.T))
    Ad, b0d, b1d = dev(Ap), dev(b0p), dev(b1p)
    D = _nan16(M, n1)
    cfg = bolt.bolt_tune(bolt.OP_B2B_GEMM, g0, g1, [Ad, W0d, b0d, W1d, b1d, D]).config
    D.fill_(float("nan"))
    bolt.bolt_b2b_gemm(g0, g1, Ad, W0d, b0d, W1d, b1d, D, cfg)
    torch.cuda.synchronize()
    got = host(D)
    assert np.all(np.isfinite(got))
    rows = _sample(M, 400, 3)
    want = ref.b2b_gemm(A[rows], W0, b0, W1, b1)
    _say("Table 1 row %d tuned %s, %d rows sampled" % (row, cfg.as_dict(), rows.size))
    assert_close(got[rows][:, :N1], want, "Table 1 row %d" % row)
    assert np.all(got[rows][:, N1:] == np.maximum(b1p[N1:].astype(np.float32), 0).astype(np.float16))  # padded columns: relu(0 + 0)


@pytest.mark.parametrize("row", [0, 1, 3, 4])
def test_table2_b2b_conv_full_size_sampled_rows(bolt, row):
    # Table 2 (Section 4.1.2), the 224 x 224 and 112 x 112 rows at batch 32: 3x3 (stride 2) -> 1x1, each with bias + ReLU
    H, IC, OC0, stride, OC1 = wl.TABLE2_B2B_CONV[row]
    x = wl.uniform_fp16(621 + row, 0, (32, H, H, IC), -1, 1)
    w0 = wl.normal_fp16(621 + row, 1, (OC0, 3, 3, IC), (2.0 / (9 * IC)) ** 0.5)
    b0 = wl.uniform_fp16(621 + row, 2, (OC0,), -1, 1)
    w1 = wl.normal_fp16(621 + row, 3, (OC1, 1, 1, OC0), (2.0 / OC0) ** 0.5)
    b1 = wl.uniform_fp16(621 + row, 4, (OC1,), -1, 1)
    ic = _pad8(IC)
    c0 = bolt.conv_desc(32, H, H, ic, OC0, 3, 3, stride, 1)
    P, Q = bolt.conv_out_hw(c0)
    c1 = bolt.conv_desc(32, P, Q, OC0, OC1, 1, 1, 1, 0)
    xd, w0d, b0d, w1d, b1d = dev(_padc(x, ic)), dev(_padc(w0, ic)), dev(b0), dev(w1), dev(b1)
    y = _nan16(32, P, Q, OC1)
    cfg = bolt.bolt_tune(bolt.OP_B2B_CONV, c0, c1, [xd, w0d, b0d, w1d, b1d, y]).config
    y.fill_(float("nan"))
    bolt.bolt_b2b_conv(c0, c1, xd, w0d, b0d, w1d, b1d, y, cfg)
    torch.cuda.synchronize()
    got = host(y).reshape(-1, OC1)
    assert np.all(np.isfinite(got))
    rows = _sample(got.shape[0], 300, 4)
    want = ref.b2b_conv_rows(x, w0, b0, w1, b1, rows, stride=stride, pad=1)
    _say("Table 2 row %d tuned %s, %d rows sampled" % (row, cfg.as_dict(), rows.size))
    assert_close(got[rows], want, "Table 2 row %d" % row)


@pytest.mark.parametrize("row", list(range(len(wl.TABLE3_PADDING))))
def test_table3_padding_full_size_sampled_both_sides(bolt, row):
    # Table 3 (Section 3.2.3): the alignment-2 kernel on the unpadded tensor and the alignment-8 kernel on the padded
    # one, each tuned at the table's own batch, against the oracle on the unpadded problem
    N, H, W, IC, OC, R, S, pad = wl.TABLE3_PADDING[row]
    x = wl.uniform_fp16(631 + row, 0, (N, H, W, IC), -1, 1)
    w = wl.normal_fp16(631 + row, 1, (OC, R, S, IC), (2.0 / (R * S * IC)) ** 0.5)
    b = wl.uniform_fp16(631 + row, 2, (OC,), -1, 1)
    ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
    want = None
    for c in (IC, _pad8(IC)):
        d = bolt.conv_desc(N, H, W, c, OC, R, S, 1, pad)
        P, Q = bolt.conv_out_hw(d)
        xd, wd, bd = dev(_padc(x, c)), dev(_padc(w, c)), dev(b)
        y = _nan16(N, P, Q, OC)
        cfg = bolt.bolt_tune(bolt.OP_CONV2D, d, None, [xd, wd, bd, y], ws).config
        y.fill_(float("nan"))
        bolt.bolt_conv2d_fprop_nhwc(d, xd, wd, bd, y, cfg, ws)
        torch.cuda.synchronize()
        got = host(y).reshape(-1)
        assert np.all(np.isfinite(got))
        idx = _sample(got.size, 4000, 5)
        if want is None:
            want = ref.conv2d_nhwc_at(x, w, idx, b, stride=1, pad=pad)
        _say("Table 3 row %d C=%d tuned %s" % (row, c, cfg.as_dict()))
        assert_close(got[idx], want, "Table 3 row %d with %d channels" % (row, c))


def test_conv_chain3_full_size_sampled_rows(bolt):
    # the 56 x 56, 64-channel chain 3x3 -> 1x1 -> 1x1 of bench.py at batch 32.  Oracle per sampled pixel: the pinned
    # two-op rows, then the third 1x1 as a GEMM over those rows (a 1x1 convolution is a GEMM per pixel).
    N, H, C = 32, 56, 64
    x = wl.uniform_fp16(641, 0, (N, H, H, C), -1, 1)
    ws = [wl.normal_fp16(641, 1, (C, 3, 3, C), (2.0 / (9 * C)) ** 0.5), wl.normal_fp16(641, 2, (C, 1, 1, C), (2.0 / C) ** 0.5),
          wl.normal_fp16(641, 3, (C, 1, 1, C), (2.0 / C) ** 0.5)]
    bs = [wl.uniform_fp16(641, 4 + i, (C,), -1, 1) for i in range(3)]
    descs = [bolt.conv_desc(N, H, H, C, C, 3, 3, 1, 1), bolt.conv_desc(N, H, H, C, C, 1, 1, 1, 0), bolt.conv_desc(N, H, H, C, C, 1, 1, 1, 0)]
    xd, wd, bd = dev(x), [dev(w) for w in ws], [dev(b) for b in bs]
    y = _nan16(N, H, H, C)
    cfg = bolt.bolt_tune_chain(bolt.OP_CONV_CHAIN3, descs, [xd, wd[0], bd[0], wd[1], bd[1], wd[2], bd[2], y]).config
    y.fill_(float("nan"))
    bolt.bolt_b2b_conv_chain(descs, xd, wd, bd, y, cfg)
    torch.cuda.synchronize()
    got = host(y).reshape(-1, C)
    assert np.all(np.isfinite(got))
    rows = _sample(got.shape[0], 300, 6)
    d1 = ref.b2b_conv_rows(x, ws[0], bs[0], ws[1], bs[1], rows, stride=1, pad=1)
    want = ref.gemm(d1, np.ascontiguousarray(ws[2].reshape(C, C).T), bs[2])
    _say("conv chain tuned %s, %d rows sampled" % (cfg.as_dict(), rows.size))
    assert_close(got[rows], want, "conv chain of three at batch 32")


# ---------------------------------------------------------------------------------------------
# host-side robustness
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("layout", ["kn", "nk"])
def test_b2b_padded_columns_stay_finite_with_a_huge_bias_term(bolt, layout):
    # N0 = 40 runs on kernels compiled for 64 columns: the 24 padded columns of D0 are multiplied by zero weights
    # in the second op.  beta0 * bias0 alone overflows FP16 in columns 0-3 (the product term brings the true value
    # back into range), so a padded column that borrowed that bias would be inf, and inf * 0 would poison every
    # output of its row.
    M, K0, N0, N1 = 100, 64, 40, 64
    A = np.full((M, K0), 30, np.float16)
    W0 = wl.uniform_fp16(651, 0, (K0, N0), -0.01, 0.01)
    W0[:, :4] = -36
    b0 = wl.uniform_fp16(651, 1, (N0,), -0.001, 0.001)
    b0[:4] = 70
    W1 = wl.uniform_fp16(651, 2, (N0, N1), -0.05, 0.05)
    b1 = wl.uniform_fp16(651, 3, (N1,), -1, 1)
    want = ref.b2b_gemm(A, W0, b0, W1, b1, beta0=1000.0, act0="none", act1="none")
    assert np.all(np.isfinite(want))
    lay = bolt.LAYOUT_KN if layout == "kn" else bolt.LAYOUT_NK
    W0d = dev(W0 if layout == "kn" else np.ascontiguousarray(W0.T))
    W1d = dev(W1 if layout == "kn" else np.ascontiguousarray(W1.T))
    g0 = bolt.gemm_desc(M, N0, K0, beta=1000.0, act="none", b_layout=lay)
    g1 = bolt.gemm_desc(M, N1, N0, act="none", b_layout=lay)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_GEMM)):
        if not bolt.bolt_instance_supports(bolt.OP_B2B_GEMM, kid, g0, g1):
            continue
        _say("padded-column b2b gemm %s instance %d" % (layout, kid))
        D = _nan16(M, N1)
        bolt.bolt_b2b_gemm(g0, g1, dev(A), W0d, dev(b0), W1d, dev(b1), D, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(D), want, "padded-column b2b gemm %s instance %d" % (layout, kid))
        ran += 1
    assert ran >= 1


def test_tune_with_a_workspace_does_not_leak_split_k_into_a_call_without_one(bolt):
    # a deep, narrow problem: with a workspace the search may pick split-K; the same problem tuned afterwards
    # without a workspace must come back with a config that runs without one
    M, N, K = 64, 64, 8192
    A, B, bias = wl.uniform_fp16(661, 0, (M, K), -1, 1), wl.uniform_fp16(661, 1, (K, N), -1, 1), wl.uniform_fp16(661, 2, (N,), -1, 1)
    d = bolt.gemm_desc(M, N, K)
    Ad, Bd, bd = dev(A), dev(B), dev(bias)
    D = _nan16(M, N)
    ws = torch.empty(8 * M * N, dtype=torch.float32, device="cuda")
    with_ws = bolt.bolt_tune(bolt.OP_GEMM, d, None, [Ad, Bd, bd, D], ws)
    without = bolt.bolt_tune(bolt.OP_GEMM, d, None, [Ad, Bd, bd, D])
    _say("with workspace: %s; without: %s" % (with_ws.config.as_dict(), without.config.as_dict()))
    assert without.config.split_k <= 1
    D.fill_(float("nan"))
    bolt.bolt_gemm_epilogue(d, Ad, Bd, bd, D, without.config)
    torch.cuda.synchronize()
    assert_close(host(D), ref.gemm(A, B, bias), "config tuned without a workspace")
    D.fill_(float("nan"))
    bolt.bolt_gemm_epilogue(d, Ad, Bd, bd, D, with_ws.config, ws)
    torch.cuda.synchronize()
    assert_close(host(D), ref.gemm(A, B, bias), "config tuned with a workspace")


def test_first_launch_of_a_kernel_inside_a_graph_capture():
    # A fresh process, so that no kernel has been launched before: the very first call of each entry point happens
    # while the stream is being captured (the opt-in to large dynamic LDS is part of that first call).  The replays
    # must reproduce what the same calls give eagerly afterwards.
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = r"""
import sys, numpy as np, torch
sys.path.insert(0, %r)
import paper_2110_15238_amd as bolt
import workloads as wl
M, N, K = 300, 264, 200
A = torch.from_numpy(wl.uniform_fp16(671, 0, (M, K), -1, 1)).cuda()
B = torch.from_numpy(wl.uniform_fp16(671, 1, (N, K), -1, 1)).cuda()
bias = torch.from_numpy(wl.uniform_fp16(671, 2, (N,), -1, 1)).cuda()
x = torch.from_numpy(wl.uniform_fp16(671, 3, (2, 12, 12, 64), -1, 1)).cuda()
w = torch.from_numpy(wl.uniform_fp16(671, 4, (72, 3, 3, 64), -0.1, 0.1)).cuda()
cb = torch.from_numpy(wl.uniform_fp16(671, 5, (72,), -1, 1)).cuda()
gd = bolt.gemm_desc(M, N, K, b_layout=bolt.LAYOUT_NK)
cd = bolt.conv_desc(2, 12, 12, 64, 72, 3, 3, 1, 1)
kids = [k for k in range(bolt.bolt_num_instances(bolt.OP_GEMM)) if bolt.bolt_instance_supports(bolt.OP_GEMM, k, gd)]
cids = [k for k in range(bolt.bolt_num_instances(bolt.OP_CONV2D)) if bolt.bolt_instance_supports(bolt.OP_CONV2D, k, cd)]
outs = [torch.zeros((M, N), dtype=torch.float16, device="cuda") for _ in kids] + [torch.zeros((2, 12, 12, 72), dtype=torch.float16, device="cuda") for _ in cids]
def calls(dst):
    for i, k in enumerate(kids):
        bolt.bolt_gemm_epilogue(gd, A, B, bias, dst[i], {"kernel_id": k})
    for i, k in enumerate(cids):
        bolt.bolt_conv2d_fprop_nhwc(cd, x, w, cb, dst[len(kids) + i], {"kernel_id": k})
torch.cuda.synchronize()
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g):
    calls(outs)
for rep in range(3):
    for o in outs:
        o.fill_(float("nan"))
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    snap = [o.clone() for o in outs]
    eager = [torch.zeros_like(o) for o in outs]
    calls(eager)
    torch.cuda.synchronize()
    for a, b in zip(snap, eager):
        assert torch.equal(a, b), "replay %%d differs from the eager result" %% rep
print("captured-first-launch ok: %%d gemm and %%d conv instances" %% (len(kids), len(cids)))
""" % root
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=240)
    _say(r.stdout[-400:] + r.stderr[-800:])
    assert r.returncode == 0 and "captured-first-launch ok" in r.stdout
