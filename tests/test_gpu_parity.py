"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Bound for floating point: |gpu - oracle| <= 1e-2 * (1 + |oracle|).  Integer-valued cases (every
partial sum exactly representable) must agree bit for bit.
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


# ---------------------------------------------------------------------------------------------
# GEMM
# ---------------------------------------------------------------------------------------------
def _run_gemm(bolt, A, B, bias, act="relu", alpha=1.0, beta=1.0, layout="kn", config=None, workspace=None):
    M, K = A.shape
    N = B.shape[1]
    if layout == "kn":
        Bd, lay = dev(B), bolt.LAYOUT_KN
    else:
        Bd, lay = dev(np.ascontiguousarray(B.T)), bolt.LAYOUT_NK
    d = bolt.gemm_desc(M, N, K, alpha=alpha, beta=beta, act=act, b_layout=lay)
    D = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_gemm_epilogue(d, dev(A), Bd, dev(bias), D, config, workspace)
    torch.cuda.synchronize()
    return host(D), d


def test_config1_gemm_bias_relu(bolt):
    t = wl.config1()
    want = ref.gemm(t["A"], t["B"], t["bias"])
    got, _ = _run_gemm(bolt, t["A"], t["B"], t["bias"])
    assert_close(got, want, "config1 heuristic")
    got, _ = _run_gemm(bolt, t["A"], t["B"], t["bias"], layout="nk")
    assert_close(got, want, "config1 NK layout")


@pytest.mark.parametrize("layout", ["kn", "nk"])
def test_gemm_every_instance_ragged_shapes(bolt, layout):
    # M, N, K chosen to give 1, 2 and 3 K-loop trips at BK = 64 / 32, ragged tiles in M and N
    shapes = [(200, 136, 64), (333, 72, 128), (97, 264, 200), (1, 8, 8), (520, 320, 72)]
    nk_off = bolt.bolt_num_instances(bolt.OP_GEMM) // 2
    for (M, N, K) in shapes:
        A = wl.uniform_fp16(101, 0, (M, K), -1, 1)
        B = wl.uniform_fp16(101, 1, (K, N), -1, 1)
        bias = wl.uniform_fp16(101, 2, (N,), -1, 1)
        want = ref.gemm(A, B, bias)
        d = bolt.gemm_desc(M, N, K, b_layout=bolt.LAYOUT_KN if layout == "kn" else bolt.LAYOUT_NK)
        ran = 0
        for kid in range(bolt.bolt_num_instances(bolt.OP_GEMM)):
            if not bolt.bolt_instance_supports(bolt.OP_GEMM, kid, d):
                continue
            _say("gemm %s shape %s instance %d" % (layout, (M, N, K), kid))
            got, _ = _run_gemm(bolt, A, B, bias, layout=layout, config={"kernel_id": kid})
            assert_close(got, want, "gemm %s %s instance %d" % (layout, (M, N, K), kid))
            ran += 1
        assert ran >= 3
    assert nk_off > 0


@pytest.mark.parametrize("layout", ["kn", "nk"])
def test_gemm_integer_inputs_bit_exact(bolt, layout):
    M, N, K = 300, 136, 128
    A = wl.integer_fp16(102, 0, (M, K), -2, 2)
    B = wl.integer_fp16(102, 1, (K, N), -2, 2)
    bias = wl.integer_fp16(102, 2, (N,), -2, 2)
    want = ref.gemm(A, B, bias, act="none")
    d = bolt.gemm_desc(M, N, K, b_layout=bolt.LAYOUT_KN if layout == "kn" else bolt.LAYOUT_NK)
    for kid in range(bolt.bolt_num_instances(bolt.OP_GEMM)):
        if bolt.bolt_instance_supports(bolt.OP_GEMM, kid, d):
            _say("gemm int %s instance %d" % (layout, kid))
            got, _ = _run_gemm(bolt, A, B, bias, act="none", layout=layout, config={"kernel_id": kid})
            assert_bit_equal(got, want, "gemm integer instance %d" % kid)


def test_gemm_alpha_beta_activations_and_no_bias(bolt):
    M, N, K = 130, 72, 96
    A = wl.uniform_fp16(103, 0, (M, K), -1, 1)
    B = wl.uniform_fp16(103, 1, (K, N), -1, 1)
    bias = wl.uniform_fp16(103, 2, (N,), -1, 1)
    for act in ["none", "relu", "gelu", "hardswish", "softplus"]:
        want = ref.gemm(A, B, bias, alpha=0.5, beta=2.0, act=act)
        got, _ = _run_gemm(bolt, A, B, bias, act=act, alpha=0.5, beta=2.0)
        assert_close(got, want, "gemm act " + act)
    want = ref.gemm(A, B, None, act="relu")
    got, _ = _run_gemm(bolt, A, B, None, act="relu")
    assert_close(got, want, "gemm without bias")


def test_gemm_split_k_and_swizzle(bolt):
    M, N, K = 384, 256, 1024
    A = wl.uniform_fp16(104, 0, (M, K), -1, 1)
    B = wl.uniform_fp16(104, 1, (K, N), -1, 1)
    bias = wl.uniform_fp16(104, 2, (N,), -1, 1)
    want = ref.gemm(A, B, bias)
    ws = torch.empty(8 * M * N, dtype=torch.float32, device="cuda")
    d = bolt.gemm_desc(M, N, K)
    kids = [k for k in range(bolt.bolt_num_instances(bolt.OP_GEMM)) if bolt.bolt_instance_supports(bolt.OP_GEMM, k, d)]
    for kid in kids[:6]:
        for split_k in (2, 3, 8):
            _say("gemm split_k=%d instance %d" % (split_k, kid))
            got, _ = _run_gemm(bolt, A, B, bias, config={"kernel_id": kid, "split_k": split_k}, workspace=ws)
            assert_close(got, want, "split_k=%d instance %d" % (split_k, kid))
        for swz in (1, 4, 7):
            got, _ = _run_gemm(bolt, A, B, bias, config={"kernel_id": kid, "swizzle": swz})
            assert_close(got, want, "swizzle=%d instance %d" % (swz, kid))
    # a missing workspace is an error, not a silent fallback
    with pytest.raises(bolt.BoltError) as e:
        _run_gemm(bolt, A, B, bias, config={"kernel_id": kids[0], "split_k": 4})
    assert e.value.status == 4


@pytest.mark.parametrize("layout", ["kn", "nk"])
def test_gemm_leading_dimensions_every_instance(bolt, layout):
    """Row strides beyond the extents on all three matrices (the bytes between are poison for B: NaN), N and K ragged
    against every tile, through the built-in pick and every instance of the layout."""
    M, N, K, lda, ldd = 300, 104, 136, 152, 120
    ldb = 112 if layout == "kn" else 144
    A = wl.uniform_fp16(105, 0, (M, lda), -1, 1)
    Bm = wl.uniform_fp16(105, 1, (K, N), -1, 1)
    bias = wl.uniform_fp16(105, 2, (N,), -1, 1)
    want = ref.gemm(np.ascontiguousarray(A[:, :K]), Bm, bias)
    Bs = np.full((K, ldb) if layout == "kn" else (N, ldb), np.nan, dtype=np.float16)
    if layout == "kn":
        Bs[:, :N] = Bm
    else:
        Bs[:, :K] = Bm.T
    d = bolt.gemm_desc(M, N, K, lda=lda, ldb=ldb, ldd=ldd, b_layout=bolt.LAYOUT_KN if layout == "kn" else bolt.LAYOUT_NK)
    Ad, Bd, bd = dev(A), dev(Bs), dev(bias)
    ids = [k for k in range(bolt.bolt_num_instances(bolt.OP_GEMM)) if bolt.bolt_instance_supports(bolt.OP_GEMM, k, d)]
    assert len(ids) >= 8
    for cfg in [None] + [{"kernel_id": k} for k in ids]:
        _say("gemm leading dimensions, weights %s, config %s" % (layout, cfg))
        D = torch.zeros((M, ldd), dtype=torch.float16, device="cuda")
        bolt.bolt_gemm_epilogue(d, Ad, Bd, bd, D, cfg)
        torch.cuda.synchronize()
        got = host(D)
        assert_close(got[:, :N], want, "gemm with leading dimensions, weights %s, config %s" % (layout, cfg))
        assert not got[:, N:].any(), "columns beyond N were written (config %s)" % (cfg,)


# ---------------------------------------------------------------------------------------------
# convolution
# ---------------------------------------------------------------------------------------------
def _run_conv(bolt, x, w, bias, stride, pad, act="relu", config=None, workspace=None, alpha=1.0, beta=1.0):
    N, H, W, Cc = x.shape
    K, R, S, _ = w.shape
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad, alpha=alpha, beta=beta, act=act)
    P, Q = bolt.conv_out_hw(d)
    y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_conv2d_fprop_nhwc(d, dev(x), dev(w), dev(bias), y, config, workspace)
    torch.cuda.synchronize()
    return host(y), d


CONV_SWEEP = [
    # N H W C K R S stride pad
    (2, 12, 12, 8, 16, 3, 3, 1, 1),
    (1, 17, 13, 24, 40, 3, 3, 2, 1),
    (2, 23, 23, 8, 64, 7, 7, 2, 3),
    (3, 9, 11, 64, 72, 1, 1, 1, 0),
    (2, 14, 14, 64, 128, 1, 1, 2, 0),
    (1, 10, 9, 16, 24, 5, 3, (1, 2), (2, 0)),
    (1, 6, 6, 136, 8, 3, 3, 1, 1),
    (1, 5, 5, 8, 8, 5, 5, 1, 0),
    # stride 1, "same" padding, C % 64 == 0: also legal for the halo re-use kernels
    (2, 12, 12, 64, 72, 3, 3, 1, 1),
    (1, 9, 11, 128, 40, 3, 3, 1, 1),
    (5, 5, 4, 64, 64, 3, 3, 1, 1),
    (2, 7, 9, 192, 136, 5, 3, 1, (2, 1)),
    (1, 30, 30, 64, 264, 3, 3, 1, 1),
    (2, 9, 10, 256, 72, 3, 3, 1, 1),   # four 64-channel chunks: the halo kernels' k-groups of 2 and 4
]


@pytest.mark.parametrize("case", CONV_SWEEP)
def test_conv_every_instance_shape_sweep(bolt, case):
    N, H, W, Cc, K, R, S, stride, pad = case
    x = wl.uniform_fp16(201, 0, (N, H, W, Cc), -1, 1)
    w = wl.uniform_fp16(201, 1, (K, R, S, Cc), -1, 1)
    bias = wl.uniform_fp16(201, 2, (K,), -1, 1)
    want = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad)
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_CONV2D)):
        if not bolt.bolt_instance_supports(bolt.OP_CONV2D, kid, d):
            continue
        _say("conv case %s instance %d" % (case, kid))
        got, _ = _run_conv(bolt, x, w, bias, stride, pad, config={"kernel_id": kid})
        assert_close(got, want, "conv %s instance %d" % (case, kid))
        ran += 1
    assert ran >= 3


def _pingpong_ids(bolt, op):
    """Instances built on the 16 x 16 x 32 matrix-core instruction (the two-wave-group 256 x 256 kernel)."""
    return [k for k in range(bolt.bolt_num_instances(op)) if bolt.bolt_instance_config(op, k).mfma_shape == 16]


PINGPONG_CONV = [
    # N H W C K R S stride pad: several 256-row tiles with a ragged last one, K_out ragged against 256, k-tiles that
    # walk taps and 64-channel chunks, strides, non-square filters, windows hanging over every image edge
    (3, 20, 20, 128, 264, 3, 3, 1, 1),
    (2, 23, 19, 64, 136, 3, 3, 2, 1),
    (1, 11, 12, 64, 264, 2, 4, 1, (1, 2)),
    (5, 9, 14, 192, 512, 3, 1, (2, 1), (1, 0)),
    (1, 40, 40, 64, 256, 1, 1, 2, 0),
]


@pytest.mark.parametrize("case", PINGPONG_CONV)
def test_conv_pingpong_instance_integer_bit_exact(bolt, case):
    N, H, W, Cc, K, R, S, stride, pad = case
    x = wl.integer_fp16(231, 0, (N, H, W, Cc), -2, 2)
    w = wl.integer_fp16(231, 1, (K, R, S, Cc), -1, 1)
    bias = wl.integer_fp16(231, 2, (K,), -3, 3)
    want = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad)
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad)
    ids = [k for k in _pingpong_ids(bolt, bolt.OP_CONV2D) if bolt.bolt_instance_supports(bolt.OP_CONV2D, k, d)]
    assert ids, "no ping-pong convolution instance accepts %s" % (case,)
    for kid in ids:
        for swz in (0, 4):
            _say("ping-pong conv %s instance %d swizzle %d" % (case, kid, swz))
            got, _ = _run_conv(bolt, x, w, bias, stride, pad, config={"kernel_id": kid, "swizzle": swz})
            assert_bit_equal(got, want, "ping-pong conv %s instance %d" % (case, kid))
    # uniform data, every activation, alpha / beta: the elementwise bound
    x = wl.uniform_fp16(232, 0, (N, H, W, Cc), -1, 1)
    w = wl.uniform_fp16(232, 1, (K, R, S, Cc), -0.1, 0.1)
    bias = wl.uniform_fp16(232, 2, (K,), -1, 1)
    for act in ("none", "gelu"):
        want = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad, alpha=0.5, beta=2.0, act=act)
        got, _ = _run_conv(bolt, x, w, bias, stride, pad, act=act, alpha=0.5, beta=2.0, config={"kernel_id": ids[0]})
        assert_close(got, want, "ping-pong conv %s act %s" % (case, act))


@pytest.mark.parametrize("layout", ["nk", "kn"])
def test_gemm_pingpong_instance_integer_bit_exact_k_tails_and_split_k_refusal(bolt, layout):
    ids = _pingpong_ids(bolt, bolt.OP_GEMM)
    assert ids
    for (M, N, K) in ((700, 264, 200), (257, 520, 64), (1, 136, 8), (513, 256, 1096)):
        A = wl.integer_fp16(233, 0, (M, K), -2, 2)
        B = wl.integer_fp16(233, 1, (K, N), -1, 1)
        bias = wl.integer_fp16(233, 2, (N,), -3, 3)
        want = ref.gemm(A, B, bias)
        d = bolt.gemm_desc(M, N, K, b_layout=bolt.LAYOUT_NK if layout == "nk" else bolt.LAYOUT_KN)
        mine = [k for k in ids if bolt.bolt_instance_supports(bolt.OP_GEMM, k, d)]
        assert mine, "no ping-pong instance for weights stored %s" % layout
        for kid in mine:
            _say("ping-pong gemm %s weights %s instance %d" % ((M, N, K), layout, kid))
            got, _ = _run_gemm(bolt, A, B, bias, layout=layout, config={"kernel_id": kid, "swizzle": 4})
            assert_bit_equal(got, want, "ping-pong gemm %s weights %s instance %d" % ((M, N, K), layout, kid))
            # the kernel has no partial-sum output: asking for split-K is an error, not a silent full-K run
            ws = torch.empty(8 * M * N, dtype=torch.float32, device="cuda")
            with pytest.raises(bolt.BoltError) as e:
                _run_gemm(bolt, A, B, bias, layout=layout, config={"kernel_id": kid, "split_k": 2}, workspace=ws)
            assert e.value.status == 2


# Even channel counts that are not multiples of 8 run on the alignment-2 instances (the unpadded side of
# Table 3): that table's geometries at a small batch, plus C = 2, a strided 1x1 and non-square strides.
ALIGN2_SWEEP = [(2,) + row[1:7] + (1, row[7]) for row in wl.TABLE3_PADDING] + [
    (3, 9, 11, 2, 16, 3, 3, 1, 1),
    (2, 14, 14, 46, 40, 1, 1, 2, 0),
    (1, 10, 9, 10, 24, 5, 3, (1, 2), (2, 0)),
    (1, 6, 6, 30, 72, 3, 3, 1, 1),
    (1, 7, 7, 6, 8, 7, 7, 1, 3),
]


@pytest.mark.parametrize("case", ALIGN2_SWEEP)
def test_conv_alignment2_every_instance(bolt, case):
    N, H, W, Cc, K, R, S, stride, pad = case
    x = wl.uniform_fp16(211, 0, (N, H, W, Cc), -1, 1)
    w = wl.uniform_fp16(211, 1, (K, R, S, Cc), -1, 1)
    bias = wl.uniform_fp16(211, 2, (K,), -1, 1)
    want = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad)
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_CONV2D)):
        if not bolt.bolt_instance_supports(bolt.OP_CONV2D, kid, d):
            continue
        _say("align-2 conv case %s instance %d" % (case, kid))
        got, _ = _run_conv(bolt, x, w, bias, stride, pad, config={"kernel_id": kid})
        assert_close(got, want, "align-2 conv %s instance %d" % (case, kid))
        ran += 1
    assert ran >= 3
    got, _ = _run_conv(bolt, x, w, bias, stride, pad)  # built-in pick rule
    assert_close(got, want, "align-2 conv %s heuristic" % (case,))


def test_conv_alignment2_integer_bit_exact_split_k_and_padding_equivalence(bolt):
    N, H, W, Cc, K, R, S, stride, pad = 2, 10, 13, 46, 32, 5, 5, 1, 2
    x = wl.integer_fp16(212, 0, (N, H, W, Cc), -2, 2)
    w = wl.integer_fp16(212, 1, (K, R, S, Cc), -2, 2)
    bias = wl.integer_fp16(212, 2, (K,), -3, 3)
    want = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad)
    got, d = _run_conv(bolt, x, w, bias, stride, pad)
    assert_bit_equal(got, want, "align-2 integer conv")
    ws = torch.empty(bolt.bolt_workspace_bytes(bolt.OP_CONV2D, d), dtype=torch.uint8, device="cuda")
    kid = next(i for i in range(bolt.bolt_num_instances(bolt.OP_CONV2D)) if bolt.bolt_instance_supports(bolt.OP_CONV2D, i, d))
    got, _ = _run_conv(bolt, x, w, bias, stride, pad, config={"kernel_id": kid, "split_k": 4}, workspace=ws)
    assert_bit_equal(got, want, "align-2 integer conv, split-K 4")
    # Table 3's two sides compute the same thing: unpadded on alignment 2 == padded to 48 on alignment 8
    xp = torch.empty((N, H, W, 48), dtype=torch.float16, device="cuda")
    wp = torch.empty((K, R, S, 48), dtype=torch.float16, device="cuda")
    bolt.bolt_pad_channels_nhwc(dev(x), xp, 48)
    bolt.bolt_pad_channels_nhwc(dev(w), wp, 48)
    got_p, _ = _run_conv(bolt, host(xp), host(wp), bias, stride, pad)
    assert_bit_equal(got_p, want, "padded integer conv")


def test_conv_integer_inputs_bit_exact(bolt):
    N, H, W, Cc, K, R, S, stride, pad = 2, 13, 11, 8, 24, 3, 3, 1, 1
    x = wl.integer_fp16(202, 0, (N, H, W, Cc), -2, 2)
    w = wl.integer_fp16(202, 1, (K, R, S, Cc), -2, 2)
    bias = wl.integer_fp16(202, 2, (K,), -2, 2)
    for act in ("none", "relu"):
        want = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad, act=act)
        d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad)
        for kid in range(bolt.bolt_num_instances(bolt.OP_CONV2D)):
            if bolt.bolt_instance_supports(bolt.OP_CONV2D, kid, d):
                got, _ = _run_conv(bolt, x, w, bias, stride, pad, act=act, config={"kernel_id": kid})
                assert_bit_equal(got, want, "conv integer instance %d act %s" % (kid, act))


def test_conv_identity_1x1_returns_input_exactly(bolt):
    x = wl.uniform_fp16(203, 0, (2, 9, 7, 64), -1, 1)
    w = np.zeros((64, 1, 1, 64), np.float16)
    for k in range(64):
        w[k, 0, 0, k] = 1.0
    got, _ = _run_conv(bolt, x, w, None, 1, 0, act="none")
    assert_bit_equal(got, x, "identity 1x1")


def test_conv_split_k(bolt):
    N, H, W, Cc, K, R, S, stride, pad = 1, 7, 7, 128, 64, 3, 3, 1, 1
    x = wl.uniform_fp16(204, 0, (N, H, W, Cc), -1, 1)
    w = wl.normal_fp16(204, 1, (K, R, S, Cc), 0.05)
    bias = wl.uniform_fp16(204, 2, (K,), -1, 1)
    want = ref.conv2d_nhwc(x, w, bias, stride=stride, pad=pad)
    ws = torch.empty(8 * 49 * K, dtype=torch.float32, device="cuda")
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_CONV2D)):
        if bolt.bolt_instance_supports(bolt.OP_CONV2D, kid, d):
            for sk in (2, 5, 8):
                if bolt.bolt_check(bolt.OP_CONV2D, d, None, {"kernel_id": kid, "split_k": sk}) == 2:  # BOLT_ERR_UNSUPPORTED
                    continue  # instance has no split-K variant (reported before any launch)
                ran += 1
                _say("conv split_k=%d instance %d" % (sk, kid))
                got, _ = _run_conv(bolt, x, w, bias, stride, pad, config={"kernel_id": kid, "split_k": sk}, workspace=ws)
                assert_close(got, want, "conv split_k=%d instance %d" % (sk, kid))
    assert ran >= 9


def test_config2_conv_small_batch_full_compare(bolt):
    t = wl.config2(batch=2)
    want = ref.conv2d_nhwc(t["x"], t["w"], t["bias"], stride=1, pad=1)
    got, _ = _run_conv(bolt, t["x"], t["w"], t["bias"], 1, 1)
    assert_close(got, want, "config2 at batch 2")


def _sample_idx(total, count, seed):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, total, size=count)
    edge = np.array([0, total - 1])
    return np.unique(np.concatenate([idx, edge]))


def test_config2_conv_full_size_tuned_sampled(bolt):
    t = wl.config2()
    s = wl.CONFIG2_SHAPE
    d = bolt.conv_desc(s.N, s.H, s.W, s.C, s.K, s.R, s.S, s.stride, s.pad)
    x, w, b = dev(t["x"]), dev(t["w"]), dev(t["bias"])
    y = torch.full((s.N, s.P, s.Q, s.K), float("nan"), dtype=torch.float16, device="cuda")
    ws_bytes = bolt.bolt_workspace_bytes(bolt.OP_CONV2D, d)
    ws = torch.empty(max(ws_bytes, 16) // 4, dtype=torch.float32, device="cuda")
    res = bolt.bolt_tune(bolt.OP_CONV2D, d, None, [x, w, b, y], ws)
    _say("config2 tuned: %s %.4f ms, %d tried" % (res.config.as_dict(), res.ms, res.tried))
    assert res.tried >= 3 and res.ms > 0
    y.fill_(float("nan"))
    bolt.bolt_conv2d_fprop_nhwc(d, x, w, b, y, res.config, ws)
    torch.cuda.synchronize()
    got = host(y).reshape(-1)
    assert np.all(np.isfinite(got))
    idx = _sample_idx(got.size, 20000, 1)
    want = ref.conv2d_nhwc_at(t["x"], t["w"], idx, t["bias"], stride=1, pad=1)
    assert_close(got[idx], want, "config2 full size, tuned, sampled")


# ---------------------------------------------------------------------------------------------
# channel padding
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("C,C8", [(3, 8), (46, 48), (8, 8), (174, 176), (1, 16)])
def test_pad_channels_bit_exact(bolt, C, C8):
    x = wl.uniform_fp16(301, 0, (3, 5, 7, C), -1, 1)
    want = ref.pad_channels(x, C8)
    dst = torch.full((3, 5, 7, C8), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_pad_channels_nhwc(dev(x), dst, C8)
    torch.cuda.synchronize()
    assert_bit_equal(host(dst), want, "pad %d -> %d" % (C, C8))


def test_padded_stem_conv_matches_unpadded_oracle(bolt):
    # C = 3 padded to 8 on the GPU; the oracle runs the original 3-channel problem
    N, H, W, K = 2, 30, 30, 64
    x = wl.uniform_fp16(302, 0, (N, H, W, 3), -1, 1)
    w = wl.normal_fp16(302, 1, (K, 7, 7, 3), 0.1)
    bias = wl.uniform_fp16(302, 2, (K,), -1, 1)
    want = ref.conv2d_nhwc(x, w, bias, stride=2, pad=3)
    xp = torch.empty((N, H, W, 8), dtype=torch.float16, device="cuda")
    wp = torch.empty((K, 7, 7, 8), dtype=torch.float16, device="cuda")
    bolt.bolt_pad_channels_nhwc(dev(x), xp, 8)
    bolt.bolt_pad_channels_nhwc(dev(w), wp, 8)
    d = bolt.conv_desc(N, H, W, 8, K, 7, 7, 2, 3)
    P, Q = bolt.conv_out_hw(d)
    y = torch.empty((N, P, Q, K), dtype=torch.float16, device="cuda")
    bolt.bolt_conv2d_fprop_nhwc(d, xp, wp, dev(bias), y)
    torch.cuda.synchronize()
    assert_close(host(y), want, "padded stem")


# ---------------------------------------------------------------------------------------------
# back-to-back GEMM
# ---------------------------------------------------------------------------------------------
def _run_b2b_gemm(bolt, t, config=None, act0="relu", act1="relu", layout="kn"):
    M, K0 = t["A"].shape
    N0, N1 = t["W0"].shape[1], t["W1"].shape[1]
    lay = bolt.LAYOUT_KN if layout == "kn" else bolt.LAYOUT_NK
    W0 = t["W0"] if layout == "kn" else np.ascontiguousarray(t["W0"].T)
    W1 = t["W1"] if layout == "kn" else np.ascontiguousarray(t["W1"].T)
    g0 = bolt.gemm_desc(M, N0, K0, act=act0, b_layout=lay)
    g1 = bolt.gemm_desc(M, N1, N0, act=act1, b_layout=lay)
    D1 = torch.full((M, N1), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_b2b_gemm(g0, g1, dev(t["A"]), dev(W0), dev(t["b0"]), dev(W1), dev(t["b1"]), D1, config)
    torch.cuda.synchronize()
    return host(D1), g0, g1


@pytest.mark.parametrize("layout", ["kn", "nk"])
@pytest.mark.parametrize("shape", [(300, 136, 56, 104), (260, 72, 32, 24), (130, 600, 128, 64)])
def test_b2b_gemm_leading_dimensions_every_instance(bolt, shape, layout):
    """Row strides beyond the extents on A, both weight matrices and D1; what lies between the rows of the weights is NaN,
    so a kernel that reads a chunk beyond N or K (instead of taking zeros for it) fails.  Every instance of the layout."""
    M, K0, N0, N1 = shape
    lda, ldd = K0 + 16, N1 + 8
    A = wl.uniform_fp16(421, 0, (M, lda), -0.5, 0.5)
    W0, W1 = wl.uniform_fp16(421, 1, (K0, N0), -0.5, 0.5), wl.uniform_fp16(421, 3, (N0, N1), -0.5, 0.5)
    b0, b1 = wl.uniform_fp16(421, 2, (N0,), -0.5, 0.5), wl.uniform_fp16(421, 4, (N1,), -0.5, 0.5)
    want = ref.b2b_gemm(np.ascontiguousarray(A[:, :K0]), W0, b0, W1, b1)

    def padded(Wm):  # the matrix as stored, 24 poisoned halves behind every row
        src = Wm if layout == "kn" else np.ascontiguousarray(Wm.T)
        out = np.full((src.shape[0], src.shape[1] + 24), np.nan, dtype=np.float16)
        out[:, :src.shape[1]] = src
        return out
    W0s, W1s = padded(W0), padded(W1)
    lay = bolt.LAYOUT_KN if layout == "kn" else bolt.LAYOUT_NK
    g0 = bolt.gemm_desc(M, N0, K0, lda=lda, ldb=W0s.shape[1], b_layout=lay)
    g1 = bolt.gemm_desc(M, N1, N0, ldb=W1s.shape[1], ldd=ldd, b_layout=lay)
    Ad, W0d, W1d, b0d, b1d = dev(A), dev(W0s), dev(W1s), dev(b0), dev(b1)
    ids = [k for k in range(bolt.bolt_num_instances(bolt.OP_B2B_GEMM)) if bolt.bolt_instance_supports(bolt.OP_B2B_GEMM, k, g0, g1)]
    assert ids, "no instance for %s weights %s" % (shape, layout)
    for cfg in [None] + [{"kernel_id": k} for k in ids]:
        _say("b2b gemm leading dimensions %s weights %s config %s" % (shape, layout, cfg))
        D1 = torch.zeros((M, ldd), dtype=torch.float16, device="cuda")
        bolt.bolt_b2b_gemm(g0, g1, Ad, W0d, b0d, W1d, b1d, D1, cfg)
        torch.cuda.synchronize()
        got = host(D1)
        assert_close(got[:, :N1], want, "b2b gemm leading dimensions %s weights %s config %s" % (shape, layout, cfg))
        assert not got[:, N1:].any(), "columns beyond N1 were written (config %s)" % (cfg,)


def test_config3_b2b_gemm_every_instance(bolt):
    t = wl.config3()
    want = ref.b2b_gemm(t["A"], t["W0"], t["b0"], t["W1"], t["b1"])
    g0 = bolt.gemm_desc(16384, 64, 256)
    g1 = bolt.gemm_desc(16384, 128, 64)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_GEMM)):
        if bolt.bolt_instance_supports(bolt.OP_B2B_GEMM, kid, g0, g1):
            _say("config3 b2b gemm instance %d %s" % (kid, bolt.bolt_instance_config(bolt.OP_B2B_GEMM, kid).as_dict()))
            got, _, _ = _run_b2b_gemm(bolt, t, {"kernel_id": kid})
            assert_close(got, want, "config3 instance %d" % kid)
            ran += 1
    assert ran >= 2
    got, _, _ = _run_b2b_gemm(bolt, t)
    assert_close(got, want, "config3 heuristic")


B2B_GEMM_SHAPES = [  # M, K0, N0, N1 (ragged M, every compiled (N0T, N1T) family, K0 tails)
    (1000, 72, 64, 128), (333, 256, 64, 16), (515, 256, 128, 64), (700, 96, 32, 96), (129, 8, 8, 8),
    (260, 200, 64, 256), (100, 64, 24, 72), (64, 128, 128, 128),
    (515, 576, 128, 64),  # a row-major W0 beyond LDS: only the multi-stage kernel streams it
]


@pytest.mark.parametrize("shape", B2B_GEMM_SHAPES)
def test_b2b_gemm_shapes_every_instance(bolt, shape):
    M, K0, N0, N1 = shape
    t = dict(A=wl.uniform_fp16(401, 0, (M, K0), -0.5, 0.5), W0=wl.uniform_fp16(401, 1, (K0, N0), -0.5, 0.5),
             b0=wl.uniform_fp16(401, 2, (N0,), -0.5, 0.5), W1=wl.uniform_fp16(401, 3, (N0, N1), -0.5, 0.5),
             b1=wl.uniform_fp16(401, 4, (N1,), -0.5, 0.5))
    want = ref.b2b_gemm(t["A"], t["W0"], t["b0"], t["W1"], t["b1"])
    g0, g1 = bolt.gemm_desc(M, N0, K0), bolt.gemm_desc(M, N1, N0)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_GEMM)):
        if bolt.bolt_instance_supports(bolt.OP_B2B_GEMM, kid, g0, g1):
            _say("b2b gemm %s instance %d" % (shape, kid))
            got, _, _ = _run_b2b_gemm(bolt, t, {"kernel_id": kid})
            assert_close(got, want, "b2b gemm %s instance %d" % (shape, kid))
            ran += 1
    assert ran >= 1, "no instance for %s" % (shape,)


@pytest.mark.parametrize("shape", [(1000, 72, 64, 128), (515, 576, 128, 64), (700, 96, 32, 96), (260, 200, 64, 256),
                                   (333, 256, 64, 16), (64, 128, 128, 128)])
def test_b2b_gemm_reduction_contiguous_weights_every_instance(bolt, shape):
    """Weights stored [N][K] (the multi-stage fused kernel; Table 1's K0 = 576, N0 = 128 row only runs here)."""
    M, K0, N0, N1 = shape
    t = dict(A=wl.uniform_fp16(403, 0, (M, K0), -0.5, 0.5), W0=wl.uniform_fp16(403, 1, (K0, N0), -0.5, 0.5),
             b0=wl.uniform_fp16(403, 2, (N0,), -0.5, 0.5), W1=wl.uniform_fp16(403, 3, (N0, N1), -0.5, 0.5),
             b1=wl.uniform_fp16(403, 4, (N1,), -0.5, 0.5))
    want = ref.b2b_gemm(t["A"], t["W0"], t["b0"], t["W1"], t["b1"])
    g0 = bolt.gemm_desc(M, N0, K0, b_layout=bolt.LAYOUT_NK)
    g1 = bolt.gemm_desc(M, N1, N0, b_layout=bolt.LAYOUT_NK)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_GEMM)):
        if bolt.bolt_instance_supports(bolt.OP_B2B_GEMM, kid, g0, g1):
            _say("b2b gemm [N][K] %s instance %d" % (shape, kid))
            got, _, _ = _run_b2b_gemm(bolt, t, {"kernel_id": kid}, layout="nk")
            assert_close(got, want, "b2b gemm [N][K] %s instance %d" % (shape, kid))
            ran += 1
    assert ran >= 1, "no instance for %s" % (shape,)


def test_b2b_gemm_integer_bit_exact(bolt):
    M, K0, N0, N1 = 300, 64, 64, 128
    t = dict(A=wl.integer_fp16(402, 0, (M, K0), -1, 1), W0=wl.integer_fp16(402, 1, (K0, N0), -1, 1),
             b0=wl.integer_fp16(402, 2, (N0,), -2, 2), W1=wl.integer_fp16(402, 3, (N0, N1), -1, 1),
             b1=wl.integer_fp16(402, 4, (N1,), -2, 2))
    # every partial sum is an integer below 2^24, exact in FP32 and in double, so both sides round the
    # same exact value to FP16: the results must be identical
    want = ref.b2b_gemm(t["A"], t["W0"], t["b0"], t["W1"], t["b1"], act1="none")
    g0, g1 = bolt.gemm_desc(M, N0, K0), bolt.gemm_desc(M, N1, N0, act="none")
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_GEMM)):
        if bolt.bolt_instance_supports(bolt.OP_B2B_GEMM, kid, g0, g1):
            got, _, _ = _run_b2b_gemm(bolt, t, {"kernel_id": kid}, act1="none")
            assert_bit_equal(got, want, "b2b gemm integer instance %d" % kid)


# ---------------------------------------------------------------------------------------------
# back-to-back conv
# ---------------------------------------------------------------------------------------------
def _run_b2b_conv(bolt, t, stride, pad, config=None):
    N, H, W, Cc = t["x"].shape
    K0, R, S, _ = t["w0"].shape
    K1 = t["w1"].shape[0]
    c0 = bolt.conv_desc(N, H, W, Cc, K0, R, S, stride, pad)
    P, Q = bolt.conv_out_hw(c0)
    c1 = bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0)
    y = torch.full((N, P, Q, K1), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_b2b_conv(c0, c1, dev(t["x"]), dev(t["w0"]), dev(t["b0"]), dev(t["w1"]), dev(t["b1"]), y, config)
    torch.cuda.synchronize()
    return host(y), c0, c1


def test_config4_b2b_conv_small_batch_every_instance(bolt):
    t = wl.config4(batch=2)
    want = ref.b2b_conv(t["x"], t["w0"], t["b0"], t["w1"], t["b1"], stride=1, pad=1)
    c0 = bolt.conv_desc(2, 56, 56, 64, 64, 3, 3, 1, 1)
    c1 = bolt.conv_desc(2, 56, 56, 64, 256, 1, 1, 1, 0)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_CONV)):
        if bolt.bolt_instance_supports(bolt.OP_B2B_CONV, kid, c0, c1):
            _say("config4 b2b conv instance %d %s" % (kid, bolt.bolt_instance_config(bolt.OP_B2B_CONV, kid).as_dict()))
            got, _, _ = _run_b2b_conv(bolt, t, 1, 1, {"kernel_id": kid})
            assert_close(got, want, "config4 (batch 2) instance %d" % kid)
            ran += 1
    assert ran >= 2


def test_config4_b2b_conv_full_size_tuned_sampled_rows(bolt):
    t = wl.config4()
    c0 = bolt.conv_desc(32, 56, 56, 64, 64, 3, 3, 1, 1)
    c1 = bolt.conv_desc(32, 56, 56, 64, 256, 1, 1, 1, 0)
    x, w0, b0, w1, b1 = (dev(t[k]) for k in ("x", "w0", "b0", "w1", "b1"))
    y = torch.full((32, 56, 56, 256), float("nan"), dtype=torch.float16, device="cuda")
    res = bolt.bolt_tune(bolt.OP_B2B_CONV, c0, c1, [x, w0, b0, w1, b1, y])
    _say("config4 tuned: %s %.4f ms, %d tried" % (res.config.as_dict(), res.ms, res.tried))
    y.fill_(float("nan"))
    bolt.bolt_b2b_conv(c0, c1, x, w0, b0, w1, b1, y, res.config)
    torch.cuda.synchronize()
    got = host(y).reshape(-1, 256)
    assert np.all(np.isfinite(got))
    rows = _sample_idx(got.shape[0], 300, 2)
    want = ref.b2b_conv_rows(t["x"], t["w0"], t["b0"], t["w1"], t["b1"], rows, stride=1, pad=1)
    assert_close(got[rows], want, "config4 full size, tuned, sampled rows")


B2B_CONV_SHAPES = [  # N H W C K0 stride K1
    (2, 20, 20, 8, 48, 2, 48), (1, 15, 17, 48, 48, 1, 48), (2, 12, 12, 64, 64, 2, 64), (1, 9, 9, 16, 32, 1, 32),
    (1, 11, 11, 24, 128, 1, 128),
    # stride-1 "same" first op over whole 64-channel chunks with a wide second op: the instances that take op1 in
    # chunks of 64 columns (a partial last chunk, a chunk that is skipped, two halo buffers)
    (1, 10, 12, 64, 64, 1, 200), (2, 9, 10, 64, 40, 1, 136), (1, 12, 9, 128, 64, 1, 256),
]


@pytest.mark.parametrize("shape", B2B_CONV_SHAPES)
def test_b2b_conv_shapes_every_instance(bolt, shape):
    N, H, W, Cc, K0, stride, K1 = shape
    t = dict(x=wl.uniform_fp16(501, 0, (N, H, W, Cc), -1, 1), w0=wl.normal_fp16(501, 1, (K0, 3, 3, Cc), (2.0 / (9 * Cc)) ** 0.5),
             b0=wl.uniform_fp16(501, 2, (K0,), -1, 1), w1=wl.normal_fp16(501, 3, (K1, 1, 1, K0), (2.0 / K0) ** 0.5),
             b1=wl.uniform_fp16(501, 4, (K1,), -1, 1))
    want = ref.b2b_conv(t["x"], t["w0"], t["b0"], t["w1"], t["b1"], stride=stride, pad=1)
    c0 = bolt.conv_desc(N, H, W, Cc, K0, 3, 3, stride, 1)
    P, Q = bolt.conv_out_hw(c0)
    c1 = bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_CONV)):
        if bolt.bolt_instance_supports(bolt.OP_B2B_CONV, kid, c0, c1):
            _say("b2b conv %s instance %d" % (shape, kid))
            got, _, _ = _run_b2b_conv(bolt, t, stride, 1, {"kernel_id": kid})
            assert_close(got, want, "b2b conv %s instance %d" % (shape, kid))
            ran += 1
    assert ran >= 1, "no instance for %s" % (shape,)


# ---------------------------------------------------------------------------------------------
# config 5: every distinct ResNet-50 layer shape at full size, tuned, sampled outputs
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("index", list(range(23)))
def test_config5_layer_full_size_tuned_sampled(bolt, index):
    shape, cnt, t = wl.config5_layer(index)
    x_log, w_log, bias = t["x"], t["w"], t["bias"]
    x, w = dev(x_log), dev(w_log)
    if shape.c_logical:
        xp = torch.empty(x_log.shape[:-1] + (shape.C,), dtype=torch.float16, device="cuda")
        wp = torch.empty(w_log.shape[:-1] + (shape.C,), dtype=torch.float16, device="cuda")
        bolt.bolt_pad_channels_nhwc(x, xp, shape.C)
        bolt.bolt_pad_channels_nhwc(w, wp, shape.C)
        x, w = xp, wp
    d = bolt.conv_desc(shape.N, shape.H, shape.W, shape.C, shape.K, shape.R, shape.S, shape.stride, shape.pad)
    y = torch.full((shape.N, shape.P, shape.Q, shape.K), float("nan"), dtype=torch.float16, device="cuda")
    ws_bytes = bolt.bolt_workspace_bytes(bolt.OP_CONV2D, d)
    ws = torch.empty(max(ws_bytes, 16) // 4, dtype=torch.float32, device="cuda")
    b = dev(bias)
    res = bolt.bolt_tune(bolt.OP_CONV2D, d, None, [x, w, b, y], ws)
    _say("layer %d %s: %s %.4f ms (%d tried) %.1f TFLOP/s" %
         (index, shape, res.config.as_dict(), res.ms, res.tried, shape.flops / res.ms / 1e9))
    y.fill_(float("nan"))
    bolt.bolt_conv2d_fprop_nhwc(d, x, w, b, y, res.config, ws)
    torch.cuda.synchronize()
    got = host(y).reshape(-1)
    assert np.all(np.isfinite(got)), "unwritten or non-finite outputs"
    idx = _sample_idx(got.size, 4000, 10 + index)
    want = ref.conv2d_nhwc_at(x_log, w_log, idx, bias, stride=shape.stride, pad=shape.pad)
    assert_close(got[idx], want, "config5 layer %d" % index)


# ---------------------------------------------------------------------------------------------
# maximum sizes: an input tensor just below the 2 GiB that one buffer descriptor addresses
# ---------------------------------------------------------------------------------------------
def test_conv_input_just_below_the_size_limit_sampled(bolt):
    N, H, W, Cc, K = 8, 512, 512, 504, 64          # 8 * 512 * 512 * 504 = 2^30 - 16.8 M elements = 2.11 GB of FP16
    assert bolt.bolt_check(bolt.OP_CONV2D, bolt.conv_desc(N, H, W, Cc + 8, K, 3, 3, 1, 1)) == 2  # one step further: unsupported
    block = wl.uniform_fp16(601, 0, (H, W, Cc), -1, 1)
    x = np.empty((N, H, W, Cc), np.float16)
    for n, scale in enumerate((1.0, -1.0, 0.5, -0.5, 0.25, -0.25, 2.0, -2.0)):  # exact in FP16, every image different
        np.multiply(block, np.float16(scale), out=x[n])
    del block
    bias = wl.uniform_fp16(601, 2, (K,), -1, 1)
    xd = dev(x)
    edge_rows = np.array([0, 1, W - 1, W, N * H * W - W - 1, N * H * W - 2, N * H * W - 1])  # first / last pixels: smallest and largest offsets
    for (R, pad) in ((3, 1), (1, 0)):               # the im2col gather, and the GEMM addressing of 1x1 / stride 1
        w = wl.normal_fp16(601, 1, (K, R, R, Cc), (2.0 / (R * R * Cc)) ** 0.5)
        d = bolt.conv_desc(N, H, W, Cc, K, R, R, 1, pad)
        y = torch.full((N, H, W, K), float("nan"), dtype=torch.float16, device="cuda")
        _say("conv %dx%d on a %.2f GB input" % (R, R, x.nbytes / 1e9))
        bolt.bolt_conv2d_fprop_nhwc(d, xd, dev(w), dev(bias), y)
        torch.cuda.synchronize()
        got = host(y).reshape(-1)
        assert np.all(np.isfinite(got)), "unwritten or non-finite outputs"
        idx = np.unique(np.concatenate([_sample_idx(got.size, 1500, 7), (edge_rows[:, None] * K + np.arange(K)[None, :]).reshape(-1)]))
        want = ref.conv2d_nhwc_at(x, w, idx, bias, stride=1, pad=pad)
        assert_close(got[idx], want, "conv %dx%d, input just below 2 GiB" % (R, R))
        del y


# ---------------------------------------------------------------------------------------------
# layout transformation
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(2, 3, 32, 32, 8), (1, 3, 224, 224, 8), (3, 64, 9, 11, 64), (2, 70, 13, 5, 72), (1, 1, 1, 1, 8),
                                   (2, 136, 7, 7, 136), (1, 46, 20, 26, 48)])
def test_layout_transforms_bit_exact(bolt, shape):
    N, Cc, H, W, C8 = shape
    x = wl.uniform_fp16(501, 0, (N, Cc, H, W), -4, 4)
    y = torch.full((N, H, W, C8), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_nchw_to_nhwc(dev(x), y)
    torch.cuda.synchronize()
    assert_bit_equal(host(y), ref.nchw_to_nhwc(x, C8), "nchw -> nhwc %s" % (shape,))
    back = torch.full((N, Cc, H, W), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_nhwc_to_nchw(y, back)
    torch.cuda.synchronize()
    assert_bit_equal(host(back), x, "nhwc -> nchw %s" % (shape,))
    assert_bit_equal(host(back), ref.nhwc_to_nchw(host(y), Cc), "nhwc -> nchw vs oracle %s" % (shape,))


def test_first_layer_from_nchw_input(bolt):
    # a framework's NCHW image through transform + padding, the tuned stem convolution, and back to NCHW
    x = wl.uniform_fp16(502, 0, (2, 3, 40, 36), -1, 1)
    w = wl.normal_fp16(502, 1, (64, 7, 7, 3), 0.1)
    b = wl.uniform_fp16(502, 2, (64,), -1, 1)
    want = ref.nhwc_to_nchw(ref.conv2d_nhwc(ref.nchw_to_nhwc(x), w, b, stride=2, pad=3))
    xp = torch.empty((2, 40, 36, 8), dtype=torch.float16, device="cuda")
    wp = torch.empty((64, 7, 7, 8), dtype=torch.float16, device="cuda")
    bolt.bolt_nchw_to_nhwc(dev(x), xp)
    bolt.bolt_pad_channels_nhwc(dev(w), wp, 8)
    d = bolt.conv_desc(2, 40, 36, 8, 64, 7, 7, 2, 3)
    P, Q = bolt.conv_out_hw(d)
    y = torch.empty((2, P, Q, 64), dtype=torch.float16, device="cuda")
    bolt.bolt_conv2d_fprop_nhwc(d, xp, wp, dev(b), y)
    out = torch.empty((2, 64, P, Q), dtype=torch.float16, device="cuda")
    bolt.bolt_nhwc_to_nchw(y, out)
    torch.cuda.synchronize()
    assert_close(host(out), want, "NCHW in, NCHW out")


# ---------------------------------------------------------------------------------------------
# residual epilogue (Eq. 1 with C a full matrix)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("layout", ["kn", "nk"])
def test_gemm_residual_every_instance(bolt, layout):
    lay = bolt.LAYOUT_KN if layout == "kn" else bolt.LAYOUT_NK
    for (M, N, K, act) in [(333, 136, 200, "relu"), (200, 72, 64, "gelu"), (1, 8, 8, "none")]:
        A = wl.uniform_fp16(401, 0, (M, K), -1, 1)
        B = wl.uniform_fp16(401, 1, (K, N), -1, 1)
        bias = wl.uniform_fp16(401, 2, (N,), -1, 1)
        Cm = wl.uniform_fp16(401, 3, (M, N), -4, 4)
        want = ref.gemm_residual(A, B, bias, Cm, 1.0, 1.0, 0.5, act)
        d = bolt.gemm_desc(M, N, K, act=act, b_layout=lay)
        Bd = dev(B) if layout == "kn" else dev(np.ascontiguousarray(B.T))
        ran = 0
        for kid in range(bolt.bolt_num_instances(bolt.OP_GEMM)):
            if not bolt.bolt_instance_supports(bolt.OP_GEMM, kid, d):
                continue
            _say("gemm residual %s %dx%dx%d instance %d" % (layout, M, N, K, kid))
            D = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
            try:
                bolt.bolt_gemm_epilogue_residual(d, dev(A), Bd, dev(bias), dev(Cm), D, 0.5, {"kernel_id": kid})
            except bolt.BoltError as e:
                assert e.status == 2  # a persistent instance: no residual epilogue
                continue
            torch.cuda.synchronize()
            assert_close(host(D), want, "gemm residual instance %d" % kid)
            ran += 1
        assert ran >= 3


@pytest.mark.parametrize("case", [(2, 12, 12, 64, 72, 3, 3, 1, 1), (1, 17, 13, 24, 40, 3, 3, 2, 1), (3, 9, 11, 64, 72, 1, 1, 1, 0),
                                  (2, 9, 10, 256, 72, 3, 3, 1, 1), (2, 10, 13, 46, 32, 5, 5, 1, 2), (2, 7, 7, 512, 64, 3, 3, 1, 1)])
def test_conv_residual_every_instance_in_place_and_split_k(bolt, case):
    N, H, W, Cc, K, R, S, stride, pad = case
    x = wl.uniform_fp16(402, 0, (N, H, W, Cc), -1, 1)
    w = wl.normal_fp16(402, 1, (K, R, S, Cc), (2.0 / (R * S * Cc)) ** 0.5)
    bias = wl.uniform_fp16(402, 2, (K,), -1, 1)
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad)
    P, Q = bolt.conv_out_hw(d)
    res = wl.uniform_fp16(402, 3, (N, P, Q, K), -2, 2)
    want = ref.conv2d_nhwc_residual(x, w, bias, res, stride=stride, pad=pad)
    ws = torch.empty(max(bolt.bolt_workspace_bytes(bolt.OP_CONV2D, d), 16), dtype=torch.uint8, device="cuda")
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_CONV2D)):
        if not bolt.bolt_instance_supports(bolt.OP_CONV2D, kid, d):
            continue
        _say("conv residual %s instance %d" % (case, kid))
        y = dev(res).clone()  # in place: the residual is the output buffer
        try:
            bolt.bolt_conv2d_fprop_nhwc_residual(d, dev(x), dev(w), dev(bias), y, y, 1.0, {"kernel_id": kid})
        except bolt.BoltError as e:
            assert e.status == 2
            continue
        torch.cuda.synchronize()
        assert_close(host(y), want, "conv residual %s instance %d" % (case, kid))
        ran += 1
        if bolt.bolt_check(bolt.OP_CONV2D, d, None, {"kernel_id": kid, "split_k": 2}) == 0:
            y2 = torch.full((N, P, Q, K), float("nan"), dtype=torch.float16, device="cuda")
            bolt.bolt_conv2d_fprop_nhwc_residual(d, dev(x), dev(w), dev(bias), dev(res), y2, 1.0,
                                                 {"kernel_id": kid, "split_k": 2}, ws)
            torch.cuda.synchronize()
            assert_close(host(y2), want, "conv residual %s instance %d split-K" % (case, kid))
    assert ran >= 3
    y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_conv2d_fprop_nhwc_residual(d, dev(x), dev(w), dev(bias), dev(res), y)  # built-in pick rule
    torch.cuda.synchronize()
    assert_close(host(y), want, "conv residual %s heuristic" % (case,))


def test_residual_integer_bit_exact(bolt):
    A = wl.integer_fp16(403, 0, (300, 72), -3, 3)
    B = wl.integer_fp16(403, 1, (72, 136), -3, 3)
    bias = wl.integer_fp16(403, 2, (136,), -4, 4)
    Cm = wl.integer_fp16(403, 3, (300, 136), -9, 9)
    want = ref.gemm_residual(A, B, bias, Cm, 1.0, 1.0, -2.0, "relu")
    d = bolt.gemm_desc(300, 136, 72)
    D = torch.empty((300, 136), dtype=torch.float16, device="cuda")
    bolt.bolt_gemm_epilogue_residual(d, dev(A), dev(B), dev(bias), dev(Cm), D, -2.0)
    torch.cuda.synchronize()
    assert_bit_equal(host(D), want, "integer gemm residual")


@pytest.mark.parametrize("shape", [(1000, 72, 64, 128), (515, 576, 128, 64), (700, 96, 32, 96), (260, 200, 64, 256),
                                   (333, 256, 64, 16), (129, 64, 64, 64)])
def test_b2b_gemm_residual_every_instance_and_tuner(bolt, shape):
    """Fused pair with Eq. 2's C1 a full matrix (weights stored [N][K]); also in place and through bolt_tune."""
    M, K0, N0, N1 = shape
    A, W0 = wl.uniform_fp16(405, 0, (M, K0), -0.5, 0.5), wl.uniform_fp16(405, 1, (K0, N0), -0.5, 0.5)
    b0, W1 = wl.uniform_fp16(405, 2, (N0,), -0.5, 0.5), wl.uniform_fp16(405, 3, (N0, N1), -0.5, 0.5)
    b1, Cm = wl.uniform_fp16(405, 4, (N1,), -0.5, 0.5), wl.uniform_fp16(405, 5, (M, N1), -4, 4)
    want = ref.b2b_gemm_residual(A, W0, b0, W1, b1, Cm, gamma=0.5)
    g0 = bolt.gemm_desc(M, N0, K0, b_layout=bolt.LAYOUT_NK)
    g1 = bolt.gemm_desc(M, N1, N0, b_layout=bolt.LAYOUT_NK)
    W0d, W1d = dev(np.ascontiguousarray(W0.T)), dev(np.ascontiguousarray(W1.T))
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_GEMM_RES)):
        if not bolt.bolt_instance_supports(bolt.OP_B2B_GEMM_RES, kid, g0, g1):
            continue
        _say("b2b gemm residual %s instance %d" % (shape, kid))
        D = dev(Cm).clone()  # in place: the residual is the output buffer
        bolt.bolt_b2b_gemm_residual(g0, g1, dev(A), W0d, dev(b0), W1d, dev(b1), D, D, 0.5, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(D), want, "b2b gemm residual %s instance %d" % (shape, kid))
        ran += 1
    assert ran >= 1, "no instance for %s" % (shape,)
    D = torch.full((M, N1), float("nan"), dtype=torch.float16, device="cuda")
    r = bolt.bolt_tune(bolt.OP_B2B_GEMM_RES, g0, g1, [dev(A), W0d, dev(b0), W1d, dev(b1), D, dev(Cm)])
    assert bolt.bolt_instance_supports(bolt.OP_B2B_GEMM_RES, r.config.kernel_id, g0, g1) and r.tried == ran
    D.fill_(float("nan"))
    bolt.bolt_b2b_gemm_residual(g0, g1, dev(A), W0d, dev(b0), W1d, dev(b1), dev(Cm), D, 0.5, r.config)
    torch.cuda.synchronize()
    assert_close(host(D), want, "b2b gemm residual %s tuned" % (shape,))


@pytest.mark.parametrize("shape", B2B_CONV_SHAPES + [(2, 14, 14, 64, 64, 1, 256), (1, 10, 12, 32, 64, 1, 200)])
def test_b2b_conv_residual_every_instance_and_tuner(bolt, shape):
    """The tail of a bottleneck block: 3x3 -> 1x1 + skip connection + ReLU in one launch."""
    N, H, W, Cc, K0, stride, K1 = shape
    x, w0 = wl.uniform_fp16(406, 0, (N, H, W, Cc), -1, 1), wl.normal_fp16(406, 1, (K0, 3, 3, Cc), (2.0 / (9 * Cc)) ** 0.5)
    b0, w1 = wl.uniform_fp16(406, 2, (K0,), -1, 1), wl.normal_fp16(406, 3, (K1, 1, 1, K0), (2.0 / K0) ** 0.5)
    b1 = wl.uniform_fp16(406, 4, (K1,), -1, 1)
    c0 = bolt.conv_desc(N, H, W, Cc, K0, 3, 3, stride, 1)
    P, Q = bolt.conv_out_hw(c0)
    c1 = bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0)
    res = wl.uniform_fp16(406, 5, (N, P, Q, K1), -2, 2)
    want = ref.b2b_conv_residual(x, w0, b0, w1, b1, res, stride=stride, pad=1)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_B2B_CONV_RES)):
        if not bolt.bolt_instance_supports(bolt.OP_B2B_CONV_RES, kid, c0, c1):
            continue
        _say("b2b conv residual %s instance %d" % (shape, kid))
        y = torch.full((N, P, Q, K1), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_b2b_conv_residual(c0, c1, dev(x), dev(w0), dev(b0), dev(w1), dev(b1), dev(res), y, 1.0, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(y), want, "b2b conv residual %s instance %d" % (shape, kid))
        ran += 1
    assert ran >= 1, "no instance for %s" % (shape,)
    y = dev(res).clone()
    r = bolt.bolt_tune(bolt.OP_B2B_CONV_RES, c0, c1, [dev(x), dev(w0), dev(b0), dev(w1), dev(b1), y, dev(res)])
    assert r.tried == ran
    y = dev(res).clone()  # in place, tuned config
    bolt.bolt_b2b_conv_residual(c0, c1, dev(x), dev(w0), dev(b0), dev(w1), dev(b1), y, y, 1.0, r.config)
    torch.cuda.synchronize()
    assert_close(host(y), want, "b2b conv residual %s tuned, in place" % (shape,))
    # an instance without the residual epilogue is refused, not silently run without it
    plain_only = [k for k in range(bolt.bolt_num_instances(bolt.OP_B2B_CONV))
                  if bolt.bolt_instance_supports(bolt.OP_B2B_CONV, k, c0, c1)
                  and not bolt.bolt_instance_supports(bolt.OP_B2B_CONV_RES, k, c0, c1)]
    if plain_only:
        with pytest.raises(bolt.BoltError) as e:
            bolt.bolt_b2b_conv_residual(c0, c1, dev(x), dev(w0), dev(b0), dev(w1), dev(b1), dev(res), y, 1.0,
                                        {"kernel_id": plain_only[0]})
        assert e.value.status == 2


@pytest.mark.parametrize("shape", [(1000, 72, 64, 128), (333, 256, 64, 16), (129, 64, 32, 96)])
def test_b2b_gemm_residual_row_major_weights_every_instance(bolt, shape):
    """Weights stored [K][N] run on the weights-resident kernels only; their residual epilogue reads C straight from
    global memory.  Closeness on fractions with a strided C, bit-exactness on small integers, every instance."""
    M, K0, N0, N1 = shape
    g0, g1 = bolt.gemm_desc(M, N0, K0), bolt.gemm_desc(M, N1, N0)
    ids = [k for k in range(bolt.bolt_num_instances(bolt.OP_B2B_GEMM_RES)) if bolt.bolt_instance_supports(bolt.OP_B2B_GEMM_RES, k, g0, g1)]
    assert ids, "no instance for %s" % (shape,)
    A, W0 = wl.uniform_fp16(415, 0, (M, K0), -0.5, 0.5), wl.uniform_fp16(415, 1, (K0, N0), -0.5, 0.5)
    b0, W1 = wl.uniform_fp16(415, 2, (N0,), -0.5, 0.5), wl.uniform_fp16(415, 3, (N0, N1), -0.5, 0.5)
    b1, Cfull = wl.uniform_fp16(415, 4, (N1,), -0.5, 0.5), wl.uniform_fp16(415, 5, (M, N1 + 24), -4, 4)
    want = ref.b2b_gemm_residual(A, W0, b0, W1, b1, np.ascontiguousarray(Cfull[:, :N1]), gamma=0.5)
    Ai, W0i = wl.integer_fp16(416, 0, (M, K0), -2, 2), wl.integer_fp16(416, 1, (K0, N0), -1, 1)
    W1i = wl.integer_fp16(416, 3, (N0, N1), -1, 1)
    for Wm in (W0i, W1i):  # sparse, so that every intermediate stays exactly representable
        Wm[np.arange(Wm.shape[0])[:, None] % 4 != np.arange(Wm.shape[1])[None, :] % 4] = 0
    b0i, b1i = wl.integer_fp16(416, 2, (N0,), -2, 2), wl.integer_fp16(416, 4, (N1,), -2, 2)
    Ci = wl.integer_fp16(416, 5, (M, N1), -9, 9)
    want_i = ref.b2b_gemm_residual(Ai, W0i, b0i, W1i, b1i, Ci, gamma=-3.0)
    assert np.abs(want_i.astype(np.float64)).max() < 2048
    for kid in ids:
        _say("b2b gemm residual [K][N] %s instance %d" % (shape, kid))
        D = torch.full((M, N1), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_b2b_gemm_residual(g0, g1, dev(A), dev(W0), dev(b0), dev(W1), dev(b1), dev(Cfull), D, 0.5, {"kernel_id": kid})  # ldc = N1 + 24
        torch.cuda.synchronize()
        assert_close(host(D), want, "b2b gemm residual [K][N] %s instance %d" % (shape, kid))
        D = dev(Ci).clone()  # in place
        bolt.bolt_b2b_gemm_residual(g0, g1, dev(Ai), dev(W0i), dev(b0i), dev(W1i), dev(b1i), D, D, -3.0, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_bit_equal(host(D), want_i, "integer b2b gemm residual [K][N] %s instance %d" % (shape, kid))


def test_b2b_residual_integer_bit_exact(bolt):
    M, K0, N0, N1 = 300, 64, 32, 96
    A, W0 = wl.integer_fp16(407, 0, (M, K0), -2, 2), wl.integer_fp16(407, 1, (K0, N0), -1, 1)
    b0, W1 = wl.integer_fp16(407, 2, (N0,), -2, 2), wl.integer_fp16(407, 3, (N0, N1), -1, 1)
    b1, Cm = wl.integer_fp16(407, 4, (N1,), -2, 2), wl.integer_fp16(407, 5, (M, N1), -9, 9)
    want = ref.b2b_gemm_residual(A, W0, b0, W1, b1, Cm, gamma=-3.0)
    g0 = bolt.gemm_desc(M, N0, K0, b_layout=bolt.LAYOUT_NK)
    g1 = bolt.gemm_desc(M, N1, N0, b_layout=bolt.LAYOUT_NK)
    D = torch.empty((M, N1), dtype=torch.float16, device="cuda")
    bolt.bolt_b2b_gemm_residual(g0, g1, dev(A), dev(np.ascontiguousarray(W0.T)), dev(b0), dev(np.ascontiguousarray(W1.T)),
                                dev(b1), dev(Cm), D, -3.0)
    torch.cuda.synchronize()
    assert_bit_equal(host(D), want, "integer b2b gemm residual")


# ---------------------------------------------------------------------------------------------
# first layers: at most 4 input channels, unpadded NHWC or NCHW input (Section 3.2.3 folded into the loader)
# ---------------------------------------------------------------------------------------------
FIRST_LAYERS = [
    # N H W C K R S stride pad
    (2, 40, 300, 3, 64, 7, 7, 2, 3),          # the stem's filter; Q = 150: two column tiles, the second ragged
    (1, 23, 23, 3, 72, 7, 7, 2, 3),           # two channel tiles, the second 8 wide
    (2, 17, 19, 3, 64, 3, 3, 1, 1),           # stride 1 (2-byte fragment reads), 9 planes
    (1, 16, 140, 3, 32, 3, 3, 1, 1),          # stride 1, Q = 140: two column tiles
    (2, 15, 33, 1, 8, 5, 5, 2, 2),            # one channel
    (1, 12, 20, 2, 16, 3, 5, (1, 2), (1, 2)),  # even C (also legal for the alignment-2 kernels), S != R
    (1, 9, 30, 4, 24, 5, 8, (2, 1), (2, 3)),   # C = 4, S = 8 (no masked tap), R * C = 20
    (3, 8, 8, 3, 16, 1, 1, 1, 0),             # 1x1
    (1, 20, 21, 3, 64, 7, 2, (3, 2), (0, 0)),  # stride_h = 3, no padding
]


@pytest.mark.parametrize("shape", FIRST_LAYERS)
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
def test_first_layer_conv_every_instance(bolt, shape, layout):
    """The input is read where it lies: no channel padding, no transformation pass.  NCHW parity is against the
    oracle's convolution of the oracle's transformed tensor; integers (bit-exact) and fractions on every instance."""
    N, H, W, Cc, K, R, S, stride, pad = shape
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad, alpha=0.5, beta=-1.0, act="relu", x_layout=layout)
    P, Q = bolt.conv_out_hw(d)
    ids = [k for k in range(bolt.bolt_num_instances(bolt.OP_CONV2D)) if bolt.bolt_instance_supports(bolt.OP_CONV2D, k, d)]
    smallc = [k for k in ids if bolt.bolt_instance_config(bolt.OP_CONV2D, k).tile_k == 32 and bolt.bolt_instance_config(bolt.OP_CONV2D, k).mfma_shape == 16]
    assert smallc, "no first-layer instance for %s" % (shape,)
    if layout == "nchw" or Cc % 2:
        assert smallc == ids
    x = wl.uniform_fp16(501, 0, (N, H, W, Cc), -1, 1)
    w = wl.normal_fp16(501, 1, (K, R, S, Cc), (2.0 / (R * S * Cc)) ** 0.5)
    b = wl.uniform_fp16(501, 2, (K,), -1, 1)
    xi = wl.integer_fp16(502, 0, (N, H, W, Cc), -3, 3)
    wi = wl.integer_fp16(502, 1, (K, R, S, Cc), -2, 2)
    bi = wl.integer_fp16(502, 2, (K,), -4, 4)
    want = ref.conv2d_nhwc(x, w, b, stride=stride, pad=pad, alpha=0.5, beta=-1.0, act="relu")
    want_i = ref.conv2d_nhwc(xi, wi, bi, stride=stride, pad=pad, alpha=0.5, beta=-1.0, act="relu")
    assert np.abs(want_i.astype(np.float64)).max() < 1024  # alpha = 0.5: halves of integers below 2048 are exact
    as_given = (lambda a: a) if layout == "nhwc" else ref.nhwc_to_nchw
    if layout == "nchw":  # the oracle's own transformation, both ways: what the kernel is handed is really NCHW
        assert np.array_equal(ref.nchw_to_nhwc(as_given(x)), x)
    xd, xid = dev(as_given(x)), dev(as_given(xi))
    for kid in smallc:
        _say("first layer %s %s instance %d" % (shape, layout, kid))
        y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_conv2d_fprop_nhwc(d, xd, dev(w), dev(b), y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(y), want, "first layer %s %s instance %d" % (shape, layout, kid))
        y.fill_(float("nan"))
        bolt.bolt_conv2d_fprop_nhwc(d, xid, dev(wi), dev(bi), y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_bit_equal(host(y), want_i, "integer first layer %s %s instance %d" % (shape, layout, kid))
    # no config: the built-in pick rule; no bias; another activation
    d2 = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad, act="hardswish", x_layout=layout)
    y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_conv2d_fprop_nhwc(d2, xd, dev(w), None, y)
    torch.cuda.synchronize()
    assert_close(host(y), ref.conv2d_nhwc(x, w, None, stride=stride, pad=pad, act="hardswish"), "first layer %s %s heuristic" % (shape, layout))


def test_first_layer_conv_equals_the_padded_path_and_ignores_infinite_neighbours(bolt):
    """Channel padding is a pure re-scheduling (Section 3.2.3): the unpadded first-layer kernel and the padded C = 8
    convolution agree bit for bit on integers.  A tap past the filter's width reads the neighbouring pixel's data
    under a zero weight: an infinity there must not leak (0 * inf) into pixels whose window does not contain it."""
    N, H, W, Cc, K, R, S, stride, pad = 2, 30, 34, 3, 64, 7, 7, 2, 3
    xi = wl.integer_fp16(503, 0, (N, H, W, Cc), -3, 3)
    wi = wl.integer_fp16(503, 1, (K, R, S, Cc), -2, 2)
    bi = wl.integer_fp16(503, 2, (K,), -4, 4)
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad)
    P, Q = bolt.conv_out_hw(d)
    y = torch.empty((N, P, Q, K), dtype=torch.float16, device="cuda")
    bolt.bolt_conv2d_fprop_nhwc(d, dev(xi), dev(wi), dev(bi), y)
    x8, w8 = torch.empty((N, H, W, 8), dtype=torch.float16, device="cuda"), torch.empty((K, R, S, 8), dtype=torch.float16, device="cuda")
    bolt.bolt_pad_channels_nhwc(dev(xi), x8, 8)
    bolt.bolt_pad_channels_nhwc(dev(wi), w8, 8)
    y8, _ = torch.empty_like(y), None
    bolt.bolt_conv2d_fprop_nhwc(bolt.conv_desc(N, H, W, 8, K, R, S, stride, pad), x8, w8, dev(bi), y8)
    torch.cuda.synchronize()
    assert_bit_equal(host(y), host(y8), "unpadded first layer vs padded path")
    assert_bit_equal(host(y), ref.conv2d_nhwc(xi, wi, bi, stride=stride, pad=pad), "unpadded first layer vs oracle")
    xinf = xi.copy()
    xinf[0, 10, 20, 1] = np.inf
    want = ref.conv2d_nhwc(xinf, np.abs(wi) + 1, bi, stride=stride, pad=pad, act="none")
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad, act="none")
    bolt.bolt_conv2d_fprop_nhwc(d, dev(xinf), dev(np.abs(wi) + 1), dev(bi), y)
    torch.cuda.synchronize()
    got = host(y)
    assert np.isinf(want).any() and not np.isnan(want).any()
    assert_bit_equal(got, want, "infinite input element")


LAST_LAYERS = [
    # N H W C K R S stride pad: P * Q odd and even, ragged M and N tiles, several images inside one tile
    (3, 7, 7, 64, 72, 1, 1, 1, 0),      # 1x1 / stride 1: GEMM addressing; P * Q = 49
    (2, 14, 14, 64, 128, 3, 3, 1, 1),   # gather
    (5, 5, 9, 16, 40, 3, 3, 2, 1),      # stride 2, P * Q = 15: up to 9 images in a 128-row tile
    (1, 20, 20, 8, 8, 5, 5, 1, 2),      # one image, N tile mostly empty
]


@pytest.mark.parametrize("shape", LAST_LAYERS)
def test_last_layer_conv_writes_nchw_every_instance(bolt, shape):
    """Section 3.2.3, layout transformation in the last layer: y_layout = NCHW stores [N][K][P][Q] from the kernel
    itself.  Against the oracle's transformation of the oracle's convolution; bit-exact on integers."""
    N, H, W, Cc, K, R, S, stride, pad = shape
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad, act="relu", y_layout="nchw")
    P, Q = bolt.conv_out_hw(d)
    ids = [k for k in range(bolt.bolt_num_instances(bolt.OP_CONV2D)) if bolt.bolt_instance_supports(bolt.OP_CONV2D, k, d)]
    assert ids
    x = wl.uniform_fp16(601, 0, (N, H, W, Cc), -1, 1)
    w = wl.normal_fp16(601, 1, (K, R, S, Cc), (2.0 / (R * S * Cc)) ** 0.5)
    b = wl.uniform_fp16(601, 2, (K,), -1, 1)
    xi, wi, bi = wl.integer_fp16(602, 0, (N, H, W, Cc), -2, 2), wl.integer_fp16(602, 1, (K, R, S, Cc), -1, 1), wl.integer_fp16(602, 2, (K,), -4, 4)
    want = ref.nhwc_to_nchw(ref.conv2d_nhwc(x, w, b, stride=stride, pad=pad))
    want_i = ref.nhwc_to_nchw(ref.conv2d_nhwc(xi, wi, bi, stride=stride, pad=pad))
    assert want.shape == (N, K, P, Q) and np.abs(want_i.astype(np.float64)).max() < 2048
    for kid in ids:
        _say("last layer %s instance %d" % (shape, kid))
        y = torch.full((N, K, P, Q), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_conv2d_fprop_nhwc(d, dev(x), dev(w), dev(b), y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(y), want, "last layer %s instance %d" % (shape, kid))
        y.fill_(float("nan"))
        bolt.bolt_conv2d_fprop_nhwc(d, dev(xi), dev(wi), dev(bi), y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_bit_equal(host(y), want_i, "integer last layer %s instance %d" % (shape, kid))
    y = torch.full((N, K, P, Q), float("nan"), dtype=torch.float16, device="cuda")
    r = bolt.bolt_tune(bolt.OP_CONV2D, d, None, [dev(x), dev(w), dev(b), y])
    assert r.config.kernel_id in ids
    y.fill_(float("nan"))
    bolt.bolt_conv2d_fprop_nhwc(d, dev(x), dev(w), dev(b), y, r.config)
    torch.cuda.synchronize()
    assert_close(host(y), want, "last layer %s tuned" % (shape,))


@pytest.mark.parametrize("shape", [FIRST_LAYERS[0], FIRST_LAYERS[1], FIRST_LAYERS[2], FIRST_LAYERS[6]])
def test_single_layer_network_nchw_in_nchw_out(bolt, shape):
    """A first layer that is also the last: NCHW in, NCHW out, no transformation or padding pass anywhere."""
    N, H, W, Cc, K, R, S, stride, pad = shape
    d = bolt.conv_desc(N, H, W, Cc, K, R, S, stride, pad, x_layout="nchw", y_layout="nchw")
    P, Q = bolt.conv_out_hw(d)
    xi = wl.integer_fp16(603, 0, (N, Cc, H, W), -3, 3)  # NCHW as given
    wi, bi = wl.integer_fp16(603, 1, (K, R, S, Cc), -2, 2), wl.integer_fp16(603, 2, (K,), -4, 4)
    x = wl.uniform_fp16(604, 0, (N, Cc, H, W), -1, 1)
    w = wl.normal_fp16(604, 1, (K, R, S, Cc), (2.0 / (R * S * Cc)) ** 0.5)
    want_i = ref.nhwc_to_nchw(ref.conv2d_nhwc(ref.nchw_to_nhwc(xi), wi, bi, stride=stride, pad=pad))
    want = ref.nhwc_to_nchw(ref.conv2d_nhwc(ref.nchw_to_nhwc(x), w, bi, stride=stride, pad=pad))
    ids = [k for k in range(bolt.bolt_num_instances(bolt.OP_CONV2D)) if bolt.bolt_instance_supports(bolt.OP_CONV2D, k, d)]
    assert ids
    for kid in ids:
        _say("single layer nchw->nchw %s instance %d" % (shape, kid))
        y = torch.full((N, K, P, Q), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_conv2d_fprop_nhwc(d, dev(xi), dev(wi), dev(bi), y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_bit_equal(host(y), want_i, "integer nchw->nchw %s instance %d" % (shape, kid))
        y.fill_(float("nan"))
        bolt.bolt_conv2d_fprop_nhwc(d, dev(x), dev(w), dev(bi), y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(y), want, "nchw->nchw %s instance %d" % (shape, kid))


# ---------------------------------------------------------------------------------------------
# three-op chains
# ---------------------------------------------------------------------------------------------
GEMM_CHAINS = [  # (M, K0, N0, N1, N2): ragged M, widths at and below the compiled bounds
    (1000, 72, 64, 64, 64), (515, 256, 64, 128, 64), (700, 96, 40, 64, 256), (260, 200, 128, 64, 120),
    (333, 64, 64, 256, 64), (129, 136, 128, 128, 128), (1, 8, 8, 8, 8), (700, 96, 32, 96, 32)]


@pytest.mark.parametrize("layout", ["nk", "kn"])
@pytest.mark.parametrize("shape", GEMM_CHAINS)
def test_gemm_chain3_every_instance(bolt, shape, layout):
    M, K0, N0, N1, N2 = shape
    L = bolt.LAYOUT_NK if layout == "nk" else bolt.LAYOUT_KN
    A = wl.uniform_fp16(301, 0, (M, K0), -0.5, 0.5)
    Ws = [wl.uniform_fp16(301, 1, (K0, N0), -0.5, 0.5), wl.uniform_fp16(301, 2, (N0, N1), -0.5, 0.5),
          wl.uniform_fp16(301, 3, (N1, N2), -0.5, 0.5)]
    bs = [wl.uniform_fp16(301, 4, (N0,), -1, 1), None, wl.uniform_fp16(301, 6, (N2,), -1, 1)]
    acts = ["relu", "gelu", "none"]
    want = ref.gemm_chain(A, Ws, bs, acts)
    descs = [bolt.gemm_desc(M, N0, K0, act=acts[0], b_layout=L), bolt.gemm_desc(M, N1, N0, act=acts[1], b_layout=L),
             bolt.gemm_desc(M, N2, N1, act=acts[2], b_layout=L)]
    Wd = [dev(np.ascontiguousarray(W.T)) if layout == "nk" else dev(W) for W in Ws]
    bd = [dev(b) for b in bs]
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_GEMM_CHAIN3)):
        if not bolt.bolt_chain_instance_supports(bolt.OP_GEMM_CHAIN3, kid, descs):
            continue
        _say("gemm chain %s weights %s instance %d" % (shape, layout, kid))
        D = torch.full((M, N2), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_b2b_gemm_chain(descs, dev(A), Wd, bd, D, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(D), want, "gemm chain %s instance %d" % (shape, kid))
        ran += 1
    assert ran >= 1
    D = torch.full((M, N2), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_b2b_gemm_chain(descs, dev(A), Wd, bd, D)  # built-in pick rule
    torch.cuda.synchronize()
    assert_close(host(D), want, "gemm chain %s heuristic" % (shape,))


CONV_CHAINS = [  # (N, H, W, C, K0, R, S, stride, pad, K1, K2)
    (2, 12, 12, 64, 64, 3, 3, 1, 1, 64, 64), (1, 17, 13, 24, 48, 3, 3, 2, 1, 48, 48), (2, 23, 23, 8, 64, 7, 7, 2, 3, 64, 256),
    (3, 9, 11, 64, 64, 1, 1, 1, 0, 256, 64), (1, 10, 9, 16, 128, 5, 3, (1, 2), (2, 0), 64, 128),
    # stride-1 "same" first filters over whole 64-channel chunks: also the chains whose first op re-uses the halo
    (2, 9, 10, 128, 64, 3, 3, 1, 1, 64, 256), (1, 11, 9, 192, 128, 5, 3, 1, (2, 1), 120, 128), (2, 12, 12, 64, 64, 3, 3, 1, 1, 128, 40),
    (3, 30, 30, 64, 64, 3, 3, 1, 1, 64, 128), (2, 10, 10, 64, 64, 3, 3, 1, 1, 128, 128), (1, 9, 12, 128, 128, 3, 3, 1, 1, 64, 64)]


@pytest.mark.parametrize("shape", CONV_CHAINS)
def test_conv_chain3_every_instance_and_tuner(bolt, shape):
    N, H, W, Cc, K0, R, S, stride, pad, K1, K2 = shape
    x = wl.uniform_fp16(302, 0, (N, H, W, Cc), -1, 1)
    ws = [wl.normal_fp16(302, 1, (K0, R, S, Cc), (2.0 / (R * S * Cc)) ** 0.5), wl.normal_fp16(302, 2, (K1, 1, 1, K0), (2.0 / K0) ** 0.5),
          wl.normal_fp16(302, 3, (K2, 1, 1, K1), (2.0 / K1) ** 0.5)]
    bs = [wl.uniform_fp16(302, 4, (K0,), -1, 1), wl.uniform_fp16(302, 5, (K1,), -1, 1), wl.uniform_fp16(302, 6, (K2,), -1, 1)]
    acts = ["relu", "relu", "hardswish"]
    want = ref.conv_chain(x, ws, bs, acts, stride=stride, pad=pad)
    d0 = bolt.conv_desc(N, H, W, Cc, K0, R, S, stride, pad, act=acts[0])
    P, Q = bolt.conv_out_hw(d0)
    descs = [d0, bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0, act=acts[1]), bolt.conv_desc(N, P, Q, K1, K2, 1, 1, 1, 0, act=acts[2])]
    wd, bd = [dev(w) for w in ws], [dev(b) for b in bs]
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_CONV_CHAIN3)):
        if not bolt.bolt_chain_instance_supports(bolt.OP_CONV_CHAIN3, kid, descs):
            continue
        _say("conv chain %s instance %d" % (shape, kid))
        y = torch.full((N, P, Q, K2), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_b2b_conv_chain(descs, dev(x), wd, bd, y, {"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(y), want, "conv chain %s instance %d" % (shape, kid))
        ran += 1
    assert ran >= 1
    y = torch.full((N, P, Q, K2), float("nan"), dtype=torch.float16, device="cuda")
    res = bolt.bolt_tune_chain(bolt.OP_CONV_CHAIN3, descs, [dev(x), wd[0], bd[0], wd[1], bd[1], wd[2], bd[2], y])
    assert res.tried == ran and res.ms > 0
    y.fill_(float("nan"))
    bolt.bolt_b2b_conv_chain(descs, dev(x), wd, bd, y, res.config)
    torch.cuda.synchronize()
    assert_close(host(y), want, "conv chain %s tuned" % (shape,))


def test_gemm_chain3_integer_bit_exact(bolt):
    M, K0, N0, N1, N2 = 300, 72, 64, 64, 128
    A = wl.integer_fp16(303, 0, (M, K0), -2, 2)
    Ws = [wl.integer_fp16(303, 1, (K0, N0), -1, 1), wl.integer_fp16(303, 2, (N0, N1), -1, 1), wl.integer_fp16(303, 3, (N1, N2), -1, 1)]
    # keep intermediates small: sparse weights so that |D_i| stays exactly representable
    for W in Ws:
        W[np.arange(W.shape[0])[:, None] % 4 != np.arange(W.shape[1])[None, :] % 4] = 0
    bs = [wl.integer_fp16(303, 4, (N0,), -2, 2), wl.integer_fp16(303, 5, (N1,), -2, 2), wl.integer_fp16(303, 6, (N2,), -2, 2)]
    want = ref.gemm_chain(A, Ws, bs, ["relu", "relu", "relu"])
    assert np.abs(want.astype(np.float64)).max() < 2048
    descs = [bolt.gemm_desc(M, N0, K0, b_layout=bolt.LAYOUT_NK), bolt.gemm_desc(M, N1, N0, b_layout=bolt.LAYOUT_NK),
             bolt.gemm_desc(M, N2, N1, b_layout=bolt.LAYOUT_NK)]
    D = torch.empty((M, N2), dtype=torch.float16, device="cuda")
    bolt.bolt_b2b_gemm_chain(descs, dev(A), [dev(np.ascontiguousarray(W.T)) for W in Ws], [dev(b) for b in bs], D)
    torch.cuda.synchronize()
    assert_bit_equal(host(D), want, "integer gemm chain")


@pytest.mark.parametrize("layout", ["nk", "kn"])
@pytest.mark.parametrize("shape", [GEMM_CHAINS[0], GEMM_CHAINS[2], GEMM_CHAINS[3], GEMM_CHAINS[6]])
def test_gemm_chain3_residual_every_instance(bolt, shape, layout):
    """Eq. 1 with a full matrix C in the last epilogue of a chain: strided C (ldc > N2), gamma != 1, every instance."""
    M, K0, N0, N1, N2 = shape
    L = bolt.LAYOUT_NK if layout == "nk" else bolt.LAYOUT_KN
    A = wl.uniform_fp16(311, 0, (M, K0), -0.5, 0.5)
    Ws = [wl.uniform_fp16(311, 1, (K0, N0), -0.5, 0.5), wl.uniform_fp16(311, 2, (N0, N1), -0.5, 0.5),
          wl.uniform_fp16(311, 3, (N1, N2), -0.5, 0.5)]
    bs = [wl.uniform_fp16(311, 4, (N0,), -1, 1), None, wl.uniform_fp16(311, 6, (N2,), -1, 1)]
    ldc = N2 + 16
    Cfull = wl.uniform_fp16(311, 7, (M, ldc), -3, 3)
    acts = ["relu", "gelu", "relu"]
    want = ref.gemm_chain_residual(A, Ws, bs, acts, np.ascontiguousarray(Cfull[:, :N2]), gamma=-0.75)
    assert not np.array_equal(want, ref.gemm_chain(A, Ws, bs, acts))
    descs = [bolt.gemm_desc(M, N0, K0, act=acts[0], b_layout=L), bolt.gemm_desc(M, N1, N0, act=acts[1], b_layout=L),
             bolt.gemm_desc(M, N2, N1, act=acts[2], b_layout=L)]
    Wd = [dev(np.ascontiguousarray(W.T)) if layout == "nk" else dev(W) for W in Ws]
    bd = [dev(b) for b in bs]
    Cd = dev(Cfull)
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_GEMM_CHAIN3)):
        if not bolt.bolt_chain_instance_supports(bolt.OP_GEMM_CHAIN3, kid, descs):
            continue
        _say("gemm chain residual %s instance %d" % (shape, kid))
        D = torch.full((M, N2), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_b2b_gemm_chain_residual(descs, dev(A), Wd, bd, Cd, D, gamma=-0.75, ldc=ldc, config={"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(D), want, "gemm chain residual %s instance %d" % (shape, kid))
        ran += 1
    assert ran >= 1
    # the residual may be the output buffer (each element is read before it is written, by the same workgroup)
    D = dev(np.ascontiguousarray(Cfull[:, :N2]))
    bolt.bolt_b2b_gemm_chain_residual(descs, dev(A), Wd, bd, D, D, gamma=-0.75)
    torch.cuda.synchronize()
    assert_close(host(D), want, "gemm chain residual %s in place" % (shape,))
    # argument errors: a missing C, a row stride below N2, a misaligned one
    D2 = torch.empty((M, N2), dtype=torch.float16, device="cuda")
    for kwargs, C_arg in [(dict(ldc=N2 - 8), Cd), (dict(ldc=N2 + 4), Cd), (dict(), None)]:
        with pytest.raises(bolt.BoltError):
            bolt.bolt_b2b_gemm_chain_residual(descs, dev(A), Wd, bd, C_arg, D2, gamma=1.0, **kwargs)


@pytest.mark.parametrize("shape", [CONV_CHAINS[0], CONV_CHAINS[1], CONV_CHAINS[3], CONV_CHAINS[5], CONV_CHAINS[6]])
def test_conv_chain3_residual_every_instance(bolt, shape):
    N, H, W, Cc, K0, R, S, stride, pad, K1, K2 = shape
    x = wl.uniform_fp16(312, 0, (N, H, W, Cc), -1, 1)
    ws = [wl.normal_fp16(312, 1, (K0, R, S, Cc), (2.0 / (R * S * Cc)) ** 0.5), wl.normal_fp16(312, 2, (K1, 1, 1, K0), (2.0 / K0) ** 0.5),
          wl.normal_fp16(312, 3, (K2, 1, 1, K1), (2.0 / K1) ** 0.5)]
    bs = [wl.uniform_fp16(312, 4, (K0,), -1, 1), wl.uniform_fp16(312, 5, (K1,), -1, 1), None]
    acts = ["relu", "relu", "relu"]
    d0 = bolt.conv_desc(N, H, W, Cc, K0, R, S, stride, pad, act=acts[0])
    P, Q = bolt.conv_out_hw(d0)
    res = wl.uniform_fp16(312, 7, (N, P, Q, K2), -2, 2)
    want = ref.conv_chain_residual(x, ws, bs, acts, res, stride=stride, pad=pad, gamma=1.0)
    assert not np.array_equal(want, ref.conv_chain(x, ws, bs, acts, stride=stride, pad=pad))
    descs = [d0, bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0, act=acts[1]), bolt.conv_desc(N, P, Q, K1, K2, 1, 1, 1, 0, act=acts[2])]
    wd, bd = [dev(w) for w in ws], [dev(b) for b in bs]
    ran = 0
    for kid in range(bolt.bolt_num_instances(bolt.OP_CONV_CHAIN3)):
        if not bolt.bolt_chain_instance_supports(bolt.OP_CONV_CHAIN3, kid, descs):
            continue
        _say("conv chain residual %s instance %d" % (shape, kid))
        y = torch.full((N, P, Q, K2), float("nan"), dtype=torch.float16, device="cuda")
        bolt.bolt_b2b_conv_chain_residual(descs, dev(x), wd, bd, dev(res), y, gamma=1.0, config={"kernel_id": kid})
        torch.cuda.synchronize()
        assert_close(host(y), want, "conv chain residual %s instance %d" % (shape, kid))
        ran += 1
    assert ran >= 1


def test_gemm_chain3_residual_integer_bit_exact(bolt):
    M, K0, N0, N1, N2 = 300, 72, 64, 64, 120
    A = wl.integer_fp16(313, 0, (M, K0), -2, 2)
    Ws = [wl.integer_fp16(313, 1, (K0, N0), -1, 1), wl.integer_fp16(313, 2, (N0, N1), -1, 1), wl.integer_fp16(313, 3, (N1, N2), -1, 1)]
    for W in Ws:
        W[np.arange(W.shape[0])[:, None] % 4 != np.arange(W.shape[1])[None, :] % 4] = 0
    bs = [wl.integer_fp16(313, 4, (N0,), -2, 2), wl.integer_fp16(313, 5, (N1,), -2, 2), wl.integer_fp16(313, 6, (N2,), -2, 2)]
    Cm = wl.integer_fp16(313, 7, (M, N2), -50, 50)
    want = ref.gemm_chain_residual(A, Ws, bs, ["relu", "relu", "relu"], Cm, gamma=2.0)
    assert np.abs(want.astype(np.float64)).max() < 2048
    descs = [bolt.gemm_desc(M, N0, K0, b_layout=bolt.LAYOUT_NK), bolt.gemm_desc(M, N1, N0, b_layout=bolt.LAYOUT_NK),
             bolt.gemm_desc(M, N2, N1, b_layout=bolt.LAYOUT_NK)]
    Wd, bd = [dev(np.ascontiguousarray(W.T)) for W in Ws], [dev(b) for b in bs]
    for kid in range(bolt.bolt_num_instances(bolt.OP_GEMM_CHAIN3)):
        if not bolt.bolt_chain_instance_supports(bolt.OP_GEMM_CHAIN3, kid, descs):
            continue
        _say("integer gemm chain residual instance %d" % kid)
        D = torch.empty((M, N2), dtype=torch.float16, device="cuda")
        bolt.bolt_b2b_gemm_chain_residual(descs, dev(A), Wd, bd, dev(Cm), D, gamma=2.0, config={"kernel_id": kid})
        torch.cuda.synchronize()
        assert_bit_equal(host(D), want, "integer gemm chain residual instance %d" % kid)


@pytest.mark.parametrize("act", ["none", "relu", "gelu", "hardswish", "softplus"])
def test_bias_act_standalone_epilogue(bolt, act):
    # several grid strides plus a ragged last block; with and without a bias; also M = 1 and M = 0
    for (M, N, seed) in [(1030, 136, 61), (1, 8, 62), (4099, 3072, 63)]:
        _say(f"bias_act act={act} M={M} N={N}")
        x = wl.uniform_fp16(seed, 0, (M, N), -6, 6)
        b = wl.uniform_fp16(seed, 1, (N,), -2, 2)
        for bias, alpha, beta in [(b, 0.75, -1.5), (None, 1.0, 1.0)]:
            D = dev(x).clone()
            bolt.bolt_bias_act(D, dev(bias), alpha, beta, act)
            torch.cuda.synchronize()
            assert_close(host(D), ref.bias_act(x, bias, alpha, beta, act), f"bias_act {act} {M}x{N}")
    empty = torch.empty((0, 16), dtype=torch.float16, device="cuda")
    bolt.bolt_bias_act(empty, None, 1.0, 1.0, act)


def test_unfused_gemm_plus_bias_act_matches_fused_on_integers(bolt):
    A = wl.integer_fp16(64, 0, (300, 72), -3, 3)
    B = wl.integer_fp16(64, 1, (72, 136), -3, 3)
    bias = wl.integer_fp16(64, 2, (136,), -4, 4)
    fused, _ = _run_gemm(bolt, A, B, bias, act="relu")
    d = bolt.gemm_desc(300, 136, 72, act="none")
    D = torch.empty((300, 136), dtype=torch.float16, device="cuda")
    bolt.bolt_gemm_epilogue(d, dev(A), dev(B), None, D)
    bolt.bolt_bias_act(D, dev(bias), 1.0, 1.0, "relu")
    torch.cuda.synchronize()
    assert_bit_equal(host(D), fused, "unfused vs fused")
    assert_bit_equal(fused, ref.gemm(A, B, bias), "fused vs oracle")


def test_calls_are_capturable_in_a_hip_graph_and_replays_repeat_the_eager_result(bolt):
    """The entry points only enqueue kernels on the given stream (no allocation, no synchronisation, no memset), so a
    caller can capture them; every replay must reproduce the eager outputs bit for bit."""
    x = wl.uniform_fp16(901, 0, (2, 14, 14, 64), -1, 1)
    w = wl.normal_fp16(901, 1, (64, 3, 3, 64), (2.0 / 576) ** 0.5)
    b = wl.uniform_fp16(901, 2, (64,), -1, 1)
    res = wl.uniform_fp16(901, 3, (2, 14, 14, 64), -2, 2)
    w1 = wl.normal_fp16(901, 4, (64, 1, 1, 64), (2.0 / 64) ** 0.5)
    b1 = wl.uniform_fp16(901, 5, (64,), -1, 1)
    x3 = wl.uniform_fp16(901, 6, (2, 14, 14, 6), -1, 1)
    d = bolt.conv_desc(2, 14, 14, 64, 64, 3, 3, 1, 1)
    d1 = bolt.conv_desc(2, 14, 14, 64, 64, 1, 1, 1, 0)
    xd, wd, bd, rd, w1d, b1d, x3d = (dev(a) for a in (x, w, b, res, w1, b1, x3))
    ws = torch.empty(max(bolt.bolt_workspace_bytes(bolt.OP_CONV2D, d), 16), dtype=torch.uint8, device="cuda")
    sk = next(k for k in range(bolt.bolt_num_instances(bolt.OP_CONV2D))
              if bolt.bolt_check(bolt.OP_CONV2D, d, None, {"kernel_id": k, "split_k": 2}) == 0)
    outs = dict(y_split=torch.empty((2, 14, 14, 64), dtype=torch.float16, device="cuda"),
                y_res=torch.empty((2, 14, 14, 64), dtype=torch.float16, device="cuda"),
                y_pair=torch.empty((2, 14, 14, 64), dtype=torch.float16, device="cuda"),
                x8=torch.empty((2, 14, 14, 8), dtype=torch.float16, device="cuda"))

    def enqueue():
        bolt.bolt_conv2d_fprop_nhwc(d, xd, wd, bd, outs["y_split"], {"kernel_id": sk, "split_k": 2}, ws)   # two kernels + workspace
        bolt.bolt_conv2d_fprop_nhwc_residual(d, xd, wd, bd, rd, outs["y_res"])
        bolt.bolt_b2b_conv(d, d1, xd, wd, bd, w1d, b1d, outs["y_pair"])
        bolt.bolt_pad_channels_nhwc(x3d, outs["x8"], 8)

    enqueue()  # eager: the expected values (and every kernel's one-time attribute call happens outside the capture)
    torch.cuda.synchronize()
    eager = {k: host(v).copy() for k, v in outs.items()}
    assert_close(eager["y_split"], ref.conv2d_nhwc(x, w, b, stride=1, pad=1), "eager split-K conv")
    assert_close(eager["y_res"], ref.conv2d_nhwc_residual(x, w, b, res, stride=1, pad=1), "eager residual conv")
    assert_close(eager["y_pair"], ref.b2b_conv(x, w, b, w1, b1, stride=1, pad=1), "eager fused pair")
    assert_bit_equal(eager["x8"], ref.pad_channels(x3, 8), "eager padding")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    for rep in range(3):
        for v in outs.values():
            v.fill_(float("nan"))
        ws.fill_(0xFF)                      # stale workspace contents must not matter
        torch.cuda.synchronize()
        _say("graph replay %d" % rep)
        graph.replay()
        torch.cuda.synchronize()
        for k, v in outs.items():
            assert_bit_equal(host(v), eager[k], "graph replay %d, %s" % (rep, k))
        enqueue()                           # eager work between replays
        torch.cuda.synchronize()


def test_tune_is_cached_and_probes_run(bolt):
    M, N, K = 512, 256, 256
    A, B = dev(wl.uniform_fp16(601, 0, (M, K), -1, 1)), dev(wl.uniform_fp16(601, 1, (K, N), -1, 1))
    D = torch.empty((M, N), dtype=torch.float16, device="cuda")
    d = bolt.gemm_desc(M, N, K)
    r1 = bolt.bolt_tune(bolt.OP_GEMM, d, None, [A, B, None, D])
    r2 = bolt.bolt_tune(bolt.OP_GEMM, d, None, [A, B, None, D])
    assert r1.config.as_dict() == r2.config.as_dict() and r1.ms == r2.ms
    peak = bolt.bolt_probe_mfma_peak(2000)
    buf = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    bw = bolt.bolt_probe_copy_bandwidth(buf, 3)
    _say("MFMA loop %.0f TFLOP/s, copy %.0f GB/s" % (peak, bw))
    assert peak > 100 and bw > 500
