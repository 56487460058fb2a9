"""GPU parity on seeded random shapes, through the paths a caller who names no kernel takes: the built-in pick rule
and the tuner's winner, for single ops, fused pairs and chains of three.  The per-instance tests elsewhere fix the
shapes and sweep the kernels; this file fixes nothing but the seed, so ragged extents, filter shapes, strides and
channel counts meet whatever instance the library chooses for them."""
import numpy as np
import pytest

import workloads as wl
from oracle import ref
from util import assert_close, dev, host

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

ACTS = ["none", "relu", "gelu", "hardswish", "softplus"]


@pytest.fixture(scope="module")
def bolt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2110_15238_amd as b
    return b


def _say(msg):
    print(msg, flush=True)


def _nan(*shape):
    return torch.full(shape, float("nan"), dtype=torch.float16, device="cuda")


def _conv_case(rng):
    R, S = int(rng.choice([1, 3, 3, 5])), int(rng.choice([1, 3, 3, 7]))
    if rng.random() < 0.5:
        S = R
    stride = int(rng.choice([1, 1, 2]))
    pad = (R // 2, S // 2) if rng.random() < 0.7 else (0, 0)
    H, W = int(rng.integers(max(R, 5), 22)), int(rng.integers(max(S, 5), 22))
    C = int(rng.choice([8, 16, 24, 48, 64, 64, 128, 136, 192, 256]))
    K = int(rng.choice([8, 16, 40, 48, 64, 64, 128, 200, 256, 264, 512]))
    return int(rng.integers(1, 4)), H, W, C, K, R, S, stride, pad


@pytest.mark.parametrize("seed", range(24))
def test_random_conv_built_in_pick_and_tuned(bolt, seed):
    rng = np.random.default_rng(9000 + seed)
    N, H, W, C, K, R, S, stride, pad = _conv_case(rng)
    act = ACTS[seed % len(ACTS)]
    alpha, beta = (1.0, 1.0) if seed % 3 else (0.5, 2.0)
    x = wl.uniform_fp16(900 + seed, 0, (N, H, W, C), -1, 1)
    w = wl.normal_fp16(900 + seed, 1, (K, R, S, C), (2.0 / (R * S * C)) ** 0.5)
    b = wl.uniform_fp16(900 + seed, 2, (K,), -1, 1) if seed % 4 else None
    want = ref.conv2d_nhwc(x, w, b, stride=stride, pad=pad, alpha=alpha, beta=beta, act=act)
    d = bolt.conv_desc(N, H, W, C, K, R, S, stride, pad, alpha=alpha, beta=beta, act=act)
    P, Q = bolt.conv_out_hw(d)
    _say("random conv %s act %s" % ((N, H, W, C, K, R, S, stride, pad), act))
    xd, wd, bd = dev(x), dev(w), dev(b)
    y = _nan(N, P, Q, K)
    bolt.bolt_conv2d_fprop_nhwc(d, xd, wd, bd, y, None)
    torch.cuda.synchronize()
    assert_close(host(y), want, "random conv %d, built-in pick" % seed)
    ws = torch.empty(8 * N * P * Q * K * 4, dtype=torch.uint8, device="cuda")
    res = bolt.bolt_tune(bolt.OP_CONV2D, d, None, [xd, wd, bd, y], workspace=ws)
    _say("  tuned %s" % (res.config.as_dict(),))
    y.fill_(float("nan"))
    bolt.bolt_conv2d_fprop_nhwc(d, xd, wd, bd, y, res.config, ws)
    torch.cuda.synchronize()
    assert_close(host(y), want, "random conv %d, tuned %s" % (seed, res.config.as_dict()))


@pytest.mark.parametrize("seed", range(12))
def test_random_gemm_both_layouts_built_in_pick_and_tuned(bolt, seed):
    rng = np.random.default_rng(9100 + seed)
    M = int(rng.integers(1, 700))
    N, K = 8 * int(rng.integers(1, 48)), 8 * int(rng.integers(1, 60))
    act = ACTS[(seed + 1) % len(ACTS)]
    A = wl.uniform_fp16(910 + seed, 0, (M, K), -1, 1)
    B = wl.normal_fp16(910 + seed, 1, (K, N), (2.0 / K) ** 0.5)
    bias = wl.uniform_fp16(910 + seed, 2, (N,), -1, 1)
    want = ref.gemm(A, B, bias, act=act)
    for layout, Bd in ((bolt.LAYOUT_KN, dev(B)), (bolt.LAYOUT_NK, dev(np.ascontiguousarray(B.T)))):
        d = bolt.gemm_desc(M, N, K, act=act, b_layout=layout)
        _say("random gemm %s layout %d act %s" % ((M, N, K), layout, act))
        D = _nan(M, N)
        Ad, bd = dev(A), dev(bias)
        bolt.bolt_gemm_epilogue(d, Ad, Bd, bd, D, None)
        torch.cuda.synchronize()
        assert_close(host(D), want, "random gemm %d layout %d, built-in pick" % (seed, layout))
        res = bolt.bolt_tune(bolt.OP_GEMM, d, None, [Ad, Bd, bd, D])
        D.fill_(float("nan"))
        bolt.bolt_gemm_epilogue(d, Ad, Bd, bd, D, res.config)
        torch.cuda.synchronize()
        assert_close(host(D), want, "random gemm %d layout %d, tuned %s" % (seed, layout, res.config.as_dict()))


@pytest.mark.parametrize("seed", range(16))
def test_random_fused_conv_pair_built_in_pick_and_tuned(bolt, seed):
    rng = np.random.default_rng(9200 + seed)
    N, H, W = int(rng.integers(1, 4)), int(rng.integers(6, 20)), int(rng.integers(6, 20))
    C = int(rng.choice([8, 24, 48, 64, 64, 128]))
    K0 = int(rng.choice([16, 32, 48, 64, 64, 128]))
    K1 = int(rng.choice([16, 48, 64, 128, 136, 200, 256]))
    if K0 > 64:
        K1 = min(K1, 128)  # the compiled widths: N0 <= 64 with N1 <= 256, or both <= 128
    stride = int(rng.choice([1, 1, 2]))
    with_res = bool(seed % 2)
    x = wl.uniform_fp16(920 + seed, 0, (N, H, W, C), -1, 1)
    w0 = wl.normal_fp16(920 + seed, 1, (K0, 3, 3, C), (2.0 / (9 * C)) ** 0.5)
    b0 = wl.uniform_fp16(920 + seed, 2, (K0,), -1, 1)
    w1 = wl.normal_fp16(920 + seed, 3, (K1, 1, 1, K0), (2.0 / K0) ** 0.5)
    b1 = wl.uniform_fp16(920 + seed, 4, (K1,), -1, 1)
    c0 = bolt.conv_desc(N, H, W, C, K0, 3, 3, stride, 1)
    P, Q = bolt.conv_out_hw(c0)
    c1 = bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0)
    assert bolt.bolt_check(bolt.OP_B2B_CONV_RES if with_res else bolt.OP_B2B_CONV, c0, c1) == 0
    _say("random fused pair %s residual %s" % ((N, H, W, C, K0, stride, K1), with_res))
    xd, w0d, b0d, w1d, b1d = dev(x), dev(w0), dev(b0), dev(w1), dev(b1)
    y = _nan(N, P, Q, K1)
    if with_res:
        r = wl.uniform_fp16(920 + seed, 5, (N, P, Q, K1), -2, 2)
        want = ref.b2b_conv_residual(x, w0, b0, w1, b1, r, stride=stride, pad=1, gamma=1.0)
        rd = dev(r)
        run = lambda cfg: bolt.bolt_b2b_conv_residual(c0, c1, xd, w0d, b0d, w1d, b1d, rd, y, 1.0, cfg)
        op, ptrs = bolt.OP_B2B_CONV_RES, [xd, w0d, b0d, w1d, b1d, y, rd]
    else:
        want = ref.b2b_conv(x, w0, b0, w1, b1, stride=stride, pad=1)
        run = lambda cfg: bolt.bolt_b2b_conv(c0, c1, xd, w0d, b0d, w1d, b1d, y, cfg)
        op, ptrs = bolt.OP_B2B_CONV, [xd, w0d, b0d, w1d, b1d, y]
    run(None)
    torch.cuda.synchronize()
    assert_close(host(y), want, "random fused pair %d, built-in pick" % seed)
    res = bolt.bolt_tune(op, c0, c1, ptrs)
    _say("  tuned %s" % (res.config.as_dict(),))
    y.fill_(float("nan"))
    run(res.config)
    torch.cuda.synchronize()
    assert_close(host(y), want, "random fused pair %d, tuned %s" % (seed, res.config.as_dict()))


@pytest.mark.parametrize("seed", range(10))
def test_random_conv_chain_built_in_pick_and_tuned(bolt, seed):
    rng = np.random.default_rng(9300 + seed)
    N, H, W = int(rng.integers(1, 3)), int(rng.integers(6, 18)), int(rng.integers(6, 18))
    C = int(rng.choice([8, 48, 64, 64, 128]))
    K0, K1 = int(rng.choice([32, 64, 64, 128])), int(rng.choice([40, 64, 64, 128]))
    K2 = int(rng.choice([48, 64, 120, 128, 256])) if max(K0, K1) <= 64 else int(rng.choice([48, 64, 128]))
    stride = int(rng.choice([1, 1, 2]))
    acts = [ACTS[(seed + i) % len(ACTS)] for i in range(3)]
    x = wl.uniform_fp16(930 + seed, 0, (N, H, W, C), -1, 1)
    ws = [wl.normal_fp16(930 + seed, 1, (K0, 3, 3, C), (2.0 / (9 * C)) ** 0.5), wl.normal_fp16(930 + seed, 2, (K1, 1, 1, K0), (2.0 / K0) ** 0.5),
          wl.normal_fp16(930 + seed, 3, (K2, 1, 1, K1), (2.0 / K1) ** 0.5)]
    bs = [wl.uniform_fp16(930 + seed, 4 + i, (k,), -1, 1) for i, k in enumerate((K0, K1, K2))]
    want = ref.conv_chain(x, ws, bs, acts, stride=stride, pad=1)
    d0 = bolt.conv_desc(N, H, W, C, K0, 3, 3, stride, 1, act=acts[0])
    P, Q = bolt.conv_out_hw(d0)
    descs = [d0, bolt.conv_desc(N, P, Q, K0, K1, 1, 1, 1, 0, act=acts[1]), bolt.conv_desc(N, P, Q, K1, K2, 1, 1, 1, 0, act=acts[2])]
    if bolt.bolt_check_chain(bolt.OP_CONV_CHAIN3, descs) != 0:
        pytest.skip("no chain instance spans these widths: %s" % ((K0, K1, K2),))
    _say("random conv chain %s acts %s" % ((N, H, W, C, K0, K1, K2, stride), acts))
    xd, wd, bd = dev(x), [dev(w) for w in ws], [dev(b) for b in bs]
    y = _nan(N, P, Q, K2)
    bolt.bolt_b2b_conv_chain(descs, xd, wd, bd, y, None)
    torch.cuda.synchronize()
    assert_close(host(y), want, "random conv chain %d, built-in pick" % seed)
    res = bolt.bolt_tune_chain(bolt.OP_CONV_CHAIN3, descs, [xd, wd[0], bd[0], wd[1], bd[1], wd[2], bd[2], y])
    y.fill_(float("nan"))
    bolt.bolt_b2b_conv_chain(descs, xd, wd, bd, y, res.config)
    torch.cuda.synchronize()
    assert_close(host(y), want, "random conv chain %d, tuned %s" % (seed, res.config.as_dict()))
