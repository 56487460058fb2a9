"""The entry point that allocates nothing: bolt_gemm_epilogue_noalloc against bolt_gemm_epilogue.

Both run the same kernels; the only difference is where the split-K partial sums live (the library's fixed device
array instead of a caller's workspace), so the outputs must be bit-identical.  Two calls in a row share the array;
the second is smaller, so stale partial sums of the first lie behind its own.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import ref
from util import assert_bit_equal, assert_close, dev, host

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bolt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2110_15238_amd as b
    return b


def _pair(bolt, seed, M, N, K, config):
    A = wl.uniform_fp16(seed, 0, (M, K), -1, 1)
    B = wl.uniform_fp16(seed, 1, (K, N), -1, 1)
    bias = wl.uniform_fp16(seed, 2, (N,), -1, 1)
    d = bolt.gemm_desc(M, N, K, act="relu")
    Ad, Bd, bd = dev(A), dev(B), dev(bias)
    ws = torch.empty(8 * M * N, dtype=torch.float32, device="cuda")
    want = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    got = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    bolt.bolt_gemm_epilogue(d, Ad, Bd, bd, want, config, ws)
    bolt.bolt_gemm_epilogue_noalloc(d, Ad, Bd, bd, got, config)
    torch.cuda.synchronize()
    return host(got), host(want), ref.gemm(A, B, bias)


def test_noalloc_matches_the_workspace_entry_point_on_two_calls_in_a_row(bolt):
    d = bolt.gemm_desc(384, 256, 1024)
    kid = [k for k in range(bolt.bolt_num_instances(bolt.OP_GEMM)) if bolt.bolt_instance_supports(bolt.OP_GEMM, k, d)][0]
    # first call: 4 x 384 x 256 partial sums (1.5 MiB of the array)
    got, want, oracle = _pair(bolt, 901, 384, 256, 1024, {"kernel_id": kid, "split_k": 4})
    assert_bit_equal(got, want, "noalloc vs workspace, first call")
    assert_close(got, oracle, "noalloc vs oracle, first call")
    # second call, smaller (ragged in M and N): 2 x 200 x 136 partial sums over the leftovers of the first
    got, want, oracle = _pair(bolt, 902, 200, 136, 512, {"kernel_id": kid, "split_k": 2})
    assert_bit_equal(got, want, "noalloc vs workspace, second call")
    assert_close(got, oracle, "noalloc vs oracle, second call")
    # no split-K: the array is not touched at all
    got, want, oracle = _pair(bolt, 903, 96, 72, 64, None)
    assert_bit_equal(got, want, "noalloc vs workspace, no split")
    assert_close(got, oracle, "noalloc vs oracle, no split")


def test_noalloc_rejects_partial_sums_beyond_the_fixed_array(bolt):
    # 8 x 2048 x 512 x 4 bytes = 32 MiB > 16 MiB: refused before any launch, output untouched
    M, N, K = 2048, 512, 1024
    d = bolt.gemm_desc(M, N, K)
    kid = [k for k in range(bolt.bolt_num_instances(bolt.OP_GEMM)) if bolt.bolt_instance_supports(bolt.OP_GEMM, k, d)][0]
    A = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    B = torch.zeros((K, N), dtype=torch.float16, device="cuda")
    D = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
    with pytest.raises(bolt.BoltError) as e:
        bolt.bolt_gemm_epilogue_noalloc(d, A, B, None, D, {"kernel_id": kid, "split_k": 8})
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert bool((D == 7.0).all())
