"""w4a4_linear_f16act (quantize_act + GEMM + epilogue in one kernel, for small token counts)
against the oracle and against the two-call path, which it must equal bit for bit."""
import numpy as np
import pytest
import torch

from tests.gpu_util import GELU_SAME, OLAY_SAME, assert_f16, dev, f16_close, has_gpu, host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]

SYM = 0


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


def _case(rng, M, N, K, bias=True):
    X = rng.standard_normal((M, K)).astype(np.float32).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    b = (rng.standard_normal(N) * 0.01).astype(np.float16) if bias else None
    return X, W, b


@pytest.mark.parametrize("M,N,K", [(128, 768, 768), (128, 2304, 768), (128, 3072, 768), (128, 768, 3072),
                                   (1, 8, 64), (33, 40, 128), (150, 264, 192), (31, 32, 4096), (257, 96, 320), (40, 2200, 832),
                                   (64, 1024, 1536), (96, 4096, 1024)])
@pytest.mark.parametrize("act", [0, 1])
def test_fused_equals_two_calls_and_oracle(B, orc, M, N, K, act):
    rng = np.random.default_rng(M * 7 + N + K + act)
    X, W, b = _case(rng, M, N, K)
    X[0, :] = 0                                                     # a constant row: scale 1, codes 0
    if M > 2:
        X[2, 5] = 60000.0                                           # one huge element: the rest of the row rounds to 0
    Q = B.quantize_weight(dev(W), SYM)
    got = host(B.linear_f16act(dev(X), Q, dev(b), act))
    A = B.quantize_act(dev(X), SYM)
    two = host(B.linear(A, Q, dev(b), act))
    assert np.array_equal(got.view(np.uint16), two.view(np.uint16))
    oa, ow = orc.quantize_act(X, SYM), orc.quantize_weight(W, SYM)
    want = orc.linear(oa, ow, SYM, 0, b, act)["out"]
    ok, ratio = f16_close(got, want)
    assert ok, ratio
    assert_f16(got, want, 1.0 if act == 0 else GELU_SAME if got.size > 200 else 0.7, f"act {act}")


def test_fused_strided_input_no_bias(B, orc):
    """X is a column slice of a wider matrix (row stride > K) and there is no bias."""
    rng = np.random.default_rng(77)
    M, N, K = 70, 136, 256
    wide = rng.standard_normal((M, 3 * K)).astype(np.float32).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    Xd = dev(wide)[:, K:2 * K]
    assert Xd.stride(0) == 3 * K
    Q = B.quantize_weight(dev(W), SYM)
    got = host(B.linear_f16act(Xd, Q, None, 0))
    X = np.ascontiguousarray(wide[:, K:2 * K])
    want = orc.linear(orc.quantize_act(X, SYM), orc.quantize_weight(W, SYM), SYM, 0, None, 0)["out"]
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_fused_does_not_write_past_the_output(B):
    rng = np.random.default_rng(78)
    M, N, K = 37, 72, 128
    X, W, b = _case(rng, M, N, K)
    Q = B.quantize_weight(dev(W), SYM)
    buf = torch.full((M + 40, N), -7.0, dtype=torch.float16, device="cuda")
    B.linear_f16act(dev(X), Q, dev(b), 0, out=buf[:M])
    assert bool((buf[M:] == -7.0).all())
    assert bool((buf[:M] != -7.0).any())


def test_fused_non_finite_inputs_do_not_fault(B):
    rng = np.random.default_rng(79)
    X, W, b = _case(rng, 64, 64, 128)
    X[3, 7] = np.inf
    X[5, 9] = np.nan
    Q = B.quantize_weight(dev(W), SYM)
    got = host(B.linear_f16act(dev(X), Q, dev(b), 1))
    rows = np.ones(64, bool)
    rows[[3, 5]] = False
    assert np.isfinite(got[rows]).all()                             # the other tokens are unaffected
