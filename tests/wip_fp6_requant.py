"""GPU parity of the fused requantize of the FP6 path (work in progress: run by naming this file)."""
import numpy as np
import pytest
import torch

from tests.gpu_util import dev, fp6_to_codes, has_gpu, host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]
SYM, FP6 = 0, 2


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def orc():
    import oracle
    return oracle


def _x(rng, M, K):
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 4, replace=False)] *= 20.0
    return x.astype(np.float16)


def _codes(want_q, N):
    """canonical packed nibbles (two's complement, low nibble first) -> int8 codes"""
    lo = (want_q & 15).astype(np.int8)
    hi = (want_q >> 4).astype(np.int8)
    c = np.empty(want_q.shape[:-1] + (N,), np.int8)
    c[..., 0::2] = np.where(lo > 7, lo - 16, lo)
    c[..., 1::2] = np.where(hi > 7, hi - 16, hi)
    return c


@pytest.mark.parametrize("M,N,K,bias", [(128, 256, 512, False), (200, 512, 768, True), (1000, 1024, 1024, True), (77, 768, 512, True),
                                        (2500, 3072, 1024, True)])
def test_fused_requantize_fp6(B, orc, M, N, K, bias):
    rng = np.random.default_rng(M + N + K)
    X, W = _x(rng, M, K), (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    print("case", M, N, K, bias, flush=True)
    A, Q = B.quantize_act(dev(X), SYM, layout=FP6), B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    a, w = orc.quantize_act(X, SYM), orc.quantize_weight(W, SYM, 0)
    b = (rng.standard_normal(N) * 0.01).astype(np.float16) if bias else None
    want = orc.linear(a, w, SYM, 0, b, 0, requant=True, requant_mode=SYM, requant_group=0)
    got = B.linear(A, Q, dev(b) if bias else None, 0, requant=True, requant_mode=SYM, requant_group=0, requant_layout=FP6)
    torch.cuda.synchronize()
    assert B.fused_fault_check() == 0
    assert np.array_equal(host(got.scale).view(np.uint32), want["s"].view(np.uint32))
    codes = fp6_to_codes(host(got.q), N, M)
    assert np.array_equal(codes, _codes(want["q"], N))
