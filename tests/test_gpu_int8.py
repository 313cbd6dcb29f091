"""The INT8 sibling (w8a8_quantize_rows, w8a8_gemm_i32, w8a8_linear) against the oracle: codes, scales
and int32 accumulators bit for bit; fp16 outputs identical without GELU, within the fp16 bar with it."""
import numpy as np
import pytest
import torch

from tests.gpu_util import GELU_SAME, OLAY_SAME, assert_f16, dev, f16_close, has_gpu, host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


def _xw(rng, M, N, K):
    X = rng.standard_normal((M, K)).astype(np.float32).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    b = (rng.standard_normal(N) * 0.01).astype(np.float16)
    return X, W, b


@pytest.mark.parametrize("M,K", [(1, 32), (130, 768), (67, 1024), (33, 4096), (5, 16384), (300, 96)])
def test_quantize_rows(B, orc, M, K):
    rng = np.random.default_rng(M + K)
    X = rng.standard_normal((M, K)).astype(np.float32).astype(np.float16)
    X[0, :] = 0
    if M > 2:
        X[2, 3] = 60000.0
    want = orc.quantize_rows8(X)
    q, s = B.quantize_rows8(dev(X))
    assert np.array_equal(host(q), want["q"])
    assert np.array_equal(host(s).view(np.uint32), want["s"].view(np.uint32))


def test_quantize_strided_rows(B, orc):
    rng = np.random.default_rng(3)
    wide = rng.standard_normal((40, 512)).astype(np.float16)
    q, s = B.quantize_rows8(dev(wide)[:, 256:])
    want = orc.quantize_rows8(np.ascontiguousarray(wide[:, 256:]))
    assert np.array_equal(host(q), want["q"]) and np.array_equal(host(s), want["s"])


@pytest.mark.parametrize("M,N,K", [(128, 768, 768), (300, 520, 512), (1, 8, 128), (700, 1024, 1024), (193, 264, 4096),
                                   (2048, 3072, 256), (4100, 1032, 192),
                                   (12288, 4096, 1024), (12288, 1024, 4096)])
def test_gemm_and_linear(B, orc, M, N, K):
    rng = np.random.default_rng(M + N + K)
    X, W, b = _xw(rng, M, N, K)
    a, w = orc.quantize_rows8(X), orc.quantize_rows8(W)
    Aq, sa = B.quantize_rows8(dev(X))
    Wq, sw = B.quantize_rows8(dev(W))
    assert np.array_equal(host(Aq), a["q"]) and np.array_equal(host(Wq), w["q"])
    rows = np.arange(M) if M <= 300 else np.sort(rng.choice(M, 64, replace=False))
    sub = dict(q=a["q"][rows], s=a["s"][rows])
    P = host(B.gemm8_i32(Aq, sa, Wq, sw))
    assert np.array_equal(P[rows], orc.gemm8_i32(sub["q"], w["q"]))
    for act in (0, 1):
        got = host(B.linear8(Aq, sa, Wq, sw, dev(b), act))[rows]
        want = orc.linear8(sub, w, b, act)["out"]
        ok, ratio = f16_close(got, want)
        assert ok, ratio
        assert_f16(got, want, 1.0 if act == 0 else GELU_SAME, f"act {act}")
    plain = host(B.linear8(Aq, sa, Wq, sw, None, 0))[rows]
    assert np.array_equal(plain.view(np.uint16), orc.linear8(sub, w, None, 0)["out"].view(np.uint16))


def test_extreme_codes_and_untouched_neighbours(B, orc):
    """All codes +-127 / -128 at K = 4096 (the largest int32 sums), and nothing written past M rows."""
    M, N, K = 70, 40, 4096
    A = np.full((M, K), -128, np.int8)
    A[::2] = 127
    W = np.full((N, K), 127, np.int8)
    W[1::3] = -128
    sa = np.ones(M, np.float32)
    sw = np.ones(N, np.float32)
    P = host(B.gemm8_i32(dev(A), dev(sa), dev(W), dev(sw)))
    assert np.array_equal(P, orc.gemm8_i32(A, W))
    buf = torch.full((M + 16, N), 3.0, dtype=torch.float16, device="cuda")
    B.linear8(dev(A), dev(sa * 1e-6), dev(W), dev(sw), None, 0, out=buf[:M])
    assert bool((buf[M:] == 3.0).all())


@pytest.mark.parametrize("M,N,K", [(128, 768, 768), (128, 3072, 768), (128, 768, 3072), (1, 8, 128), (37, 200, 4096),
                                   (300, 96, 256), (32, 2304, 768), (130, 1024, 1024), (512, 512, 1536)])
@pytest.mark.parametrize("act", [0, 1])
def test_one_kernel_linear_equals_the_two_calls_and_the_oracle(B, orc, M, N, K, act):
    """w8a8_linear_f16act (token quantize inside the GEMM kernel): bit for bit the two-call path, whichever
    tile, wave count and weight staging the shape selects; against the oracle as w8a8_linear."""
    rng = np.random.default_rng(M + N + K + act)
    X, W, b = _xw(rng, M, N, K)
    X[0, :] = 0                                                      # an all-zero token: scale 1, codes 0
    Wq, sw = B.quantize_rows8(dev(W))
    got = B.linear8_f16act(dev(X), Wq, sw, dev(b), act)
    Aq, sa = B.quantize_rows8(dev(X))
    ref = B.linear8(Aq, sa, Wq, sw, dev(b), act)
    assert torch.equal(got, ref)
    want = orc.linear8(orc.quantize_rows8(X), orc.quantize_rows8(W), b, act)["out"]
    if act == 0:
        assert np.array_equal(host(got).view(np.uint16), want.view(np.uint16))
    else:
        ok, ratio = f16_close(host(got), want)
        assert ok, ratio


def test_one_kernel_linear_reads_strided_rows(B, orc):
    rng = np.random.default_rng(77)
    M, N, K = 70, 64, 128
    X, W, b = _xw(rng, M, N, 3 * K)
    Wq, sw = B.quantize_rows8(dev(np.ascontiguousarray(W[:, :K])))
    Xd = dev(X)
    got = B.linear8_f16act(Xd[:, K:2 * K], Wq, sw)
    want = orc.linear8(orc.quantize_rows8(np.ascontiguousarray(X[:, K:2 * K])), orc.quantize_rows8(np.ascontiguousarray(W[:, :K])))["out"]
    assert np.array_equal(host(got).view(np.uint16), want.view(np.uint16))


def test_small_problem_path_reads_a_column_slice_of_codes(B, orc):
    """w8a8_linear / w8a8_gemm_i32 on a few tiles go to the split-K kernel; the codes may sit in a wider matrix."""
    rng = np.random.default_rng(78)
    M, N, K = 100, 72, 256
    A = rng.integers(-127, 128, size=(M, 3 * K), dtype=np.int8)
    W = rng.integers(-127, 128, size=(N, K), dtype=np.int8)
    sa = (rng.random(M) * 0.01 + 0.001).astype(np.float32)
    sw = (rng.random(N) * 0.01 + 0.001).astype(np.float32)
    Ad = dev(A)
    view = Ad[:, K:2 * K]
    P = host(B.gemm8_i32(view, dev(sa), dev(W), dev(sw)))
    assert np.array_equal(P, orc.gemm8_i32(np.ascontiguousarray(A[:, K:2 * K]), W))
    got = host(B.linear8(view, dev(sa), dev(W), dev(sw)))
    want = orc.linear8(dict(q=np.ascontiguousarray(A[:, K:2 * K]), s=sa), dict(q=W, s=sw))["out"]
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
