"""Pins for the oracle's INT8 sibling (Sec. 3.1 symmetric mapping with b = 8; the INT8 pipeline
is what the paper measures the INT4 one against, Sec. 4.1 / 4.3): closed forms, the half-step
bound, brute force against NumPy's int64 matmul, and a float64 evaluation of the layer from
the dequantized operands."""
import math

import numpy as np
import pytest
from scipy.special import erf


@pytest.mark.parametrize("e", [-12, 0, 3])
def test_closed_form_grid(orc, e):
    c = np.float32(2.0 ** e)
    v = np.arange(-127, 128, dtype=np.float32) * c
    q, S = orc.quant_sym8(v)
    assert S == c and list(q) == list(range(-127, 128))


def test_absmax_maps_to_127_and_half_step_bound(orc):
    rng = np.random.default_rng(1)
    for _ in range(100):
        v = rng.standard_normal(200).astype(np.float32) * np.float32(rng.uniform(1e-3, 30))
        q, S = orc.quant_sym8(v)
        i = int(np.argmax(np.abs(v)))
        assert abs(int(q[i])) == 127 and np.sign(q[i]) == np.sign(v[i])
        assert q.min() >= -127                                         # -128 is never produced with S = absmax/127
        assert S == np.float32(np.abs(v).max()) / np.float32(127.0)
        assert np.all(np.abs(v.astype(np.float64) - float(S) * q) <= float(S) / 2 * (1 + 1e-5))


def test_zero_vector_and_ties(orc):
    q, S = orc.quant_sym8(np.zeros(16, np.float32))
    assert S == 1.0 and not q.any()
    # absmax 127 -> inv = 1: exact half-integers round to even
    v = np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -126.5], np.float32)
    q, S = orc.quant_sym8(v)
    assert S == 1.0 and list(q) == [127, 0, 2, 2, 0, -2, -126]


def test_rows_are_independent_and_fp16_is_read_exactly(orc):
    rng = np.random.default_rng(2)
    X = rng.standard_normal((9, 64)).astype(np.float16)
    out = orc.quantize_rows8(X)
    for m in range(9):
        q, S = orc.quant_sym8(X[m].astype(np.float32))
        assert np.array_equal(out["q"][m], q) and out["s"][m] == S


def test_gemm_against_numpy_and_extremes(orc):
    rng = np.random.default_rng(3)
    A = rng.integers(-128, 128, (13, 96)).astype(np.int8)
    W = rng.integers(-128, 128, (17, 96)).astype(np.int8)
    assert np.array_equal(orc.gemm8_i32(A, W), A.astype(np.int64) @ W.astype(np.int64).T)
    K = 4096
    A = np.full((2, K), -128, np.int8)
    W = np.stack([np.full(K, -128, np.int8), np.full(K, 127, np.int8)])
    assert orc.gemm8_i32(A, W).tolist() == [[16384 * K, -16256 * K]] * 2   # 6.7e7: fits int32


@pytest.mark.parametrize("act", [0, 1])
def test_linear_against_float64_of_the_dequantized_operands(orc, act):
    rng = np.random.default_rng(4)
    M, N, K = 11, 24, 256
    X = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    b = (rng.standard_normal(N) * 0.01).astype(np.float16)
    a, w = orc.quantize_rows8(X), orc.quantize_rows8(W)
    out = orc.linear8(a, w, b, act)
    xh = a["q"].astype(np.float64) * a["s"].astype(np.float64)[:, None]
    wh = w["q"].astype(np.float64) * w["s"].astype(np.float64)[:, None]
    y = xh @ wh.T + b.astype(np.float64)[None, :]
    if act:
        y = 0.5 * y * (1 + erf(y / math.sqrt(2)))
    np.testing.assert_allclose(out["y"].astype(np.float64), y, rtol=1e-5, atol=1e-6)
    # 8-bit codes reproduce the fp16 layer to about 1 %
    ref = X.astype(np.float64) @ W.astype(np.float64).T + b.astype(np.float64)[None, :]
    if act:
        ref = 0.5 * ref * (1 + erf(ref / math.sqrt(2)))
    assert np.sqrt(np.mean((y - ref) ** 2)) < 0.02 * np.sqrt(np.mean(ref ** 2)) + 1e-3
