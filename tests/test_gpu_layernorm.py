"""w4a4_layernorm_quantize against the oracle.

The oracle evaluates the LayerNorm in float64 and quantizes its fp32 rounding; the device
evaluates it in fp32.  The two y differ by a few fp32 ulp, so: the fp16 copy may differ by one
fp16 step on near-ties (> 98 % identical); scales and zero points agree to 1e-5 relative; codes
are equal except +-1 where the oracle's scaled value lies within 2e-3 of a half-integer; code
sums must equal the sums of the device's OWN codes exactly.
"""
import numpy as np
import pytest
import torch

from tests.gpu_util import act_to_canonical, dev, has_gpu, host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]

SYM, ASYM, MFMA = 0, 1, 1


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


def _inputs(rng, M, K, res=True):
    x = (rng.standard_normal((M, K)) * 2.0).astype(np.float32).astype(np.float16)
    r = rng.standard_normal((M, K)).astype(np.float32).astype(np.float16) if res else None
    g = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    b = (0.1 * rng.standard_normal(K)).astype(np.float16)
    return x, r, g, b


def _check(orc, got_q, got_s, got_z, got_y, want, mode):
    if got_y is not None:
        y, wy = got_y.astype(np.float64), want["y16"].astype(np.float64)
        ulp = np.maximum(np.abs(wy) * 2.0 ** -10, 2.0 ** -24)
        assert np.all(np.abs(y - wy) <= ulp)
        assert np.mean(got_y.view(np.uint16) == want["y16"].view(np.uint16)) > 0.98
    np.testing.assert_allclose(got_s, want["s"], rtol=1e-5)
    if mode == ASYM:
        np.testing.assert_allclose(got_z, want["z"], rtol=1e-5, atol=1e-6)
    gc = orc.unpack(got_q, mode).astype(np.int32)
    wc = orc.unpack(want["q"], mode).astype(np.int32)
    diff = gc != wc
    t = (want["y32"].astype(np.float64) - want["z"].astype(np.float64)[:, None]) / want["s"].astype(np.float64)[:, None]
    frac = np.abs(t - np.floor(t) - 0.5)
    assert np.all(np.abs(gc - wc)[diff] == 1) and np.all(frac[diff] < 2e-3)
    assert diff.mean() <= 2e-3
    return gc


@pytest.mark.parametrize("M,K", [(128, 768), (300, 1024), (33, 4096), (5, 32), (64, 1536), (1, 96)])
@pytest.mark.parametrize("res", [False, True])
def test_symmetric_canonical(B, orc, M, K, res):
    rng = np.random.default_rng(M + K + res)
    x, r, g, b = _inputs(rng, M, K, res)
    x[0, :] = x[0, 0]                                               # constant row: y = beta
    want = orc.layernorm_quantize(x, r if res else None, g, b, 1e-5, SYM)
    A, y = B.layernorm_quantize(dev(x), dev(r) if res else None, dev(g), dev(b), 1e-5, SYM)
    _check(orc, host(A.q), host(A.scale), None, host(y), want, SYM)


@pytest.mark.parametrize("M,K,group", [(130, 768, 0), (130, 768, 128), (40, 1024, 256), (7, 64, 32)])
def test_asymmetric_with_group_sums(B, orc, M, K, group):
    rng = np.random.default_rng(M + K + group)
    x, r, g, b = _inputs(rng, M, K)
    want = orc.layernorm_quantize(x, r, g, b, 1e-5, ASYM, group)
    A, y = B.layernorm_quantize(dev(x), dev(r), dev(g), dev(b), 1e-5, ASYM, group)
    gc = _check(orc, host(A.q), host(A.scale), host(A.zero), host(y), want, ASYM)
    G = K if group == 0 else group
    assert np.array_equal(host(A.gsum).astype(np.int64), gc.reshape(M, K // G, G).sum(axis=2))


def test_operand_layout_and_no_fp16_copy(B, orc):
    rng = np.random.default_rng(5)
    M, K = 200, 1024
    x, r, g, b = _inputs(rng, M, K)
    want = orc.layernorm_quantize(x, r, g, b, 1e-12, SYM)
    A, y = B.layernorm_quantize(dev(x), dev(r), dev(g), dev(b), 1e-12, SYM, layout=MFMA, want_y=False)
    assert y is None
    gc = _check(orc, act_to_canonical(host(A.q)), host(A.scale), None, None, want, SYM)
    assert np.array_equal(host(A.osum).astype(np.int64), gc[:, 1::2].sum(axis=1))
    # and the packed activations feed the GEMM: same result as quantizing the oracle's y32 with quantize_act
    W = (rng.standard_normal((256, K)) * 0.02).astype(np.float16)
    Q = B.quantize_weight(dev(W), SYM, layout=MFMA)
    Y = host(B.linear(A, Q, None, 0))
    assert np.isfinite(Y).all()


def test_bench_shape_sampled_rows(B, orc):
    """The shape bench.py times (12288 x 1024, residual, fp16 copy, operand layout): sampled rows."""
    rng = np.random.default_rng(8)
    M, K = 12288, 1024
    x, r, g, b = _inputs(rng, M, K)
    A, y = B.layernorm_quantize(dev(x), dev(r), dev(g), dev(b), 1e-12, SYM, layout=MFMA)
    rows = np.sort(np.concatenate([[0, M - 1], rng.choice(M, 62, replace=False)]))
    want = orc.layernorm_quantize(x[rows], r[rows], g, b, 1e-12, SYM)
    gc = _check(orc, act_to_canonical(host(A.q)[rows]), host(A.scale)[rows], None, host(y)[rows], want, SYM)
    assert np.array_equal(host(A.osum)[rows].astype(np.int64), gc[:, 1::2].sum(axis=1))


def test_strided_rows_and_untouched_neighbours(B, orc):
    rng = np.random.default_rng(6)
    M, K = 50, 256
    wide_x = rng.standard_normal((M, 2 * K)).astype(np.float16)
    wide_r = rng.standard_normal((M, 2 * K)).astype(np.float16)
    _, _, g, b = _inputs(rng, 1, K)
    X, R = dev(wide_x)[:, K:], dev(wide_r)[:, K:]
    ybuf = torch.full((M + 8, K), 9.0, dtype=torch.float16, device="cuda")
    A, y = B.layernorm_quantize(X, R, dev(g), dev(b), 1e-5, SYM, y=ybuf[:M])
    want = orc.layernorm_quantize(np.ascontiguousarray(wide_x[:, K:]), np.ascontiguousarray(wide_r[:, K:]), g, b, 1e-5, SYM)
    _check(orc, host(A.q), host(A.scale), None, host(y), want, SYM)
    assert bool((ybuf[M:] == 9.0).all())
