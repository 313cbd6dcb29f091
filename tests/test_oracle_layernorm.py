"""Pins for the oracle's LayerNorm + token-wise quantize (Sec. 4.2: the quantize of an
activation is fused with the LayerNorm that produces it).

The LayerNorm is pinned to closed forms, to NumPy's mean / var (a library routine, and the
one-pass E[v^2] - E[v]^2 form rather than the oracle's two passes), to its invariants and to
planted-mistake checks; the quantize half is the already pinned fp32 row quantizer, checked
here through the half-step bound on the values the LayerNorm hands it.
"""
import numpy as np
import pytest

EPS = 1e-12


def _rand(rng, M, K, scale=1.0):
    return (rng.standard_normal((M, K)) * scale).astype(np.float32).astype(np.float16)


def test_constant_row_gives_beta(orc):
    K = 64
    x = np.full((3, K), 2.5, np.float16)
    g = np.linspace(0.5, 1.5, K).astype(np.float16)
    b = np.linspace(-1, 1, K).astype(np.float16)
    out = orc.layernorm_quantize(x, None, g, b, EPS)
    assert np.array_equal(out["y32"], np.broadcast_to(b.astype(np.float32), (3, K)))
    assert np.array_equal(out["y16"], np.broadcast_to(b, (3, K)))


def test_two_level_row_closed_form(orc):
    """A row of -a and +a in equal numbers: mean 0, var a^2, so y = +-gamma / sqrt(1 + eps/a^2) + beta."""
    K, a, eps = 32, 0.75, 0.25
    x = np.tile(np.array([-a, a], np.float16), K // 2)[None, :]
    g = np.full(K, 2.0, np.float16)
    b = np.full(K, 0.5, np.float16)
    out = orc.layernorm_quantize(x, None, g, b, eps)
    want = np.tile(np.array([-1.0, 1.0]), K // 2) * 2.0 / np.sqrt(1.0 + eps / a ** 2) + 0.5
    assert np.array_equal(out["y32"][0], want.astype(np.float32))


@pytest.mark.parametrize("with_res", [False, True])
def test_against_numpy_mean_and_var(orc, with_res):
    rng = np.random.default_rng(11)
    M, K = 17, 96
    x, r = _rand(rng, M, K, 3.0), _rand(rng, M, K, 0.5)
    g = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    b = (0.1 * rng.standard_normal(K)).astype(np.float16)
    out = orc.layernorm_quantize(x, r if with_res else None, g, b, 1e-5)
    v = x.astype(np.float64) + (r.astype(np.float64) if with_res else 0.0)
    mean = np.mean(v, axis=1, keepdims=True)
    var = np.mean(v * v, axis=1, keepdims=True) - mean ** 2            # one-pass form
    want = (v - mean) / np.sqrt(var + 1e-5) * g.astype(np.float64) + b.astype(np.float64)
    np.testing.assert_allclose(out["y32"].astype(np.float64), want, rtol=3e-7, atol=1e-7)
    assert np.array_equal(np.var(v, axis=1) > 0, np.ones(M, bool))
    # fp16 copy = the fp32 value rounded once
    assert np.array_equal(out["y16"], out["y32"].astype(np.float16))


def test_invariants(orc):
    rng = np.random.default_rng(12)
    M, K = 9, 128
    x = _rand(rng, M, K)
    one, zero = np.ones(K, np.float16), np.zeros(K, np.float16)
    y = orc.layernorm_quantize(x, None, one, zero, EPS)["y32"].astype(np.float64)
    assert np.all(np.abs(y.sum(axis=1)) < 1e-4)                         # zero mean
    assert np.all(np.abs((y * y).mean(axis=1) - 1.0) < 1e-5)            # unit variance (eps negligible)
    # adding a constant that keeps every element representable does not change the result
    xi = np.round(x.astype(np.float32) * 8) / 8                         # multiples of 1/8, |x| < 8
    ya = orc.layernorm_quantize(xi.astype(np.float16), None, one, zero, EPS)["y32"]
    yb = orc.layernorm_quantize((xi + 16.0).astype(np.float16), None, one, zero, EPS)["y32"]
    np.testing.assert_allclose(ya, yb, rtol=0, atol=2e-7)
    # a power-of-two rescale of the row does not change it either (eps negligible)
    yc = orc.layernorm_quantize((xi * 4.0).astype(np.float16), None, one, zero, EPS)["y32"]
    np.testing.assert_allclose(ya, yc, rtol=0, atol=2e-7)
    # the residual is added before the statistics: x + r in one tensor gives the same rows
    r = (np.round(rng.standard_normal((M, K)) * 8) / 8).astype(np.float16)
    yd = orc.layernorm_quantize(xi.astype(np.float16), r, one, zero, EPS)["y32"]
    ye = orc.layernorm_quantize((xi + r.astype(np.float32)).astype(np.float16), None, one, zero, EPS)["y32"]
    assert np.array_equal(yd, ye)
    assert not np.array_equal(yd, ya)


def test_eps_and_affine_are_used(orc):
    """Planted mistakes: a dropped eps, gamma and beta swapped, an unbiased variance."""
    rng = np.random.default_rng(13)
    K = 16
    x = _rand(rng, 1, K, 0.01)                                          # small variance: eps matters
    g = (1.0 + 0.5 * rng.standard_normal(K)).astype(np.float16)
    b = rng.standard_normal(K).astype(np.float16)
    eps = 1e-3
    y = orc.layernorm_quantize(x, None, g, b, eps)["y32"].astype(np.float64)[0]
    v = x.astype(np.float64)[0]
    n = (v - v.mean())

    def ln(var, gg, bb, e):
        return n / np.sqrt(var + e) * gg.astype(np.float64) + bb.astype(np.float64)
    right = ln(np.mean(n * n), g, b, eps)
    assert np.max(np.abs(y - right)) < 1e-6
    for wrong in (ln(np.mean(n * n), g, b, 0.0), ln(np.mean(n * n), b, g, eps), ln(np.sum(n * n) / (K - 1), g, b, eps)):
        assert np.max(np.abs(y - wrong)) > 1e-3


@pytest.mark.parametrize("mode,group", [(0, 0), (1, 0), (1, 32)])
def test_quantized_output_obeys_the_half_step_bound(orc, mode, group):
    rng = np.random.default_rng(14)
    M, K = 12, 128
    x, r = _rand(rng, M, K), _rand(rng, M, K)
    g = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    b = (0.1 * rng.standard_normal(K)).astype(np.float16)
    out = orc.layernorm_quantize(x, r, g, b, 1e-5, mode, group)
    codes = orc.unpack(out["q"], mode).astype(np.float64)
    S, Z = out["s"].astype(np.float64)[:, None], out["z"].astype(np.float64)[:, None]
    err = np.abs(out["y32"].astype(np.float64) - (S * codes + Z))
    assert np.all(err <= S / 2 * (1 + 1e-5))
    # and it is exactly the fp32 row quantizer applied to y32
    ref = orc.quantize_rows_f32(out["y32"], mode, group)
    assert np.array_equal(ref["q"], out["q"]) and np.array_equal(ref["s"], out["s"])
    assert np.array_equal(ref["z"], out["z"]) and np.array_equal(ref["gsum"], out["gsum"])
