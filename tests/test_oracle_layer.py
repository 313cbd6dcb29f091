"""Pins of the oracle's FP16 attention (Sec. 4.2: attention stays in FP16 between the quantized linears) and of
the layer composition: special cases with closed forms, an independent formulation, invariances."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle


def _qkv(seed, batch, seq, heads, d=64, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((batch * seq, 3 * heads * d)) * scale).astype(np.float16)


def test_equal_keys_give_the_mean_of_the_values():
    batch, seq, heads, d = 2, 9, 3, 64
    QKV = _qkv(1, batch, seq, heads)
    h = heads * d
    QKV[:, h:2 * h] = QKV[0, h:2 * h]                      # every key row of every sequence is the same vector
    out = oracle.attention(QKV, batch, seq, heads)
    V = QKV[:, 2 * h:].astype(np.float64).reshape(batch, seq, h)
    want = np.repeat(V.mean(axis=1), seq, axis=0)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-12)


def test_a_dominant_key_selects_its_value_row():
    batch, seq, heads, d = 1, 6, 2, 64
    QKV = np.zeros((seq, 3 * heads * d), np.float16)
    h = heads * d
    rng = np.random.default_rng(2)
    QKV[:, 2 * h:] = rng.standard_normal((seq, h)).astype(np.float16)
    QKV[:, :h] = 8.0                                       # q . k = 64 * 8 * 8 / 8 = 512 for key 4, 0 for the others
    QKV[4, h:2 * h] = 8.0
    out = oracle.attention(QKV, batch, seq, heads)
    np.testing.assert_allclose(out, np.repeat(QKV[4:5, 2 * h:].astype(np.float64), seq, axis=0), atol=1e-12)


def test_against_an_einsum_and_scipy_softmax_formulation():
    batch, seq, heads, d = 3, 17, 4, 64
    QKV = _qkv(3, batch, seq, heads)
    h = heads * d
    x = QKV.astype(np.float64).reshape(batch, seq, 3, heads, d)
    s = np.einsum("bqhd,bkhd->bhqk", x[:, :, 0], x[:, :, 1]) / 8.0
    want = np.einsum("bhqk,bkhd->bqhd", softmax(s, axis=-1), x[:, :, 2]).reshape(batch * seq, h)
    np.testing.assert_allclose(oracle.attention(QKV, batch, seq, heads), want, rtol=1e-10, atol=1e-12)


def test_key_order_does_not_matter_and_sequences_do_not_mix():
    batch, seq, heads, d = 2, 11, 2, 64
    QKV = _qkv(4, batch, seq, heads)
    h = heads * d
    base = oracle.attention(QKV, batch, seq, heads)
    perm = np.random.default_rng(5).permutation(seq)
    P = QKV.copy()
    P[:seq, h:] = QKV[:seq][perm][:, h:]                   # keys and values of sequence 0 permuted together
    np.testing.assert_allclose(oracle.attention(P, batch, seq, heads), base, rtol=1e-10, atol=1e-12)
    Z = QKV.copy()
    Z[seq:, :] = 0                                         # changing sequence 1 leaves sequence 0 alone
    np.testing.assert_array_equal(oracle.attention(Z, batch, seq, heads)[:seq], base[:seq])


def _layer_inputs(seed, M, h, f):
    rng = np.random.default_rng(seed)
    n = lambda *s, std=1.0: (rng.standard_normal(s) * std).astype(np.float16)
    return dict(X=n(M, h), Wqkv=n(3 * h, h, std=0.05), bqkv=n(3 * h, std=0.02), Wao=n(h, h, std=0.05), bao=n(h, std=0.02),
                W1=n(f, h, std=0.05), b1=n(f, std=0.02), W2=n(h, f, std=0.05), b2=n(h, std=0.02),
                g1=(1 + 0.1 * rng.standard_normal(h)).astype(np.float16), be1=n(h, std=0.1),
                g2=(1 + 0.1 * rng.standard_normal(h)).astype(np.float16), be2=n(h, std=0.1))


def _run(t, batch, seq, heads, strategy):
    return oracle.encoder_layer(t["X"], batch, seq, heads, t["Wqkv"], t["bqkv"], t["Wao"], t["bao"], t["W1"], t["b1"],
                                t["W2"], t["b2"], t["g1"], t["be1"], t["g2"], t["be2"], 1e-12, strategy)


def test_layer_in_either_precision_tracks_the_unquantized_layer():
    batch, seq, heads, h, f = 2, 12, 2, 128, 256
    t = _layer_inputs(6, batch * seq, h, f)
    # the same layer in float64 from the fp16 parameters, nothing quantized
    X = t["X"].astype(np.float64)
    lin = lambda a, W, b: a @ t[W].astype(np.float64).T + t[b].astype(np.float64)
    ln = lambda v, g, b: (v - v.mean(1, keepdims=True)) / np.sqrt(v.var(1, keepdims=True) + 1e-12) * t[g].astype(np.float64) + t[b].astype(np.float64)
    qkv = lin(X, "Wqkv", "bqkv")
    ctx = oracle.attention(qkv.astype(np.float16), batch, seq, heads)
    x1 = ln(X + lin(ctx, "Wao", "bao"), "g1", "be1")
    from scipy.special import erf
    gelu = lambda y: 0.5 * y * (1 + erf(y / np.sqrt(2)))
    want = ln(x1 + lin(gelu(lin(x1, "W1", "b1")), "W2", "b2"), "g2", "be2")
    rms = np.sqrt((want ** 2).mean())
    e8 = np.sqrt(((_run(t, batch, seq, heads, 0).astype(np.float64) - want) ** 2).mean())
    e4 = np.sqrt(((_run(t, batch, seq, heads, 15).astype(np.float64) - want) ** 2).mean())
    assert e8 < 0.03 * rms and e8 < e4 < 0.5 * rms


def test_layer_strategy_flags():
    batch, seq, heads, h, f = 1, 10, 2, 128, 256
    t = _layer_inputs(7, batch * seq, h, f)
    a = _run(t, batch, seq, heads, 15).astype(np.float64)
    for s in (15 | 32, 31, 31 | 32):
        b = _run(t, batch, seq, heads, s).astype(np.float64)
        assert np.sqrt(((a - b) ** 2).mean()) < 0.1 * np.sqrt((a ** 2).mean())    # same layer, roundings moved
    with pytest.raises(ValueError):
        _run(t, batch, seq, heads, 32 | 3)                 # LN hand-over without FFN1 in INT4
